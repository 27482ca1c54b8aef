// Weight-gradient update (Algorithm 8 of the paper, with padding) for bf16 layers with
// at most 4 input channels (the first layer of an image network) on the bf16 MFMA,
// any stride; fp32 accumulation and output.
//
//   dW[k,c,r,s] = sum over (n,oj,oi) of I[n,c,oj*stride-pad_h+r,oi*stride-pad_w+s] * dO[n,k,oj,oi]
//
// As in the fp32 kernel for such layers the small GEMM of Algorithm 9 is turned round:
// one operand's 32 rows are (s, c) -- up to 8 taps of one filter row times the 4 channel
// slots -- the other's 32 columns are output channels, the reduction runs over pixels,
// and a wave keeps one accumulator tile per filter row r.
//
// The MFMA wants 8 consecutive reduction indices (output pixels) per lane, while a staged
// input pixel holds its channels together and consecutive output pixels are `stride`
// input pixels apart.  gfx950's transposing LDS read does both at once: in a group of 16
// lanes every lane supplies the address of 8 bytes (4 channels of one pixel) and receives
// one channel of four of the addressed pixels, so the lanes simply address the pixels
// stride*(q+j) + s of their tap.  The bands stay in LDS exactly as they sit in HBM; no
// transposed or strided copy of the input exists (the transpose the paper pays for up
// front on Knights Mill, Section III-B).
//
// Eight waves = 2 x 32 output channels x four pixel groups that take alternate pairs of
// 8-pixel runs into private accumulators, summed through LDS after the last band (the
// "T copies + reduction" of Section II-J inside the workgroup).  Bands are double
// buffered, staged by loads that write straight into LDS (Section II-E).
#include "conv_internal.h"

namespace convmi {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <int R, int S>
__global__ __launch_bounds__(512) void upd_c4_bf16_kernel(const UpdArgs a)
{
    constexpr int V = 8;
    constexpr int NTAPS = R * S;
    constexpr int NW = 8;
    constexpr int NPO = 8;  // staged dO planes of 8 channels: 64 output channels per workgroup
    static_assert(S <= 8, "one filter row must fit the 32 rows of a fragment");
    static_assert(R * 16 <= 128, "two waves per SIMD");

    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int ibytes = a.PLS_in * 16;
    const int bufbytes = ibytes + NPO * a.PLS_out * 16;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5;
    const int l32 = lane & 31;
    const int grp = (lane >> 4) & 1;
    const int i16 = lane & 15;
    const int wave_k = wave & 1;
    const int wave_p = wave >> 1;

    const int bid = blockIdx.x;
    const int lin = (bid & 7) * a.per_xcd + (bid >> 3);
    if (lin >= a.total) return;
    const int kt = lin % a.n_kt;
    const int split = lin / a.n_kt;
    const int kb0 = kt * NPO;

    const int NP = a.N * a.P;
    const int rho_begin = split * a.rows_per_split;
    const int rho_end = min(NP, rho_begin + a.rows_per_split);
    const int RP = a.runs * 8;           // staged dO row pitch (pixels), zero beyond Q
    const int npxO = a.TR * RP + 8;      // ... plus one all-zero run for idle lane halves
    const int HW = a.H * a.W, PQ = a.P * a.Q;
    const float inv_LW = 1.0f / (float)a.LW, inv_Hs = 1.0f / (float)a.Hs;
    const float inv_RP = 1.0f / (float)RP, inv_P = 1.0f / (float)a.P;
    const float inv_runs = 1.0f / (float)a.runs;
    const rsrc_t rsrc_in = make_rsrc(a.in, 0, (size_t)a.N * HW * 16);
    const rsrc_t rsrc_out = make_rsrc(a.dout, 0, (size_t)a.N * a.Kb * PQ * 16);

    // byte offset of staged input position p / staged dO position p (channel block 0) of
    // the band that starts at linear output row rho0; positions outside the image, the
    // split or the tensor are out of range and arrive as zeros
    auto in_off = [&](int p, int lam0) -> unsigned {
        if (p >= a.LRW) return kOutOfRange;
        const int row = fast_div(p, inv_LW);
        const int col = p - row * a.LW;
        const int lam = lam0 + row;
        const int n = fast_div(lam, inv_Hs);
        const int ih = lam - n * a.Hs - a.pad;
        const int iw = col - a.pad_w;
        const bool ok = n < a.N && ih >= 0 && ih < a.H && iw >= 0 && iw < a.W;
        return ok ? (unsigned)((n * a.H + ih) * a.W + iw) * 16u : kOutOfRange;
    };
    auto out_off = [&](int p, int rho0) -> unsigned {
        if (p >= a.TR * RP) return kOutOfRange;
        const int trow = fast_div(p, inv_RP);
        const int col = p - trow * RP;
        const int rho = rho0 + trow;
        if (rho >= rho_end || col >= a.Q) return kOutOfRange;
        const int n = fast_div(rho, inv_P);
        const int oj = rho - n * a.P;
        return (unsigned)((n * a.Kb * a.P + oj) * a.Q + col) * 16u;
    };
    auto band_lam0 = [&](int rho0) {
        const int n0 = fast_div(rho0, inv_P);
        return n0 * a.Hs + (rho0 - n0 * a.P) * a.stride;
    };
    // Stage the band of linear output rows [rho0, rho0+TR) into buffer `buf`: wave-level
    // loads of 64 consecutive positions of one plane; the units (input chunks, then
    // (dO chunk, plane) pairs) go to the waves in equal contiguous shares.
    auto fetch = [&](int rho0, int buf) {
        unsigned char *ib = lds + buf * bufbytes;
        unsigned char *ob = ib + ibytes;
        const int lam0 = band_lam0(rho0);
        const int nch_in = (a.LRW + 63) >> 6, nch_out = (npxO + 63) >> 6;
        const int total = nch_in + nch_out * NPO;
        const int share = (total + NW - 1) / NW;
        const int first = wave * share, last = min(total, first + share);
        int cur = -1;
        unsigned off = kOutOfRange;
        for (int e = first; e < last; ++e) {
            if (e < nch_in) {
                load_to_lds_16<CONVMI_UPD_POLICY>(rsrc_in, in_off(e * 64 + lane, lam0), 0u, ib + e * 64 * 16);
            } else {
                const int u = e - nch_in;
                const int ch = u >> 3, pl = u & 7;
                if (ch != cur) {
                    cur = ch;
                    off = out_off(ch * 64 + lane, rho0);
                }
                load_to_lds_16<CONVMI_UPD_POLICY>(rsrc_out, kb0 + pl < a.Kb ? off : kOutOfRange,
                               (unsigned)(kb0 + pl) * (unsigned)PQ * 16u,
                               ob + (pl * a.PLS_out + ch * 64) * 16);
            }
        }
    };

    f32x16 acc[R];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[r][e] = 0.0f;

    // What this lane addresses in a transposing read.
    // Input: row (s, c) = 16*grp + i16 of the fragment is tap s = 4*grp + i16/4, channel
    // i16 % 4; the lane that supplies slot j of tap t is lane 4*j + t, so this lane
    // addresses pixel stride*(i16/4) + 4*grp + (i16 % 4) of the window, channels 0..3.
    const int a_lane = (a.stride * (i16 >> 2) + 4 * grp + (i16 & 3)) * 16;
    // dO: pixel i16/4 of the 4-pixel group, channels 16*grp + 4*(i16 % 4) .. +3 of the
    // wave's 32 output channels.
    const int k_lane = wave_k * 32 + grp * 16 + (i16 & 3) * 4;
    const int b_lane = ((k_lane / V) * a.PLS_out + (i16 >> 2)) * 16 + (k_lane % V) * 2;
    const int a_step = a.stride * 4 * 16;  // four output pixels further along the input row
    const int row_bytes = a.LW * 16;

    if (rho_begin < rho_end) fetch(rho_begin, 0);
    wait_all_memory();
    __syncthreads();
    int buf = 0;
    for (int rho0 = rho_begin; rho0 < rho_end; rho0 += a.TR, buf ^= 1) {
        // (the even waves issue the next band's loads at the top of the band, the odd ones halfway
        // through their run pairs)
        bool pending = rho0 + a.TR < rho_end;
        if (pending && (wave & 1) == 0) {
            fetch(rho0 + a.TR, buf ^ 1);
            pending = false;
        }
        const unsigned char *ib = lds + buf * bufbytes;
        const unsigned char *ob = ib + ibytes;
        const unsigned ib_a = lds_address(ib), ob_a = lds_address(ob);
        const int lam0 = band_lam0(rho0);
        const int rows = min(a.TR, rho_end - rho0);
        const int nruns = rows * a.runs;
        // Pairs of 8-pixel runs: lane half h takes run 2*t + h, the pixel groups alternate t.
        for (int t = wave_p; 2 * t < nruns; t += 4) {
            if (pending && 4 * t >= nruns) {
                fetch(rho0 + a.TR, buf ^ 1);
                pending = false;
            }
            const int q = 2 * t + h;
            const bool live = q < nruns;
            const int trow = fast_div(q, inv_runs);
            const int ri = q - trow * a.runs;
            const int rho = rho0 + trow;
            const int n = fast_div(rho, inv_P);
            const int oj = rho - n * a.P;
            const int lrow = n * a.Hs + oj * a.stride - lam0;  // staged row of tap row 0
            const int ipix = live ? (lrow * a.LW + a.stride * 8 * ri) * 16 : 0;
            const int opix = live ? (trow * RP + ri * 8) * 16 : a.TR * RP * 16;  // else: the zero run
            // (untracked reads: the next band's loads stay in flight behind them)
            u32x2 bq[2], aq[R][2];
            {
                const unsigned p = ob_a + b_lane + opix;
                bq[0] = lds_read_tr16_b64_untracked<0>(p);
                bq[1] = lds_read_tr16_b64_untracked<4 * 16>(p);
            }
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const unsigned p = ib_a + a_lane + ipix + r * row_bytes;
                aq[r][0] = lds_read_tr16_b64_untracked<0>(p);
                aq[r][1] = lds_read_tr16_b64_untracked<0>(p + a_step);
            }
            static_for<0, R>([&](auto rr) {
                constexpr int r = decltype(rr)::value;
                lds_reads_pending<2 * (R - 1 - r)>();
                if constexpr (r == 0) {
                    lds_read_landed(bq[0]);
                    lds_read_landed(bq[1]);
                }
                lds_read_landed(aq[r][0]);
                lds_read_landed(aq[r][1]);
                const u32x4 af = {aq[r][0][0], aq[r][0][1], aq[r][1][0], aq[r][1][1]};
                const u32x4 bf = {bq[0][0], bq[0][1], bq[1][0], bq[1][1]};
                acc[r] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, af),
                                                                 __builtin_bit_cast(bf16x8, bf), acc[r],
                                                                 0, 0, 0);
            });
        }
        if (pending) fetch(rho0 + a.TR, buf ^ 1);
        wait_all_memory();
        __syncthreads();
    }

    // ---- the pixel groups' sums are added up through LDS, group after group in a fixed
    // order, two accumulator tiles per round (all staged bands have been consumed)
    f32x4 *xch = reinterpret_cast<f32x4 *>(lds) + (size_t)wave_k * 2 * 4 * 64 + lane;
#pragma unroll
    for (int g = 1; g < 4; ++g) {
#pragma unroll
        for (int r0 = 0; r0 < R; r0 += 2) {
            if (wave_p == g) {
#pragma unroll
                for (int rr = 0; rr < 2 && r0 + rr < R; ++rr)
#pragma unroll
                    for (int vq = 0; vq < 4; ++vq) {
                        const f32x4 v = {acc[r0 + rr][4 * vq + 0], acc[r0 + rr][4 * vq + 1],
                                         acc[r0 + rr][4 * vq + 2], acc[r0 + rr][4 * vq + 3]};
                        xch[(rr * 4 + vq) * 64] = v;
                    }
            }
            __syncthreads();
            if (wave_p == 0) {
#pragma unroll
                for (int rr = 0; rr < 2 && r0 + rr < R; ++rr)
#pragma unroll
                    for (int vq = 0; vq < 4; ++vq) {
                        const f32x4 v = xch[(rr * 4 + vq) * 64];
                        acc[r0 + rr][4 * vq + 0] += v[0];
                        acc[r0 + rr][4 * vq + 1] += v[1];
                        acc[r0 + rr][4 * vq + 2] += v[2];
                        acc[r0 + rr][4 * vq + 3] += v[3];
                    }
            }
            __syncthreads();
        }
    }
    if (wave_p != 0) return;

    // ---- this split's partial dW: [split][tap][k][8]; accumulator rows 8*vq + 4*h + e are
    // tap s = 2*vq + h, channels e = 0..3; the block's upper four slots stay zero
    const size_t copy = (size_t)NTAPS * a.Kp * V;
    float *dst = a.partial + (size_t)split * copy;
    const int k = kb0 * V + wave_k * 32 + l32;
    if (k >= a.Kp) return;
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
            const int s = 2 * vq + h;
            if (s < S) {
                float *d = dst + ((size_t)(r * S + s) * a.Kp + k) * V;
                const f32x4 v = {acc[r][4 * vq + 0], acc[r][4 * vq + 1], acc[r][4 * vq + 2],
                                 acc[r][4 * vq + 3]};
                *reinterpret_cast<f32x4 *>(d) = v;
                *reinterpret_cast<f32x4 *>(d + 4) = zero;
            }
        }
}

bool upd_c4_bf16_exists(int r, int s) { return (r == 7 && s == 7) || (r == 3 && s == 3); }

hipError_t launch_upd_c4_bf16(int r, int s, const UpdArgs &a, size_t lds_bytes, int grid,
                              hipStream_t stream)
{
    typedef void (*fn_t)(const UpdArgs);
    fn_t fn = nullptr;
    if (r == 7 && s == 7) fn = upd_c4_bf16_kernel<7, 7>;
    if (r == 3 && s == 3) fn = upd_c4_bf16_kernel<3, 3>;
    if (!fn) return hipErrorInvalidDeviceFunction;
    if (hipError_t err = ensure_dynamic_lds(reinterpret_cast<const void *>(fn), lds_bytes);
        err != hipSuccess)
        return err;
    hipLaunchKernelGGL(fn, dim3(grid), dim3(512), lds_bytes, stream, a);
    return hipGetLastError();
}

}  // namespace convmi
