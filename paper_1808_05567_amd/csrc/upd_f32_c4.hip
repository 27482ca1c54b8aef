// Weight-gradient update (Algorithm 8 of the paper, with padding) for layers with
// at most 4 input channels (the first layer of an image network), any stride; fp32
// tensors, or bf16 tensors widened to fp32 on their way into LDS (the products are
// then exact, accumulation and output are fp32 as for every bf16 update).
//
//   dW[k,c,r,s] = sum over (n,oj,oi) of I[n,c,oj*stride-pad+r,oi*stride-pad+s] * dO[n,k,oj,oi]
//
// With so few channels the roles of Algorithm 9's small GEMM are swapped: M = output
// channels (dO is the A operand), N = (tap, c) -- all R*S taps times the channels that
// exist, numbered through and cut into accumulator tiles of 32 columns (7x7 and three
// channels: 147 columns in 5 tiles; one tile per filter row with the padded fourth slot
// in it would be 7).  A lane's column is a fixed offset from the pair's first input
// pixel in the staged band, (r * row pitch + s) pixels and c floats on; all tiles are
// resident in the wave.
// Eight waves = 2 x 32 output channels x FOUR pixel groups that take alternate pixel
// pairs of a band into private accumulators, summed through LDS after the last band
// (the "T copies + reduction" of Section II-J inside the workgroup).  The band of the
// next step (dO rows and the input rows they touch) streams into the second LDS buffer
// while the current one is consumed (Section II-E), one barrier per band: fp32 by loads
// that write straight into LDS, bf16 through registers (where it is converted).
#include "conv_internal.h"

namespace convmi {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

// BF16IN: the tensors are bf16 in blocks of 8 channels (the input's first 4 slots are
// used); LDS holds the same fp32 bands either way.
// NTL: accumulator tiles = ceil(R * S * live channels / 32).
template <int R, int S, bool BF16IN, int NTL>
__global__ __launch_bounds__(512) void upd_c4_f32_kernel(const UpdArgs a)
{
    constexpr int V = 4;
    constexpr int NTAPS = R * S;
    constexpr int NW = 8;
    constexpr int NPO = 16;  // staged dO planes: 64 output channels per workgroup
    static_assert(NTL * 32 >= NTAPS && NTL * 32 < NTAPS * V + 32, "tiles for one to four channels");

    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int ibytes = a.PLS_in * 16;
    const int bufbytes = ibytes + NPO * a.PLS_out * 16;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5;
    const int l32 = lane & 31;
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
    const int Qp = (a.Q + 1) & ~1;  // dO row pitch in the staged band: pairs stay inside a row
    const int npxO = a.TR * Qp;
    const int HW = a.H * a.W, PQ = a.P * a.Q;
    const float inv_LW = 1.0f / (float)a.LW, inv_Hs = 1.0f / (float)a.Hs;
    const float inv_Qp = 1.0f / (float)Qp, inv_P = 1.0f / (float)a.P;
    const float inv_npx = 1.0f / (float)npxO;
    const rsrc_t rsrc_in = make_rsrc(a.in, 0, (size_t)a.N * HW * 16);
    const rsrc_t rsrc_out = make_rsrc(a.dout, 0, (size_t)a.N * a.Kb * PQ * 16);
    // (bf16: a.Kb counts blocks of 8 channels; a pixel's block is 16 bytes in both types)

    // Stage the input rows and the dO rows of linear output rows [rho0, rho0+TR) into
    // buffer `buf`: wave-level loads of 64 consecutive positions of one plane straight
    // into LDS; positions outside the image, the split or the tensor arrive as zeros.
    // byte offset of staged input position p / staged dO position p (channel block 0) of
    // the band that starts at linear output row rho0
    auto in_off = [&](int p, int lam0) -> unsigned {
        if (p >= a.LRW) return kOutOfRange;
        const int row = fast_div(p, inv_LW);
        const int col = p - mul24(row, a.LW);
        const int lam = lam0 + row;
        const int n = fast_div(lam, inv_Hs);
        const int ih = lam - mul24(n, a.Hs) - a.pad;
        const int iw = col - a.pad_w;
        const bool ok = n < a.N && ih >= 0 && ih < a.H && iw >= 0 && iw < a.W;
        return ok ? (unsigned)(mul24(mul24(n, a.H) + ih, a.W) + iw) * 16u : kOutOfRange;
    };
    auto out_off = [&](int p, int rho0) -> unsigned {
        if (p >= npxO) return kOutOfRange;
        const int trow = fast_div(p, inv_Qp);
        const int col = p - mul24(trow, Qp);
        const int rho = rho0 + trow;
        if (rho >= rho_end || col >= a.Q) return kOutOfRange;
        const int n = fast_div(rho, inv_P);
        const int oj = rho - mul24(n, a.P);
        return (unsigned)(mul24(mul24(mul24(n, a.Kb), a.P) + oj, a.Q) + col) * 16u;
    };
    auto band_lam0 = [&](int rho0) {
        const int n0 = fast_div(rho0, inv_P);
        return n0 * a.Hs + (rho0 - n0 * a.P) * a.stride;
    };
    // fp32: stage the input rows and the dO rows of linear output rows [rho0, rho0+TR) into
    // buffer `buf`: wave-level loads of 64 consecutive positions of one plane straight
    // into LDS; positions outside the image, the split or the tensor arrive as zeros.
    auto fetch = [&](int rho0, int buf) {
        unsigned char *ib = lds + buf * bufbytes;
        unsigned char *ob = ib + ibytes;
        const int lam0 = band_lam0(rho0);
        const int nch_in = (a.LRW + 63) >> 6, nch_out = (npxO + 63) >> 6;
        // units: the input chunks, then (dO chunk, plane) pairs; equal contiguous shares
        const int total = nch_in + nch_out * NPO;
        const int share = (total + NW - 1) / NW;
        const int first = wave * share, last = min(total, first + share);
        int cur = -1;
        unsigned off = kOutOfRange;
        for (int e = first; e < last; ++e) {
            if (e < nch_in) {
                load_to_lds_16(rsrc_in, in_off(e * 64 + lane, lam0), 0u, ib + e * 64 * 16);
            } else {
                const int u = e - nch_in;
                const int ch = u >> 4, pl = u & 15;
                if (ch != cur) {
                    cur = ch;
                    off = out_off(ch * 64 + lane, rho0);
                }
                load_to_lds_16(rsrc_out, kb0 + pl < a.Kb ? off : kOutOfRange,
                               (unsigned)(kb0 + pl) * (unsigned)PQ * 16u,
                               ob + (pl * a.PLS_out + ch * 64) * 16);
            }
        }
    };
    // bf16: the same band through registers.  Thread t takes input positions t, t+512, ...
    // (8 bytes each: channel slots 0-3) and (dO position, block of 8 channels) pairs
    // t, t+512, ... (16 bytes each), widens them and writes fp32 planes of 4 channels.
    constexpr int NI = 8, NO = 4;  // at most 4096 input positions, 256 dO positions x 8 blocks
    u32x2 ri[BF16IN ? NI : 1];
    u32x4 ro[BF16IN ? NO : 1];
    const int kbb0 = kt * (NPO / 2);  // first block of 8 output channels
    auto fetch_regs = [&](int rho0) {
        const int lam0 = band_lam0(rho0);
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int p = tid + 512 * i;
            ri[i] = __builtin_amdgcn_raw_buffer_load_b64(rsrc_in, in_off(p, lam0), 0u, CONVMI_UPD_POLICY);
        }
#pragma unroll
        for (int i = 0; i < NO; ++i) {
            const int u = tid + 512 * i;  // = block * npxO + position
            const int blk = fast_div(u, inv_npx), p = u - blk * npxO;
            unsigned off = out_off(p, rho0);
            // (the block rides in the per-lane offset: the lanes of a wave differ in it)
            if (blk < NPO / 2 && kbb0 + blk < a.Kb && off != kOutOfRange)
                off += (unsigned)(kbb0 + blk) * (unsigned)PQ * 16u;
            else
                off = kOutOfRange;
            ro[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_out, off, 0u, CONVMI_UPD_POLICY);
        }
    };
    auto commit_regs = [&](int buf) {
        float *bi = reinterpret_cast<float *>(lds + buf * bufbytes);
        float *bo = reinterpret_cast<float *>(lds + buf * bufbytes + ibytes);
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int p = tid + 512 * i;
            if (p < a.PLS_in - 8) {
                const f32x4 v = {__uint_as_float(ri[i][0] << 16), __uint_as_float(ri[i][0] & 0xFFFF0000u),
                                 __uint_as_float(ri[i][1] << 16), __uint_as_float(ri[i][1] & 0xFFFF0000u)};
                *reinterpret_cast<f32x4 *>(bi + (size_t)p * V) = v;
            }
        }
#pragma unroll
        for (int i = 0; i < NO; ++i) {
            const int u = tid + 512 * i;
            const int blk = fast_div(u, inv_npx), p = u - blk * npxO;
            if (blk < NPO / 2) {
                const f32x4 lo = {__uint_as_float(ro[i][0] << 16), __uint_as_float(ro[i][0] & 0xFFFF0000u),
                                  __uint_as_float(ro[i][1] << 16), __uint_as_float(ro[i][1] & 0xFFFF0000u)};
                const f32x4 hi = {__uint_as_float(ro[i][2] << 16), __uint_as_float(ro[i][2] & 0xFFFF0000u),
                                  __uint_as_float(ro[i][3] << 16), __uint_as_float(ro[i][3] & 0xFFFF0000u)};
                *reinterpret_cast<f32x4 *>(bo + ((size_t)(2 * blk) * a.PLS_out + p) * V) = lo;
                *reinterpret_cast<f32x4 *>(bo + ((size_t)(2 * blk + 1) * a.PLS_out + p) * V) = hi;
            }
        }
    };

    f32x16 acc[NTL];
#pragma unroll
    for (int t = 0; t < NTL; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.0f;

    // A operand: output channel wave_k*32 + l32 of the staged dO pixel
    const int k_lane = wave_k * 32 + l32;
    const int a_lane = (k_lane / V) * a.PLS_out * V + (k_lane % V);
    // column 32*t + l32 of the B operand = (tap, c), c < live_ch: that float of the staged band,
    // counted from the pair's first input pixel (columns past the last tap read float 0 and
    // are never stored)
    const int live = a.live_ch;
    int b_lane[NTL], b_tap[NTL];
#pragma unroll
    for (int t = 0; t < NTL; ++t) {
        const int j = 32 * t + l32;
        const int tap = j / live, c = j - tap * live;
        const int r = tap / S, sx = tap - r * S;
        b_tap[t] = tap < NTAPS ? tap : -1;
        b_lane[t] = tap < NTAPS ? (r * a.LW + sx) * V + c : 0;
    }

    if (rho_begin < rho_end) {
        if constexpr (BF16IN) {
            fetch_regs(rho_begin);
            wait_all_memory();
            commit_regs(0);
        } else {
            fetch(rho_begin, 0);
        }
    }
    wait_all_memory();
    __syncthreads();
    int buf = 0;
    for (int rho0 = rho_begin; rho0 < rho_end; rho0 += a.TR, buf ^= 1) {
        const bool more = rho0 + a.TR < rho_end;
        if (more) {
            if constexpr (BF16IN)
                fetch_regs(rho0 + a.TR);
            else
                fetch(rho0 + a.TR, buf ^ 1);
        }
        const float *ldsI = reinterpret_cast<const float *>(lds + buf * bufbytes);
        const float *ldsO = reinterpret_cast<const float *>(lds + buf * bufbytes + ibytes);
        const int n0 = fast_div(rho0, inv_P);
        const int lam0 = n0 * a.Hs + (rho0 - n0 * a.P) * a.stride;
        const int rows = min(a.TR, rho_end - rho0);
        for (int trow = 0; trow < rows; ++trow) {
            const int rho = rho0 + trow;
            const int n = fast_div(rho, inv_P);
            const int oj = rho - n * a.P;
            const int irow = (n * a.Hs + oj * a.stride - lam0) * a.LW;
            const int orow = trow * Qp;
            // The lane halves take the two pixels of a pair, the pixel groups alternate pairs.
            // The operands of a wave's next pair are read before the MFMAs of this pair issue,
            // one LDS read behind each MFMA (left to itself the compiler reads, waits, and only
            // then issues the MFMAs: the matrix core idles through every LDS latency).
            // (Qp is even: both lane halves make the same number of rounds.)
            auto read_pair = [&](int col, float &av, float (&bv)[NTL]) {
                av = ldsO[a_lane + (orow + col) * V];
#pragma unroll
                for (int t = 0; t < NTL; ++t) bv[t] = ldsI[(irow + col * a.stride) * V + b_lane[t]];
            };
            int col = 2 * wave_p + h;
            float ac = 0.0f, bc[NTL];
            if (col < Qp) read_pair(col, ac, bc);
            for (; col < Qp; col += 8) {
                float an = 0.0f, bn[NTL];
#pragma unroll
                for (int t = 0; t < NTL; ++t) bn[t] = 0.0f;
                if (col + 8 < Qp) read_pair(col + 8, an, bn);
#pragma unroll
                for (int t = 0; t < NTL; ++t)
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(ac, bc[t], acc[t], 0, 0, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // LDS read
#pragma unroll
                for (int t = 0; t < NTL; ++t) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // LDS read
                }
                __builtin_amdgcn_sched_barrier(0);
                ac = an;
#pragma unroll
                for (int t = 0; t < NTL; ++t) bc[t] = bn[t];
            }
        }
        wait_all_memory();
        if constexpr (BF16IN) {
            if (more) commit_regs(buf ^ 1);
        }
        __syncthreads();
    }

    // ---- the pixel groups' sums are added up through LDS, group after group in a fixed
    // order, two accumulator tiles per round (all staged bands have been consumed)
    f32x4 *xch = reinterpret_cast<f32x4 *>(lds) + (size_t)wave_k * 2 * 4 * 64 + lane;
#pragma unroll
    for (int g = 1; g < 4; ++g) {
#pragma unroll
        for (int r0 = 0; r0 < NTL; r0 += 2) {
            if (wave_p == g) {
#pragma unroll
                for (int rr = 0; rr < 2 && r0 + rr < NTL; ++rr)
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
                for (int rr = 0; rr < 2 && r0 + rr < NTL; ++rr)
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

    // ---- this split's partial dW: [split][tap][k][c] (one channel block of 4 slots, or of
    // 8 for bf16 tensors, whose upper four stay zero)
    constexpr int VB = BF16IN ? 8 : 4;
    const size_t copy = (size_t)NTAPS * a.Kp * VB;
    float *dst = a.partial + (size_t)split * copy;
    const int kbase = (BF16IN ? kbb0 * 8 : kb0 * V) + wave_k * 32;
#pragma unroll
    for (int t = 0; t < NTL; ++t) {
        const int tap = b_tap[t];
        const int c = 32 * t + l32 - tap * live;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int k = kbase + (e / 4) * 8 + h * 4 + (e % 4);
            if (tap >= 0 && k < a.Kp) {
                float *d = dst + ((size_t)tap * a.Kp + k) * VB;
                d[c] = acc[t][e];
                // (the lane of a tap's last channel also clears the slots behind it)
                if (c == live - 1)
                    for (int cc = live; cc < VB; ++cc) d[cc] = 0.0f;
            }
        }
    }
}

hipError_t launch_upd_c4(int dtype, int r, int s, const UpdArgs &a, size_t lds_bytes, int grid,
                         hipStream_t stream)
{
    typedef void (*fn_t)(const UpdArgs);
    fn_t fn = nullptr;
    const bool bf = dtype == CONV_BF16;
    if (a.live_ch < 1 || a.live_ch > 4) return hipErrorInvalidValue;
    const int ntl = (r * s * a.live_ch + 31) / 32;
#define C4_PICK(R_, S_, NTL_) \
    if (r == R_ && s == S_ && ntl == NTL_) \
        fn = bf ? upd_c4_f32_kernel<R_, S_, true, NTL_> : upd_c4_f32_kernel<R_, S_, false, NTL_>;
    C4_PICK(7, 7, 2) C4_PICK(7, 7, 4) C4_PICK(7, 7, 5) C4_PICK(7, 7, 7)
    C4_PICK(3, 3, 1) C4_PICK(3, 3, 2)
#undef C4_PICK
    if (!fn) return hipErrorInvalidDeviceFunction;
    if (hipError_t err = ensure_dynamic_lds(reinterpret_cast<const void *>(fn), lds_bytes);
        err != hipSuccess)
        return err;
    hipLaunchKernelGGL(fn, dim3(grid), dim3(512), lds_bytes, stream, a);
    return hipGetLastError();
}

}  // namespace convmi
