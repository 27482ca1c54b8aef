// bf16 weight-gradient update (Algorithm 8 of the paper; fp32 accumulation and
// output) for 1x1 filters without padding, any stride: eight waves per
// workgroup on the flat pixel list.
//
//   dW[k,c] = sum over (n,oj,oi) of I[n,c,oj*stride,oi*stride] * dO[n,k,oj,oi]
//
// Mapping of Section II-J / Algorithm 9:
//   * the dW block kept in registers across the spatial loops is an
//     (FC*32) x (FK*32) channel block per wave, up to 64 x 128 (eight 32x32 MFMA
//     accumulator tiles): M = input channels, N = output channels;
//   * the reduction runs over pixels, 16 per MFMA.  The MFMA takes 8 consecutive
//     pixels per lane while the blocked layout keeps 8 channels of one pixel
//     together (the transpose the paper pays for up front on Knights Mill,
//     Section III-B): the bands stay in LDS as they sit in HBM
//     ([plane][pixel][8 channels]) and the transposing LDS read hands each lane
//     four consecutive pixels of its channel;
//   * spatial blocking: bands of 64 pixels of the flat pixel list (n, oj, oi) --
//     no row structure, so no pixel slot is padding, whatever the image extent --
//     staged through registers into a double-buffered LDS tile, one barrier per
//     band; the loads of the next two bands are in flight while this one is consumed;
//   * parallelisation: grid = (split of the pixel list) x (channel blocks); where
//     the channel block needs fewer than eight waves the spare waves take
//     alternate 16-pixel groups into private accumulators, summed through LDS
//     after the last band ("T copies + reduction" of Section II-J inside the
//     workgroup).  Every split writes a private partial dW that the reduce kernel
//     sums in a fixed order.
#include <type_traits>

#include "conv_internal.h"

namespace convmi {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// Transposing 64-bit LDS read: within a group of 16 lanes, lane i slot j
// receives 16-bit element (i % 4) of the 8 bytes addressed by lane 4*j + i/4.
static __device__ __forceinline__ u32x2 lds_read_tr16_b64(const unsigned char *p)
{
    typedef s16x4 __attribute__((address_space(3))) * lds_ptr_t;
    s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p));
    return __builtin_bit_cast(u32x2, v);
}

// WC x WK waves over (input, output) channels, WP pixel groups (WC*WK*WP = 8);
// FC x FK 32x32 fragments per wave.
template <int WC, int WK, int WP, int FC, int FK>
__global__ __launch_bounds__(512) void upd_bf16_1x1_kernel(const UpdArgs a)
{
    static_assert(WC * WK * WP == 8, "eight waves");
    static_assert(WP <= 4, "a band has four 16-pixel steps");
    static_assert(FC * FK * 16 <= 128, "two waves per SIMD");
    constexpr int V = 8;
    constexpr int TC = WC * FC * 32, TK = WK * FK * 32;
    constexpr int NPI = TC / V, NPO = TK / V;  // staged planes
    constexpr int BP = 64;                     // pixels per band: four 16-pixel MFMA steps
    // plane pitch in pixels: the two planes a 16-lane transposing read touches start 64
    // bytes apart in the 256-byte bank row
    constexpr int PL = BP + 4;
    constexpr int LI = NPI / 8, LO = NPO / 8;  // loads per thread and band
    static_assert(NPI % 8 == 0 && NPO % 8 == 0, "plane groups of eight");
    constexpr int IBYTES = NPI * PL * 16;
    constexpr int BUF = (NPI + NPO) * PL * 16;

    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5;
    const int l32 = lane & 31;
    const int grp = (lane >> 4) & 1;
    const int i16 = lane & 15;
    const int wave_c = wave % WC;
    const int wave_k = (wave / WC) % WK;
    const int wave_p = wave / (WC * WK);

    const int bid = blockIdx.x;
    const int lin = (bid & 7) * a.per_xcd + (bid >> 3);
    if (lin >= a.total) return;
    const int kt = lin % a.n_kt;
    const int rest = lin / a.n_kt;
    const int ct = rest % a.n_ct;
    const int split = rest / a.n_ct;
    const int cb0 = ct * NPI;
    const int kb0 = kt * NPO;

    const int HW = a.H * a.W, PQ = a.P * a.Q;
    const int npix = a.N * PQ;
    const int g_begin = split * a.rows_per_split;  // (here: pixels per split, a multiple of BP)
    const int g_end = min(npix, g_begin + a.rows_per_split);
    const int nbands = (g_end - g_begin + BP - 1) / BP;
    const float inv_PQ = 1.0f / (float)PQ, inv_Q = 1.0f / (float)a.Q;
    const rsrc_t rsrc_in = make_rsrc(a.in, 0, (size_t)a.N * a.Cb * HW * 16);
    const rsrc_t rsrc_out = make_rsrc(a.dout, 0, (size_t)a.N * a.Kb * PQ * 16);

    // Staging map: lane -> pixel `lane` of the band, planes wave + 8*j.  Two register sets:
    // a band's loads are issued two bands ahead of its use (a band is only ~1 us of MFMA
    // work, less than a trip to memory).
    u32x4 si[2][LI], so[2][LO];
    auto fetch = [&](int band, auto set_tag) {
        constexpr int SET = decltype(set_tag)::value;
        const int g = g_begin + band * BP + lane;
        unsigned off_in = kOutOfRange, off_out = kOutOfRange;
        if (g < g_end) {
            const int n = fast_div(g, inv_PQ);
            const int rem = g - mul24(n, PQ);
            int pos = rem;
            if (a.stride != 1) {
                const int oj = fast_div(rem, inv_Q);
                const int oi = rem - mul24(oj, a.Q);
                pos = mul24(mul24(oj, a.stride), a.W) + mul24(oi, a.stride);
            }
            off_in = (unsigned)(mul24(mul24(n, a.Cb), HW) + pos) * 16u;
            off_out = (unsigned)(mul24(mul24(n, a.Kb), PQ) + rem) * 16u;
        }
        // (channel blocks beyond the tensor are out of range as a whole: zeros; the check
        // is wave-uniform)
#pragma unroll
        for (int j = 0; j < LI; ++j)
            si[SET][j] = __builtin_amdgcn_raw_buffer_load_b128(
                rsrc_in, cb0 + wave + 8 * j < a.Cb ? off_in : kOutOfRange,
                (unsigned)(cb0 + wave + 8 * j) * (unsigned)HW * 16u, CONVMI_UPD_POLICY);
#pragma unroll
        for (int j = 0; j < LO; ++j)
            so[SET][j] = __builtin_amdgcn_raw_buffer_load_b128(
                rsrc_out, kb0 + wave + 8 * j < a.Kb ? off_out : kOutOfRange,
                (unsigned)(kb0 + wave + 8 * j) * (unsigned)PQ * 16u, CONVMI_UPD_POLICY);
    };
    auto commit = [&](int buf, auto set_tag) {
        constexpr int SET = decltype(set_tag)::value;
        unsigned char *bi = lds + buf * BUF;
        unsigned char *bo = bi + IBYTES;
#pragma unroll
        for (int j = 0; j < LI; ++j)
            *reinterpret_cast<u32x4 *>(bi + ((wave + 8 * j) * PL + lane) * 16) = si[SET][j];
#pragma unroll
        for (int j = 0; j < LO; ++j)
            *reinterpret_cast<u32x4 *>(bo + ((wave + 8 * j) * PL + lane) * 16) = so[SET][j];
    };

    f32x16 acc[FC][FK];
#pragma unroll
    for (int i = 0; i < FC; ++i)
#pragma unroll
        for (int j = 0; j < FK; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    // Byte offset, within a staged band, of what this lane addresses in a transposing
    // read: pixel (i16 / 4) of a 4-pixel group, channels 16*grp + 4*(i16 % 4) .. +3 of the
    // fragment; the lane half takes the second 8 pixels of a 16-pixel step.
    int a_lane[FC], b_lane[FK];
#pragma unroll
    for (int i = 0; i < FC; ++i) {
        const int c = (wave_c * FC + i) * 32 + grp * 16 + (i16 & 3) * 4;
        a_lane[i] = ((c / V) * PL + (i16 >> 2) + 8 * h) * 16 + (c % V) * 2;
    }
#pragma unroll
    for (int j = 0; j < FK; ++j) {
        const int k = (wave_k * FK + j) * 32 + grp * 16 + (i16 & 3) * 4;
        b_lane[j] = IBYTES + ((k / V) * PL + (i16 >> 2) + 8 * h) * 16 + (k % V) * 2;
    }

    // (Every band issues the same loads in the same order, beyond the end of the split with
    // out-of-range offsets that move no data: with straight-line code the compiler can wait
    // for exactly the loads a register needs and leaves the newer ones in flight.)
    using set0_t = std::integral_constant<int, 0>;
    using set1_t = std::integral_constant<int, 1>;
    fetch(0, set0_t{});
    fetch(1, set1_t{});
    commit(0, set0_t{});
    __syncthreads();
    // One band: LDS buffer band & 1 is consumed; register set band & 1, whose contents are
    // in LDS already, takes the loads of band + 2; then the loads of band + 1 are awaited
    // and written to the other LDS buffer.
    // The LDS writes of band + 1 are spread over the band's MFMA steps (the buffer they go to
    // was last read in band - 1, before the barrier that ended it): written in one go after
    // the last step they, and the barrier behind them, were half of a band's time with no
    // MFMA running (measured with timestamps: 0.95 of 1.96 us per band on the 7x7 layers).
    constexpr int NS = BP / 16 / WP;  // MFMA steps per band and wave
    auto commit_part = [&](int buf, auto set_tag, int s) {
        constexpr int SET = decltype(set_tag)::value;
        unsigned char *bi = lds + buf * BUF;
        unsigned char *bo = bi + IBYTES;
#pragma unroll
        for (int j = 0; j < LI + LO; ++j) {
            if (j * NS / (LI + LO) != s) continue;  // (this step's share)
            if (j < LI)
                *reinterpret_cast<u32x4 *>(bi + ((wave + 8 * j) * PL + lane) * 16) = si[SET][j];
            else
                *reinterpret_cast<u32x4 *>(bo + ((wave + 8 * (j - LI)) * PL + lane) * 16) = so[SET][j - LI];
        }
    };
    auto do_band = [&](int band, auto set_tag, auto other_tag) {
        fetch(band + 2, set_tag);
        const unsigned char *buf = lds + (band & 1) * BUF;
        // 16-pixel steps wave_p, wave_p + WP, ... of the band
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const int pix = (wave_p + s * WP) * 16 * 16;  // byte offset of the step's first pixel
            u32x4 af[FC], bf[FK];
#pragma unroll
            for (int i = 0; i < FC; ++i) {
                const u32x2 lo = lds_read_tr16_b64(buf + a_lane[i] + pix);
                const u32x2 hi = lds_read_tr16_b64(buf + a_lane[i] + pix + 4 * 16);
                af[i] = u32x4{lo[0], lo[1], hi[0], hi[1]};
            }
#pragma unroll
            for (int j = 0; j < FK; ++j) {
                const u32x2 lo = lds_read_tr16_b64(buf + b_lane[j] + pix);
                const u32x2 hi = lds_read_tr16_b64(buf + b_lane[j] + pix + 4 * 16);
                bf[j] = u32x4{lo[0], lo[1], hi[0], hi[1]};
            }
#pragma unroll
            for (int i = 0; i < FC; ++i)
#pragma unroll
                for (int j = 0; j < FK; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8, af[i]), __builtin_bit_cast(bf16x8, bf[j]), acc[i][j],
                        0, 0, 0);
            commit_part((band + 1) & 1, other_tag, s);  // (after the last band: zeros nobody reads)
        }
        __syncthreads();
    };
    int band = 0;
    for (; band + 1 < nbands; band += 2) {
        do_band(band, set0_t{}, set1_t{});
        do_band(band + 1, set1_t{}, set0_t{});
    }
    if (band < nbands) do_band(band, set0_t{}, set1_t{});

    // ---- the pixel groups' sums are added up through LDS, group after group in a fixed
    // order, two accumulator tiles per round (all staged bands have been consumed: the
    // last barrier is behind us)
    if constexpr (WP > 1) {
        constexpr int NTL = FC * FK;
        f32x4 *xch = reinterpret_cast<f32x4 *>(lds) + (size_t)(wave % (WC * WK)) * 2 * 4 * 64 + lane;
#pragma unroll
        for (int g = 1; g < WP; ++g) {
#pragma unroll
            for (int t0 = 0; t0 < NTL; t0 += 2) {
                if (wave_p == g) {
#pragma unroll
                    for (int tt = 0; tt < 2 && t0 + tt < NTL; ++tt)
#pragma unroll
                        for (int vq = 0; vq < 4; ++vq) {
                            const f32x16 &t = acc[(t0 + tt) / FK][(t0 + tt) % FK];
                            const f32x4 v = {t[4 * vq + 0], t[4 * vq + 1], t[4 * vq + 2], t[4 * vq + 3]};
                            xch[(tt * 4 + vq) * 64] = v;
                        }
                }
                __syncthreads();
                if (wave_p == 0) {
#pragma unroll
                    for (int tt = 0; tt < 2 && t0 + tt < NTL; ++tt)
#pragma unroll
                        for (int vq = 0; vq < 4; ++vq) {
                            f32x16 &t = acc[(t0 + tt) / FK][(t0 + tt) % FK];
                            const f32x4 v = xch[(tt * 4 + vq) * 64];
                            t[4 * vq + 0] += v[0];
                            t[4 * vq + 1] += v[1];
                            t[4 * vq + 2] += v[2];
                            t[4 * vq + 3] += v[3];
                        }
                }
                __syncthreads();
            }
        }
        if (wave_p != 0) return;
    }

    // ---- this split's partial dW tile: [split][cb][k][c%8]
    const size_t copy = (size_t)a.Cb * a.Kp * V;
    float *dst = a.partial + (size_t)split * copy;
#pragma unroll
    for (int i = 0; i < FC; ++i)
#pragma unroll
        for (int j = 0; j < FK; ++j) {
            const int k = kb0 * V + (wave_k * FK + j) * 32 + l32;
            if (k >= a.Kp) continue;
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                const int c = cb0 * V + (wave_c * FC + i) * 32 + vq * 8;
                const int cb = c / V;
                if (cb >= a.Cb) continue;
                f32x4 v = {acc[i][j][4 * vq + 0], acc[i][j][4 * vq + 1], acc[i][j][4 * vq + 2],
                           acc[i][j][4 * vq + 3]};
                *reinterpret_cast<f32x4 *>(dst + ((size_t)cb * a.Kp + k) * V + 4 * h) = v;
            }
        }
}

typedef void (*upd_flat_fn_t)(const UpdArgs);
struct UpdFlatEntry {
    UpdRowsVariant v;  // (r = s = 1)
    upd_flat_fn_t fn;
};
#define UPD_FLAT_ENTRY(WC, WK, WP, FC, FK) \
    {{1, 1, WC, WK, WP, FC, FK}, upd_bf16_1x1_kernel<WC, WK, WP, FC, FK>}
static UpdFlatEntry g_flat[] = {
    // input channels x output channels of the workgroup's dW block
    UPD_FLAT_ENTRY(4, 2, 1, 2, 4),  // 256 x 256
    UPD_FLAT_ENTRY(2, 2, 2, 2, 4),  // 128 x 256
    UPD_FLAT_ENTRY(1, 2, 4, 2, 4),  //  64 x 256
    UPD_FLAT_ENTRY(4, 1, 2, 2, 4),  // 256 x 128
    UPD_FLAT_ENTRY(2, 1, 4, 2, 4),  // 128 x 128
    UPD_FLAT_ENTRY(2, 2, 2, 1, 2),  //  64 x 128
    UPD_FLAT_ENTRY(4, 1, 2, 2, 2),  // 256 x  64
    UPD_FLAT_ENTRY(2, 1, 4, 2, 2),  // 128 x  64
    UPD_FLAT_ENTRY(2, 2, 2, 1, 1),  //  64 x  64
};

static UpdFlatEntry *find_flat(const UpdRowsVariant &v)
{
    for (auto &e : g_flat)
        if (e.v.wc == v.wc && e.v.wk == v.wk && e.v.wp == v.wp && e.v.fc == v.fc && e.v.fk == v.fk)
            return &e;
    return nullptr;
}
bool upd_bf16_1x1_variant_exists(const UpdRowsVariant &v) { return find_flat(v) != nullptr; }
size_t upd_bf16_1x1_lds_bytes(const UpdRowsVariant &v)
{
    const int planes = (v.wc * v.fc * 32 + v.wk * v.fk * 32) / 8;
    return (size_t)2 * planes * 68 * 16;
}

hipError_t launch_upd_bf16_1x1(const UpdRowsVariant &v, const UpdArgs &a, int grid, hipStream_t stream)
{
    UpdFlatEntry *e = find_flat(v);
    if (!e) return hipErrorInvalidDeviceFunction;
    const size_t lds_bytes = upd_bf16_1x1_lds_bytes(v);
    if (hipError_t err = ensure_dynamic_lds(reinterpret_cast<const void *>(e->fn), lds_bytes);
        err != hipSuccess)
        return err;
    hipLaunchKernelGGL(e->fn, dim3(grid), dim3(512), lds_bytes, stream, a);
    return hipGetLastError();
}

}  // namespace convmi
