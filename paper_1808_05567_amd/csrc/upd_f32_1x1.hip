// fp32 weight-gradient update (Algorithm 8 of the paper) for 1x1 filters without
// padding, any stride: eight waves per workgroup, a 256-channel by up to
// 256-channel block of dW per workgroup.
//
//   dW[k,c] = sum over (n,oj,oi) of I[n,c,oj*stride,oi*stride] * dO[n,k,oj,oi]
//
// Mapping of Section II-J / Algorithm 9:
//   * the dW block kept in registers across the spatial loops is a 128 x 64
//     channel block per wave (eight 32x32 MFMA accumulator tiles);
//   * the reduction runs over pixels, two per MFMA (the lane halves).  The blocked
//     layout keeps the 4 channels of a pixel together, so one 16-byte LDS read
//     gives a lane 4 channels of its pixel.  They are used as the operands of 4
//     MFMAs: MFMA t takes channel t of every lane's block, i.e. its 32 rows are
//     the channels {4*block + t}.  The rows of an accumulator tile are therefore
//     a permutation of the channels, undone by the addresses of the final store.
//     One 16-byte read (side A, 128 channels) and one 8-byte read (side B, 64
//     channels) feed 8 MFMAs.  Side A is the tensor with more channels.
//   * spatial blocking: bands of 32 pixels of the flat pixel list (n, oj, oi),
//     staged through registers into a double-buffered LDS tile, one barrier per
//     band; the loads of the next band are in flight while this one is consumed;
//   * parallelisation: the grid is (split of the pixel list) x (channel blocks);
//     where side B has fewer than 256 channels the spare waves take alternate
//     pixel pairs into private accumulators, summed through LDS after the last
//     band ("T copies + reduction" of Section II-J inside the workgroup).  Every
//     split writes a private partial dW that the reduce kernel sums in a fixed order.
#include "conv_internal.h"

namespace convmi {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// WB waves along side B (4, 2 or 1: 256, 128 or 64 channels), WP = 4 / WB pixel groups;
// A_IS_IN: side A is the input tensor (rows of an accumulator tile = input channels).
template <int WB, bool A_IS_IN>
__global__ __launch_bounds__(512) void upd_f32_1x1_kernel(const UpdArgs a)
{
    constexpr int V = 4;
    constexpr int WP = 4 / WB;
    constexpr int BP = 32;        // pixels per band
    constexpr int PL = BP + 1;    // LDS plane pitch in pixels: planes 4 banks apart
    constexpr int NPA = 64;       // staged planes of side A (256 channels)
    constexpr int NPB = 16 * WB;  // staged planes of side B
    constexpr int LA = NPA / 16, LB = NPB / 16;  // loads per thread and band
    constexpr int BUF = (NPA + NPB) * PL * 16;   // bytes of one LDS buffer

    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5;
    const int l32 = lane & 31;
    const int wave_a = wave & 1;         // 128-channel half of side A
    const int wave_b = (wave >> 1) % WB; // 64-channel part of side B
    const int wave_p = (wave >> 1) / WB; // pixel group

    const int bid = blockIdx.x;
    const int lin = (bid & 7) * a.per_xcd + (bid >> 3);
    if (lin >= a.total) return;
    // tiles over side B fastest, then side A, then the split
    const int n_at = A_IS_IN ? a.n_ct : a.n_kt, n_bt = A_IS_IN ? a.n_kt : a.n_ct;
    const int bt = lin % n_bt;
    const int rest = lin / n_bt;
    const int at = rest % n_at;
    const int split = rest / n_at;
    const int pa0 = at * NPA;  // first channel block (plane) of the tile, side A
    const int pb0 = bt * NPB;  //                                        side B

    const int HW = a.H * a.W, PQ = a.P * a.Q;
    const int npix = a.N * PQ;
    const int g_begin = split * a.rows_per_split;  // (here: pixels per split, a multiple of BP)
    const int g_end = min(npix, g_begin + a.rows_per_split);
    const int nbands = (g_end - g_begin + BP - 1) / BP;
    const float inv_PQ = 1.0f / (float)PQ, inv_Q = 1.0f / (float)a.Q;

    const int nplA = A_IS_IN ? a.Cb : a.Kb, nplB = A_IS_IN ? a.Kb : a.Cb;
    const rsrc_t rsrc_in = make_rsrc(a.in, 0, (size_t)a.N * a.Cb * HW * 16);
    const rsrc_t rsrc_out = make_rsrc(a.dout, 0, (size_t)a.N * a.Kb * PQ * 16);
    const rsrc_t rsrcA = A_IS_IN ? rsrc_in : rsrc_out, rsrcB = A_IS_IN ? rsrc_out : rsrc_in;
    const unsigned planeA = (unsigned)(A_IS_IN ? HW : PQ) * 16u;  // bytes between channel blocks
    const unsigned planeB = (unsigned)(A_IS_IN ? PQ : HW) * 16u;

    // Staging map: lane -> pixel l32 of the band, plane 2*wave + h + 16*j.
    // Byte offsets of the lane's pixel in channel block 0 of both tensors.
    auto pixel_offsets = [&](int g, unsigned &off_in, unsigned &off_out) {
        off_in = kOutOfRange;
        off_out = kOutOfRange;
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
    };
    u32x4 sa[LA], sb[LB];
    const int my_plane = 2 * wave + h;
    auto fetch = [&](int band) {
        unsigned off_in, off_out;
        pixel_offsets(g_begin + band * BP + l32, off_in, off_out);
        const unsigned offA = A_IS_IN ? off_in : off_out, offB = A_IS_IN ? off_out : off_in;
        const unsigned laneA = offA == kOutOfRange ? kOutOfRange : offA + (unsigned)h * planeA;
        const unsigned laneB = offB == kOutOfRange ? kOutOfRange : offB + (unsigned)h * planeB;
#pragma unroll
        for (int j = 0; j < LA; ++j) {
            const bool ok = pa0 + my_plane + 16 * j < nplA;
            sa[j] = __builtin_amdgcn_raw_buffer_load_b128(
                rsrcA, ok ? laneA : kOutOfRange, (unsigned)(pa0 + 2 * wave + 16 * j) * planeA, CONVMI_UPD_POLICY);
        }
#pragma unroll
        for (int j = 0; j < LB; ++j) {
            const bool ok = pb0 + my_plane + 16 * j < nplB;
            sb[j] = __builtin_amdgcn_raw_buffer_load_b128(
                rsrcB, ok ? laneB : kOutOfRange, (unsigned)(pb0 + 2 * wave + 16 * j) * planeB, CONVMI_UPD_POLICY);
        }
    };
    auto commit = [&](int buf) {
        unsigned char *ba = lds + buf * BUF;
        unsigned char *bb = ba + NPA * PL * 16;
#pragma unroll
        for (int j = 0; j < LA; ++j)
            *reinterpret_cast<u32x4 *>(ba + ((my_plane + 16 * j) * PL + l32) * 16) = sa[j];
#pragma unroll
        for (int j = 0; j < LB; ++j)
            *reinterpret_cast<u32x4 *>(bb + ((my_plane + 16 * j) * PL + l32) * 16) = sb[j];
    };

    f32x16 acc[4][2];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[t][u][e] = 0.0f;

    // This lane's operand positions in a staged band: side A block wave_a*32 + l32 (all 4
    // channels), side B block and channel pair as below.
    const int blkB = WB == 1 ? (l32 & 15) : (wave_b >> 1) * 32 + l32;
    const int subB = WB == 1 ? (l32 >> 4) : (wave_b & 1);
    const int a_lane = ((wave_a * 32 + l32) * PL + h) * 16;
    const int b_lane = NPA * PL * 16 + (blkB * PL + h) * 16 + subB * 8;

    if (nbands > 0) {
        fetch(0);
        wait_all_memory();
        commit(0);
    }
    __syncthreads();
    for (int band = 0; band < nbands; ++band) {
        const bool more = band + 1 < nbands;
        // All eight waves forming addresses and issuing loads at the top of a band leaves the
        // matrix cores idle for the 0.7 us it takes.  Half of the waves (the even ones) do it
        // there, the others halfway through their pixel pairs, while the first half has MFMAs
        // to issue (measured at N = 256: 256-channel tiles -4 to -5 %, the rest -1 to -2 %;
        // odd waves first or waves 0-3 first do the same, waves 4-7 first loses 7 %).
        const bool early = (wave & 1) == 0;
        if (more && early) fetch(band + 1);
        const unsigned char *buf = lds + (band & 1) * BUF;
        // pixel pairs wave_p, wave_p + WP, ... of the band; the operands of the next pair are
        // read before this pair's MFMAs issue
        const unsigned char *pa = buf + a_lane + wave_p * 32, *pb = buf + b_lane + wave_p * 32;
        f32x4 an = *reinterpret_cast<const f32x4 *>(pa);
        f32x2 bn = *reinterpret_cast<const f32x2 *>(pb);
#pragma unroll
        for (int i = 0; i < BP / 2 / WP; ++i) {
            if (i == BP / 4 / WP && more && !early) fetch(band + 1);
            const f32x4 av = an;
            const f32x2 bv = bn;
            if (i + 1 < BP / 2 / WP) {
                an = *reinterpret_cast<const f32x4 *>(pa + (i + 1) * WP * 32);
                bn = *reinterpret_cast<const f32x2 *>(pb + (i + 1) * WP * 32);
            }
            // side A supplies the rows, side B the columns of every tile
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int u = 0; u < 2; ++u)
                    acc[t][u] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[t], bv[u], acc[t][u], 0, 0, 0);
        }
        if (more) {
            wait_all_memory();
            commit((band + 1) & 1);
        }
        __syncthreads();
    }

    // ---- the pixel groups' sums are added up through LDS, group after group in a fixed
    // order, two accumulator tiles per round (all staged bands have been consumed: the
    // last barrier is behind us)
    if constexpr (WP > 1) {
        f32x4 *xch = reinterpret_cast<f32x4 *>(lds) + (size_t)(wave_a + 2 * wave_b) * 2 * 4 * 64 + lane;
#pragma unroll
        for (int g = 1; g < WP; ++g) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                if (wave_p == g) {
#pragma unroll
                    for (int u = 0; u < 2; ++u)
#pragma unroll
                        for (int vq = 0; vq < 4; ++vq) {
                            const f32x4 v = {acc[t][u][4 * vq + 0], acc[t][u][4 * vq + 1],
                                             acc[t][u][4 * vq + 2], acc[t][u][4 * vq + 3]};
                            xch[(u * 4 + vq) * 64] = v;
                        }
                }
                __syncthreads();
                if (wave_p == 0) {
#pragma unroll
                    for (int u = 0; u < 2; ++u)
#pragma unroll
                        for (int vq = 0; vq < 4; ++vq) {
                            const f32x4 v = xch[(u * 4 + vq) * 64];
                            acc[t][u][4 * vq + 0] += v[0];
                            acc[t][u][4 * vq + 1] += v[1];
                            acc[t][u][4 * vq + 2] += v[2];
                            acc[t][u][4 * vq + 3] += v[3];
                        }
                }
                __syncthreads();
            }
        }
        if (wave_p != 0) return;
    }

    // ---- this split's partial dW tile: [split][cb][k][c%V]
    // Tile (t,u): row i = side-A channel 4*(pa0 + wave_a*32 + i) + t, column l32 = side-B
    // channel 4*(pb0 + blkB) + 2*subB + u; register e of a lane holds row 8*(e/4) + 4*h + e%4.
    const size_t copy = (size_t)a.Cb * a.Kp * V;
    float *dst = a.partial + (size_t)split * copy;
    const int bB = pb0 + blkB;
    if (bB < nplB) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int bA = pa0 + wave_a * 32 + 8 * (e / 4) + 4 * h + (e % 4);
            if (bA >= nplA) continue;
            if (A_IS_IN) {
                // rows = input channels: the four t are the channels of block bA, for
                // output channel k = 4*bB + 2*subB + u
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int k = 4 * bB + 2 * subB + u;
                    const f32x4 v = {acc[0][u][e], acc[1][u][e], acc[2][u][e], acc[3][u][e]};
                    *reinterpret_cast<f32x4 *>(dst + ((size_t)bA * a.Kp + k) * V) = v;
                }
            } else {
                // rows = output channels k = 4*bA + t: the two u are input channels 2*subB + u
                // of block bB
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int k = 4 * bA + t;
                    const f32x2 v = {acc[t][0][e], acc[t][1][e]};
                    *reinterpret_cast<f32x2 *>(dst + ((size_t)bB * a.Kp + k) * V + 2 * subB) = v;
                }
            }
        }
    }
}

size_t upd_f32_1x1_lds_bytes(int wb) { return (size_t)2 * (64 + 16 * wb) * 33 * 16; }

hipError_t launch_upd_f32_1x1(int wb, bool a_is_in, const UpdArgs &a, int grid, hipStream_t stream)
{
    typedef void (*fn_t)(const UpdArgs);
    fn_t fn = nullptr;
    if (wb == 4) { fn = a_is_in ? upd_f32_1x1_kernel<4, true> : upd_f32_1x1_kernel<4, false>; }
    if (wb == 2) { fn = a_is_in ? upd_f32_1x1_kernel<2, true> : upd_f32_1x1_kernel<2, false>; }
    if (wb == 1) { fn = a_is_in ? upd_f32_1x1_kernel<1, true> : upd_f32_1x1_kernel<1, false>; }
    if (!fn) return hipErrorInvalidDeviceFunction;
    const size_t lds_bytes = upd_f32_1x1_lds_bytes(wb);
    if (hipError_t err = ensure_dynamic_lds(reinterpret_cast<const void *>(fn), lds_bytes);
        err != hipSuccess)
        return err;
    hipLaunchKernelGGL(fn, dim3(grid), dim3(512), lds_bytes, stream, a);
    return hipGetLastError();
}

}  // namespace convmi
