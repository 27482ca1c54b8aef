// Weight-gradient update (Algorithm 8 of the paper, with padding) on MFMA.
//
//   dW[k,c,r,s] = sum over (n,oj,oi) of I[n,c,oj*stride-pad+r,oi*stride-pad+s] * dO[n,k,oj,oi]
//
// Mapping of the paper's ingredients (Section II-J, Algorithm 9):
//   * the VLEN x VLEN dW block kept in registers across the spatial loops becomes
//     a (32*FC) x (32*FK) MFMA accumulator tile per filter tap, all R*S taps
//     of the tile resident in one wave (M = input channels, N = output
//     channels, reduction = pixels);
//   * the spatial blocking B_P x B_Q becomes the band of TR linear output rows
//     (n*P+oj) staged in LDS per step: the dO band and the input halo band it
//     touches, the latter reused by all R*S taps;
//   * the parallelisation trade-off (one dW vs T private copies + reduction):
//     the grid is (split of the pixel range) x (channel tiles); each split
//     writes a private partial dW and a second kernel sums the copies in a
//     fixed order, so results are bitwise reproducible.  The split also keeps
//     every fp32 accumulation chain short.
#include "conv_internal.h"

namespace convmi {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// fp32 activations and gradients (vlen 4).  256 threads = 2 x 2 waves over
// (input channels, output channels); a wave owns FC x FK fragments per tap.
// Tiles are small enough for two workgroups per CU: one computes while the
// other stages its next band, so the staging is a plain load -> LDS copy.
// Staging map: thread -> (pixel p = tid % (256/G), plane group g = tid / (256/G)),
// planes g, g+G, ...; GI / GO are the group counts for the input / dO band.
template <int R, int S, int FC, int FK, int GI, int GO, bool PREFETCH>
__global__ __launch_bounds__(256, 2) void upd_f32_kernel(const UpdArgs a)
{
    constexpr int V = 4;
    constexpr int NTAPS = R * S;
    constexpr int TC = 2 * FC * 32;
    constexpr int TK = 2 * FK * 32;
    constexpr int NPI = TC / V;  // staged input planes
    constexpr int NPO = TK / V;  // staged dO planes
    constexpr int PXI = 256 / GI, PXO = 256 / GO;
    static_assert(NPI % GI == 0 && NPO % GO == 0, "plane groups");

    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    float *ldsI = reinterpret_cast<float *>(lds);
    float *ldsO = ldsI + (size_t)NPI * a.PLS_in * V;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // (uniform: kept in a scalar register)
    const int h = lane >> 5;
    const int l32 = lane & 31;
    const int wave_c = wave & 1;
    const int wave_k = wave >> 1;

    const int bid = blockIdx.x;
    const int lin = (bid & 7) * a.per_xcd + (bid >> 3);
    if (lin >= a.total) return;
    const int kt = lin % a.n_kt;
    const int rest = lin / a.n_kt;
    const int ct = rest % a.n_ct;
    const int split = rest / a.n_ct;
    const int cb0 = ct * NPI;  // first input channel block of the tile
    const int kb0 = kt * NPO;  // first output channel block of the tile

    const int NP = a.N * a.P;
    const int rho_begin = split * a.rows_per_split;
    const int rho_end = min(NP, rho_begin + a.rows_per_split);
    const int Qp = a.Qp;  // dO row pitch in the staged band
    const int npxO = a.TR * Qp;
    // A flat (unpadded 1x1) band is walked in pixel pairs: one with an odd number of
    // pixels is staged with one more, zero, pixel in both tensors.
    const int npxO_st = a.sampled ? (npxO + 1) & ~1 : npxO;
    const int lrw_st = a.sampled ? (a.LRW + 1) & ~1 : a.LRW;
    const int HW = a.H * a.W;
    const int PQ = a.P * a.Qpitch;
    const int ls = a.sampled ? 1 : a.stride;
    const float inv_LW = 1.0f / (float)a.LW, inv_Hs = 1.0f / (float)a.Hs;
    const float inv_Qp = 1.0f / (float)Qp, inv_P = 1.0f / (float)a.P;
    const u32x4 zero4 = {0u, 0u, 0u, 0u};

    // Stage the input halo band and the dO band of linear rows [rho0, rho0+TR):
    // fetch() loads into registers, commit() writes them to LDS.  With PREFETCH
    // the next band's loads are in flight while the current one is consumed.
    u32x4 vi[NPI / GI], vo[NPO / GO];
    const int gi = tid / PXI, pi = tid - gi * PXI;
    const int go = tid / PXO, po = tid - go * PXO;
    auto fetch = [&](int rho0) {
        const int n0 = fast_div(rho0, inv_P);
        const int lam0 = n0 * a.Hs + (rho0 - n0 * a.P) * a.stride;
        if (pi < lrw_st) {
            const int row = fast_div(pi, inv_LW);
            const int col = pi - row * a.LW;
            int n, ih, iw;
            bool ok;
            if (a.sampled) {
                const int rho = rho0 + row;
                n = fast_div(rho, inv_P);
                ih = (rho - n * a.P) * a.stride;
                iw = (a.q0 + col) * a.stride;
                ok = row < a.TR && rho < rho_end && col < a.Q;
            } else {
                const int lam = lam0 + row;
                n = fast_div(lam, inv_Hs);
                ih = lam - n * a.Hs - a.pad;
                iw = col + a.q0 * a.stride - a.pad_w;
                ok = n < a.N && ih >= 0 && ih < a.H && iw >= 0 && iw < a.W;
            }
            const u32x4 *ip = static_cast<const u32x4 *>(a.in) +
                              ((size_t)(n * a.Cb + cb0 + gi) * a.H + ih) * a.W + iw;
#pragma unroll
            for (int j = 0; j < NPI / GI; ++j)
                vi[j] = (ok && cb0 + gi + GI * j < a.Cb) ? __builtin_nontemporal_load(ip + (size_t)j * GI * HW) : zero4;
        }
        if (po < npxO_st) {
            const int trow = fast_div(po, inv_Qp);
            const int col = po - trow * Qp;
            const int rho = rho0 + trow;
            const int n = fast_div(rho, inv_P);
            const int oj = rho - n * a.P;
            const bool ok = trow < a.TR && rho < rho_end && col < a.Q;
            const u32x4 *op = static_cast<const u32x4 *>(a.dout) +
                              ((size_t)(n * a.Kb + kb0 + go) * a.P + oj) * a.Qpitch + a.q0 + col;
#pragma unroll
            for (int j = 0; j < NPO / GO; ++j)
                vo[j] = (ok && kb0 + go + GO * j < a.Kb) ? __builtin_nontemporal_load(op + (size_t)j * GO * PQ) : zero4;
        }
    };
    auto commit = [&]() {
        if (pi < lrw_st) {
#pragma unroll
            for (int j = 0; j < NPI / GI; ++j)
                *reinterpret_cast<u32x4 *>(ldsI + ((size_t)(gi + GI * j) * a.PLS_in + pi) * V) = vi[j];
        }
        if (po < npxO_st) {
#pragma unroll
            for (int j = 0; j < NPO / GO; ++j)
                *reinterpret_cast<u32x4 *>(ldsO + ((size_t)(go + GO * j) * a.PLS_out + po) * V) = vo[j];
        }
    };

    f32x16 acc[NTAPS][FC][FK];
#pragma unroll
    for (int t = 0; t < NTAPS; ++t)
#pragma unroll
        for (int i = 0; i < FC; ++i)
#pragma unroll
            for (int j = 0; j < FK; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[t][i][j][e] = 0.0f;

    // LDS element offsets of this lane's channel within a staged pixel
    int a_lane[FC], b_lane[FK];
#pragma unroll
    for (int i = 0; i < FC; ++i) {
        const int c = (wave_c * FC + i) * 32 + l32;
        a_lane[i] = (c / V) * a.PLS_in * V + (c % V);
    }
#pragma unroll
    for (int j = 0; j < FK; ++j) {
        const int k = (wave_k * FK + j) * 32 + l32;
        b_lane[j] = (k / V) * a.PLS_out * V + (k % V);
    }

    if (PREFETCH && rho_begin < rho_end) fetch(rho_begin);
    for (int rho0 = rho_begin; rho0 < rho_end; rho0 += a.TR) {
        __syncthreads();  // everyone is done reading the previous band
        if (!PREFETCH) fetch(rho0);
        commit();
        __syncthreads();
        if (PREFETCH && rho0 + a.TR < rho_end) fetch(rho0 + a.TR);

        const int n0 = rho0 / a.P;
        const int lam0 = n0 * a.Hs + (rho0 - n0 * a.P) * a.stride;
        const int rows = min(a.TR, rho_end - rho0);
        if (NTAPS == 1 && a.sampled) {
            // 1x1 without padding: the two staged bands hold the same pixels in
            // the same order, so the band is one flat list; the lane halves
            // take its even and odd pixels.  (An odd count ends on a staged
            // zero: the band is staged whole and is an even number of pixels.)
            // The operands of the next pair are read before this pair's MFMAs.
            const int npairs = (rows * a.Q + 1) / 2;
            const int last = 2 * (npairs - 1) + h;
            float an[FC], bn[FK];
#pragma unroll
            for (int i = 0; i < FC; ++i) an[i] = ldsI[a_lane[i] + h * V];
#pragma unroll
            for (int j = 0; j < FK; ++j) bn[j] = ldsO[b_lane[j] + h * V];
#pragma unroll 2
            for (int pr = 0; pr < npairs; ++pr) {
                const int px = 2 * pr + h;
                float av[FC], bv[FK];
#pragma unroll
                for (int i = 0; i < FC; ++i) av[i] = an[i];
#pragma unroll
                for (int j = 0; j < FK; ++j) bv[j] = bn[j];
                const int nx = min(px + 2, last);
#pragma unroll
                for (int i = 0; i < FC; ++i) an[i] = ldsI[a_lane[i] + nx * V];
#pragma unroll
                for (int j = 0; j < FK; ++j) bn[j] = ldsO[b_lane[j] + nx * V];
#pragma unroll
                for (int i = 0; i < FC; ++i)
#pragma unroll
                    for (int j = 0; j < FK; ++j)
                        acc[0][i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i], bv[j], acc[0][i][j],
                                                                            0, 0, 0);
            }
            continue;
        }
        for (int trow = 0; trow < rows; ++trow) {
            const int rho = rho0 + trow;
            const int n = rho / a.P;
            const int oj = rho - n * a.P;
            const int lrow = a.sampled ? trow : (n * a.Hs + oj * a.stride - lam0);
            const int irow = lrow * a.LW;
            const int orow = trow * Qp;
#pragma unroll 2
            for (int col = h; col < Qp; col += 2) {
                float bv[FK];
#pragma unroll
                for (int j = 0; j < FK; ++j) bv[j] = ldsO[b_lane[j] + (orow + col) * V];
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int s = 0; s < S; ++s) {
#pragma unroll
                        for (int i = 0; i < FC; ++i) {
                            const float av =
                                ldsI[a_lane[i] + (irow + r * a.LW + col * ls + s) * V];
#pragma unroll
                            for (int j = 0; j < FK; ++j)
                                acc[r * S + s][i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(
                                    av, bv[j], acc[r * S + s][i][j], 0, 0, 0);
                        }
                    }
            }
        }
    }

    // ---- write this split's partial dW tile: [split][cb][tap][k][c%V]
    const size_t copy = (size_t)a.Cb * a.ntaps_all * a.Kp * V;
    float *dst = a.partial + (size_t)(a.copy0 + split) * copy;
#pragma unroll
    for (int t = 0; t < NTAPS; ++t)
#pragma unroll
        for (int i = 0; i < FC; ++i)
#pragma unroll
            for (int j = 0; j < FK; ++j) {
                const int k = kb0 * V + (wave_k * FK + j) * 32 + l32;
                if (k >= a.Kp) continue;
#pragma unroll
                for (int vq = 0; vq < 4; ++vq) {
                    const int c = cb0 * V + (wave_c * FC + i) * 32 + vq * 8 + h * 4;
                    const int cb = c / V;
                    if (cb >= a.Cb) continue;
                    f32x4 v = {acc[t][i][j][4 * vq + 0], acc[t][i][j][4 * vq + 1],
                               acc[t][i][j][4 * vq + 2], acc[t][i][j][4 * vq + 3]};
                    *reinterpret_cast<f32x4 *>(dst + (((size_t)cb * a.ntaps_all + a.tap0 + t) * a.Kp + k) * V) = v;
                }
            }
}

// bf16 activations and gradients (vlen 8), fp32 accumulation and output.
//
// The MFMA wants 8 consecutive reduction indices (pixels) per lane, while the
// blocked layout keeps 8 channels of one pixel together -- the transpose the
// paper pays for up front on Knights Mill (Section III-B).  Here the tiles stay
// in LDS exactly as they sit in HBM ([plane][pixel][8 channels]) and the
// transposing LDS read of gfx950 (ds_read_b64_tr_b16) delivers, to the lane that
// owns channel m, four consecutive pixels of that channel: within a group of 16
// lanes, lane i slot j receives element (i % 4) of the 8 bytes addressed by lane
// 4*j + i/4.  Lane s of a group therefore addresses [pixel s/4][channels 4*(s%4)..].
// 256 threads = WC x WK waves; a wave owns FC x FK fragments per tap.
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

static __device__ __forceinline__ u32x2 lds_read_tr16(const unsigned char *p)
{
    typedef s16x4 __attribute__((address_space(3))) * lds_ptr_t;
    s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p));
    return __builtin_bit_cast(u32x2, v);
}

template <int R, int S, int WC, int WK, int FC, int FK, int PPTI, int PPTO>
__global__ __launch_bounds__(256) void upd_bf16_kernel(const UpdArgs a)
{
    constexpr int V = 8;
    constexpr int NT = 256;
    constexpr int NTAPS = R * S;
    constexpr int TC = WC * FC * 32;
    constexpr int TK = WK * FK * 32;
    constexpr int NPI = TC / V;
    constexpr int NPO = TK / V;
    static_assert(WC * WK == 4, "four waves");

    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    unsigned char *ldsI = lds;
    unsigned char *ldsO = lds + (size_t)NPI * a.PLS_in * 16;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // (uniform: kept in a scalar register)
    const int h = lane >> 5;
    const int l32 = lane & 31;
    const int grp = (lane >> 4) & 1;  // which 16 rows of the 32-row fragment
    const int i16 = lane & 15;
    const int wave_c = wave % WC;
    const int wave_k = wave / WC;

    const int bid = blockIdx.x;
    const int lin = (bid & 7) * a.per_xcd + (bid >> 3);
    if (lin >= a.total) return;
    const int kt = lin % a.n_kt;
    const int rest = lin / a.n_kt;
    const int ct = rest % a.n_ct;
    const int split = rest / a.n_ct;
    const int cb0 = ct * NPI;
    const int kb0 = kt * NPO;

    const int NP = a.N * a.P;
    const int rho_begin = split * a.rows_per_split;
    const int rho_end = min(NP, rho_begin + a.rows_per_split);
    const int npxO = ((a.TR * a.Q + 15) / 16) * 16;  // staged dO pixels, zero padded
    const int ls = a.sampled ? 1 : a.stride;
    const int gap = a.sampled ? 0 : a.Hs - a.P * a.stride;  // extra staged rows between images

    u32x4 ireg[PPTI];
    u32x4 oreg[PPTO];
    const u32x4 zero4 = {0u, 0u, 0u, 0u};

    auto fetch = [&](int rho0) {
        const int n0 = rho0 / a.P;
        const int lam0 = n0 * a.Hs + (rho0 - n0 * a.P) * a.stride;
        const u32x4 *ip = static_cast<const u32x4 *>(a.in);
        const u32x4 *op = static_cast<const u32x4 *>(a.dout);
#pragma unroll
        for (int i = 0; i < PPTI; ++i) {
            const int ci = tid + i * NT;
            u32x4 v = zero4;
            if (ci < NPI * a.LRW) {
                const int pl = ci / a.LRW;
                const int p = ci - pl * a.LRW;
                const int row = p / a.LW;
                const int col = p - row * a.LW;
                int n, ih, iw;
                bool ok;
                if (a.sampled) {
                    const int rho = rho0 + row;
                    n = rho / a.P;
                    ih = (rho - n * a.P) * a.stride;
                    iw = (a.q0 + col) * a.stride;
                    ok = rho < rho_end && col < a.Q;
                } else {
                    const int lam = lam0 + row;
                    n = lam / a.Hs;
                    ih = lam - n * a.Hs - a.pad;
                    iw = col + a.q0 * a.stride - a.pad_w;
                    ok = n < a.N && ih >= 0 && ih < a.H && iw >= 0 && iw < a.W;
                }
                ok = ok && (cb0 + pl) < a.Cb;
                if (ok) v = __builtin_nontemporal_load(ip + ((size_t)(n * a.Cb + cb0 + pl) * a.H + ih) * a.W + iw);
            }
            ireg[i] = v;
        }
#pragma unroll
        for (int i = 0; i < PPTO; ++i) {
            const int ci = tid + i * NT;
            u32x4 v = zero4;
            if (ci < NPO * npxO) {
                const int pl = ci / npxO;
                const int p = ci - pl * npxO;
                const int trow = p / a.Q;
                const int col = p - trow * a.Q;
                const int rho = rho0 + trow;
                if (trow < a.TR && rho < rho_end && (kb0 + pl) < a.Kb) {
                    const int n = rho / a.P;
                    const int oj = rho - n * a.P;
                    v = __builtin_nontemporal_load(op + ((size_t)(n * a.Kb + kb0 + pl) * a.P + oj) * a.Qpitch + a.q0 + col);
                }
            }
            oreg[i] = v;
        }
    };
    auto commit = [&]() {
#pragma unroll
        for (int i = 0; i < PPTI; ++i) {
            const int ci = tid + i * NT;
            if (ci < NPI * a.LRW) {
                const int pl = ci / a.LRW;
                const int p = ci - pl * a.LRW;
                *reinterpret_cast<u32x4 *>(ldsI + ((size_t)pl * a.PLS_in + p) * 16) = ireg[i];
            }
        }
#pragma unroll
        for (int i = 0; i < PPTO; ++i) {
            const int ci = tid + i * NT;
            if (ci < NPO * npxO) {
                const int pl = ci / npxO;
                const int p = ci - pl * npxO;
                *reinterpret_cast<u32x4 *>(ldsO + ((size_t)pl * a.PLS_out + p) * 16) = oreg[i];
            }
        }
    };

    f32x16 acc[NTAPS][FC][FK];
#pragma unroll
    for (int t = 0; t < NTAPS; ++t)
#pragma unroll
        for (int i = 0; i < FC; ++i)
#pragma unroll
            for (int j = 0; j < FK; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[t][i][j][e] = 0.0f;

    // Byte offsets, within a staged tile, of the 4-channel group this lane
    // addresses in a transposing read: channels 16*grp + 4*(i16 % 4) of a fragment.
    int a_lane[FC], b_lane[FK];
#pragma unroll
    for (int i = 0; i < FC; ++i) {
        const int c = (wave_c * FC + i) * 32 + grp * 16 + (i16 & 3) * 4;
        a_lane[i] = (c / V) * a.PLS_in * 16 + (c % V) * 2;
    }
#pragma unroll
    for (int j = 0; j < FK; ++j) {
        const int k = (wave_k * FK + j) * 32 + grp * 16 + (i16 & 3) * 4;
        b_lane[j] = (k / V) * a.PLS_out * 16 + (k % V) * 2;
    }
    // pixel (within a 16-pixel reduction step) this lane addresses, per half-read
    const int pix_lane = 8 * h + (i16 >> 2);
    // 16 = qa * Q + qb
    const int qa = 16 / a.Q, qb = 16 - qa * a.Q;

    if (rho_begin < rho_end) fetch(rho_begin);
    for (int rho0 = rho_begin; rho0 < rho_end; rho0 += a.TR) {
        __syncthreads();
        commit();
        __syncthreads();
        if (rho0 + a.TR < rho_end) fetch(rho0 + a.TR);

        const int rows = min(a.TR, rho_end - rho0);
        const int valid = rows * a.Q;
        const int n0 = rho0 / a.P;
        const int oj0 = rho0 - n0 * a.P;
        // per-lane walk over the band's pixels m = 16*ks + pix_lane + 4*t
        int col[2], oj[2], lrow[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int m = pix_lane + 4 * t;
            const int trow = m / a.Q;
            col[t] = m - trow * a.Q;
            int o = oj0 + trow, lr = a.sampled ? trow : trow * a.stride;
            while (o >= a.P) { o -= a.P; lr += gap; }
            oj[t] = o;
            lrow[t] = lr;
        }
        for (int m0 = 0; m0 < valid; m0 += 16) {
            int ipix[2], opix[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int m = m0 + pix_lane + 4 * t;
                const bool ok = m < valid;
                ipix[t] = ok ? (lrow[t] * a.LW + col[t] * ls) * 16 : 0;
                opix[t] = m * 16;  // zero padded beyond the valid pixels
                // advance by 16 pixels
                col[t] += qb;
                int adv = qa;
                if (col[t] >= a.Q) { col[t] -= a.Q; ++adv; }
                oj[t] += adv;
                lrow[t] += a.sampled ? adv : adv * a.stride;
                while (oj[t] >= a.P) { oj[t] -= a.P; lrow[t] += gap; }
            }
            u32x4 bf[FK];
#pragma unroll
            for (int j = 0; j < FK; ++j) {
                const u32x2 lo = lds_read_tr16(ldsO + b_lane[j] + opix[0]);
                const u32x2 hi = lds_read_tr16(ldsO + b_lane[j] + opix[1]);
                bf[j] = u32x4{lo[0], lo[1], hi[0], hi[1]};
            }
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int s = 0; s < S; ++s) {
                    const int toff = (r * a.LW + s) * 16;
#pragma unroll
                    for (int i = 0; i < FC; ++i) {
                        const u32x2 lo = lds_read_tr16(ldsI + a_lane[i] + ipix[0] + toff);
                        const u32x2 hi = lds_read_tr16(ldsI + a_lane[i] + ipix[1] + toff);
                        const u32x4 af = {lo[0], lo[1], hi[0], hi[1]};
#pragma unroll
                        for (int j = 0; j < FK; ++j)
                            acc[r * S + s][i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                __builtin_bit_cast(bf16x8, af), __builtin_bit_cast(bf16x8, bf[j]),
                                acc[r * S + s][i][j], 0, 0, 0);
                    }
                }
        }
    }

    const size_t copy = (size_t)a.Cb * a.ntaps_all * a.Kp * V;
    float *dst = a.partial + (size_t)(a.copy0 + split) * copy;
#pragma unroll
    for (int t = 0; t < NTAPS; ++t)
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
                    f32x4 v = {acc[t][i][j][4 * vq + 0], acc[t][i][j][4 * vq + 1],
                               acc[t][i][j][4 * vq + 2], acc[t][i][j][4 * vq + 3]};
                    *reinterpret_cast<f32x4 *>(dst + (((size_t)cb * a.ntaps_all + a.tap0 + t) * a.Kp + k) * V +
                                               4 * h) = v;
                }
            }
}

// dW[e] = sum_j partial[j][e] in a fixed order: 8 interleaved chains over j
// (chain g takes j = g, g+8, ...), each ascending, then chains 0..7 ascending.
__global__ __launch_bounds__(256) void upd_reduce_kernel(const f32x4 *__restrict__ partial,
                                                         f32x4 *__restrict__ dwt, size_t n4,
                                                         int splits)
{
    __shared__ f32x4 part[8][32];
    const int colt = threadIdx.x & 31;
    const int g = threadIdx.x >> 5;
    const size_t idx = (size_t)blockIdx.x * 32 + colt;
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    if (idx < n4) {
        for (int j = g; j < splits; j += 8) {
            const f32x4 v = partial[(size_t)j * n4 + idx];
            s[0] += v[0];
            s[1] += v[1];
            s[2] += v[2];
            s[3] += v[3];
        }
    }
    part[g][colt] = s;
    __syncthreads();
    if (g == 0 && idx < n4) {
        f32x4 t = part[0][colt];
        for (int q = 1; q < 8; ++q) {
            const f32x4 v = part[q][colt];
            t[0] += v[0];
            t[1] += v[1];
            t[2] += v[2];
            t[3] += v[3];
        }
        dwt[idx] = t;
    }
}

typedef void (*upd_fn_t)(const UpdArgs);
struct UpdEntry {
    UpdVariant v;
    upd_fn_t fn;
};

#define UPD_F32_ENTRY(R, S, FC, FK, GI, GO, PF)                                          \
    {                                                                                    \
        {CONV_F32, R, S, 2, 2, FC, FK, GI, GO}, upd_f32_kernel<R, S, FC, FK, GI, GO, PF>    \
    }
#define UPD_BF16_ENTRY(R, S, WC, WK, FC, FK, PI, PO)                                     \
    {                                                                                    \
        {CONV_BF16, R, S, WC, WK, FC, FK, PI, PO},                                       \
            upd_bf16_kernel<R, S, WC, WK, FC, FK, PI, PO>                                \
    }

static UpdEntry g_upd[] = {
    UPD_F32_ENTRY(3, 3, 1, 1, 1, 4, false),
    UPD_F32_ENTRY(1, 1, 1, 1, 4, 4, true),
    UPD_F32_ENTRY(1, 1, 1, 2, 4, 4, true),
    UPD_F32_ENTRY(1, 1, 2, 1, 4, 4, true),
    UPD_F32_ENTRY(1, 1, 2, 2, 4, 4, true),
    UPD_BF16_ENTRY(3, 3, 2, 2, 1, 2, 8, 8),
    UPD_BF16_ENTRY(1, 1, 2, 2, 2, 2, 8, 8),
    // one filter row of a 1 x S, R x 1 or R x S filter per launch
    UPD_F32_ENTRY(1, 3, 1, 1, 1, 4, false),
    UPD_F32_ENTRY(1, 5, 1, 1, 1, 4, false),
    UPD_F32_ENTRY(1, 7, 1, 1, 1, 4, false),
    UPD_BF16_ENTRY(1, 3, 2, 2, 1, 2, 8, 8),
    UPD_BF16_ENTRY(1, 5, 2, 2, 1, 2, 8, 8),
    UPD_BF16_ENTRY(1, 7, 2, 2, 1, 2, 8, 8),
    // tall one-column filters, all rows in one launch
    UPD_F32_ENTRY(3, 1, 1, 1, 1, 4, false),
    UPD_F32_ENTRY(7, 1, 1, 1, 1, 4, false),
    UPD_BF16_ENTRY(3, 1, 2, 2, 1, 2, 8, 8),
    UPD_BF16_ENTRY(7, 1, 2, 2, 1, 2, 8, 8),
};

static UpdEntry *find_upd(const UpdVariant &v)
{
    for (auto &e : g_upd)
        if (e.v.dtype == v.dtype && e.v.r == v.r && e.v.s == v.s && e.v.wc == v.wc &&
            e.v.wk == v.wk && e.v.fc == v.fc && e.v.fk == v.fk && e.v.ppt_in == v.ppt_in &&
            e.v.ppt_out == v.ppt_out)
            return &e;
    return nullptr;
}

bool upd_variant_exists(const UpdVariant &v) { return find_upd(v) != nullptr; }

hipError_t launch_upd(const UpdVariant &v, const UpdArgs &a, size_t lds_bytes, int grid,
                      hipStream_t stream)
{
    UpdEntry *e = find_upd(v);
    if (!e) return hipErrorInvalidDeviceFunction;
    if (hipError_t err = ensure_dynamic_lds(reinterpret_cast<const void *>(e->fn), lds_bytes);
        err != hipSuccess)
        return err;
    hipLaunchKernelGGL(e->fn, dim3(grid), dim3(256), lds_bytes, stream, a);
    return hipGetLastError();
}

hipError_t launch_upd_reduce(const float *partial, float *dwt, size_t n_elems, int splits,
                             hipStream_t stream)
{
    const size_t n4 = n_elems / 4;
    hipLaunchKernelGGL(upd_reduce_kernel, dim3((unsigned)((n4 + 31) / 32)), dim3(256), 0, stream,
                       reinterpret_cast<const f32x4 *>(partial), reinterpret_cast<f32x4 *>(dwt), n4,
                       splits);
    return hipGetLastError();
}

}  // namespace convmi
