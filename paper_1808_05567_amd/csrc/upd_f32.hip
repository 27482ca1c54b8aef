// fp32 weight-gradient update (Algorithm 8 of the paper, with padding) for
// filters larger than 1x1: eight waves per workgroup, bands staged by loads
// that write straight into LDS, double buffered.
//
//   dW[k,c,r,s] = sum over (n,oj,oi) of I[n,c,oj*stride-pad+r,oi*stride-pad+s] * dO[n,k,oj,oi]
//
// Same mapping of Section II-J / Algorithm 9 as the four-wave kernel (M = 64
// input channels, N = 64 output channels, reduction = pixels, all R*S taps of
// a 32x32 block resident in one wave), with these differences:
//   * 2 x 2 waves over (input, output) channels times TWO pixel groups: the
//     groups take alternate pixel pairs of a band into private accumulators, which
//     are summed through LDS after the last band (the "T copies + reduction"
//     of Section II-J inside the workgroup).  A CU therefore always runs two
//     waves per SIMD, which is what keeps the matrix core busy while a wave
//     issues its LDS reads.
//   * One workgroup owns the whole LDS: the band of the next step streams in
//     (Section II-E) while the current one is consumed, one barrier per band.
#include "conv_internal.h"

namespace convmi {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// ODDQ: rows of an odd number of pixels
// WCC x WCK: waves along input / output channels (32 each); the other 8 / (WCC*WCK) wave
// groups share the pixels.  2 x 2 (a 64 x 64 block of dW, two pixel groups) is the
// workhorse; 1 x 2 and 1 x 1 serve layers with at most 32 channels on a side, where three
// quarters of a 64 x 64 block would be padding (odd rows only).
template <int R, int S, bool ODDQ, int WCC = 2, int WCK = 2>  // unit stride
__global__ __launch_bounds__(512) void upd_f32_bands_kernel(const UpdArgs a)
{
    constexpr int V = 4;
    constexpr int NT = 512, NW = NT / 64;
    constexpr int NTAPS = R * S;
    constexpr int G = NW / (WCC * WCK);         // pixel groups
    constexpr int NPI = WCC * 8, NPO = WCK * 8;  // staged planes of 4 input / output channels
    static_assert(G == 2 || ODDQ, "more than two pixel groups: the odd-row path only");

    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int ibytes = NPI * a.PLS_in * 16;
    const int bufbytes = ibytes + NPO * a.PLS_out * 16;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // (uniform: kept in a scalar register)
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);  // the same, known to be uniform
    const int h = lane >> 5;
    const int l32 = lane & 31;
    const int wave_c = wave % WCC;
    const int wave_k = (wave / WCC) % WCK;
    const int wave_p = wave / (WCC * WCK);

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
    const int Qp = a.Q;          // the staged dO band is the plain pixel list ...
    const int npxO = a.TR * Qp + 1;  // ... followed by one zero
    const int HW = a.H * a.W, PQ = a.P * a.Qpitch;
    const float inv_LW = 1.0f / (float)a.LW, inv_Hs = 1.0f / (float)a.Hs;
    const float inv_Qp = 1.0f / (float)Qp, inv_P = 1.0f / (float)a.P, inv_Q = inv_Qp;
    const rsrc_t rsrc_in = make_rsrc(a.in, 0, (size_t)a.N * a.Cb * HW * 16);
    const rsrc_t rsrc_out = make_rsrc(a.dout, 0, (size_t)a.N * a.Kb * PQ * 16);

    // Stage the input halo band and the dO band of linear rows [rho0, rho0+TR)
    // into buffer `buf`.  A wave-level load fills 64 consecutive positions of one
    // plane; positions outside the image, the split or the tensor arrive as zeros.
    auto fetch = [&](int rho0, int buf) {
        unsigned char *ib = lds + buf * bufbytes;
        unsigned char *ob = ib + ibytes;
        const int n0 = fast_div(rho0, inv_P);
        const int lam0 = n0 * a.Hs + (rho0 - n0 * a.P) * a.stride;
        const int cov_in = (a.LRW + 63) & ~63, cov_out = (npxO + 63) & ~63;
        auto in_off = [&](int p) -> unsigned {
            if (p >= a.LRW) return kOutOfRange;
            const int row = fast_div(p, inv_LW);
            const int col = p - row * a.LW;
            const int lam = lam0 + row;
            const int n = fast_div(lam, inv_Hs);
            const int ih = lam - n * a.Hs - a.pad;
            const int iw = col + a.q0 * a.stride - a.pad_w;
            const bool ok = n < a.N && ih >= 0 && ih < a.H && iw >= 0 && iw < a.W;
            return ok ? (unsigned)((n * a.Cb * a.H + ih) * a.W + iw) * 16u : kOutOfRange;
        };
        auto out_off = [&](int p) -> unsigned {
            if (p >= npxO - 1) return kOutOfRange;
            const int trow = fast_div(p, inv_Qp);
            const int col = p - trow * Qp;
            const int rho = rho0 + trow;
            if (rho >= rho_end || col >= a.Q) return kOutOfRange;
            const int n = fast_div(rho, inv_P);
            const int oj = rho - n * a.P;
            return (unsigned)((n * a.Kb * a.P + oj) * a.Qpitch + a.q0 + col) * 16u;
        };
        // The (64-position chunk, plane) loads, input band first, are shared out
        // in equal contiguous runs: a wave computes the source offsets of one
        // chunk (rarely two) and issues its planes.
        const int nch_in = cov_in >> 6, nch_out = cov_out >> 6;
        const int n_in = nch_in * NPI;
        const int total = n_in + nch_out * NPO;
        const int share = (total + NW - 1) / NW;
        const int first = wave_u * share, last = min(total, first + share);
        int cur = -1;
        unsigned off = kOutOfRange;
        for (int e = first; e < last; ++e) {
            const bool is_in = e < n_in;
            const int u = is_in ? e : e - n_in;
            const int ch = is_in ? u / NPI : u / NPO, pl = is_in ? u % NPI : u % NPO;
            const int key = is_in ? ch : nch_in + ch;
            if (key != cur) {
                cur = key;
                off = is_in ? in_off(ch * 64 + lane) : out_off(ch * 64 + lane);
            }
            // (default cache policy for the input: consecutive bands share R-1 staged rows, which
            // the second band then finds in the L2 -- 1-2 % on the 3x3 layers; dO streams past once)
            if (is_in)
                load_to_lds_16<0>(rsrc_in, cb0 + pl < a.Cb ? off : kOutOfRange,
                               (unsigned)(cb0 + pl) * (unsigned)HW * 16u,
                               ib + (pl * a.PLS_in + ch * 64) * 16);
            else
                load_to_lds_16<CONVMI_UPD_POLICY>(rsrc_out, kb0 + pl < a.Kb ? off : kOutOfRange,
                               (unsigned)(kb0 + pl) * (unsigned)PQ * 16u,
                               ob + (pl * a.PLS_out + ch * 64) * 16);
        }
    };

    f32x16 acc[NTAPS];
#pragma unroll
    for (int t = 0; t < NTAPS; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.0f;

    // LDS float offsets of this lane's channel within a staged pixel
    const int c_lane = wave_c * 32 + l32, k_lane = wave_k * 32 + l32;
    const int a_lane = (c_lane / V) * a.PLS_in * V + (c_lane % V);
    const int b_lane = (k_lane / V) * a.PLS_out * V + (k_lane % V);

    if (rho_begin < rho_end) fetch(rho_begin, 0);
    wait_all_memory();
    __syncthreads();
    int buf = 0;
    for (int rho0 = rho_begin; rho0 < rho_end; rho0 += a.TR, buf ^= 1) {
        // The two pixel groups of a channel pair are the two waves of one SIMD.  With even
        // rows group 0 issues its share of the next band's loads before its pixels, group 1
        // between the two halves of its pixels: while one wave computes addresses and
        // issues loads the other has MFMAs to issue (2-3 % at 56 and 28 pixels per row; the
        // odd-row path lost 5 % to a split loop and issues all loads up front).
        const bool more = rho0 + a.TR < rho_end;
        if (more && (ODDQ || wave_p == 0)) fetch(rho0 + a.TR, buf ^ 1);
        const float *ldsI = reinterpret_cast<const float *>(lds + buf * bufbytes);
        const float *ldsO = reinterpret_cast<const float *>(lds + buf * bufbytes + ibytes);

        const int n0 = fast_div(rho0, inv_P);
        const int lam0 = n0 * a.Hs + (rho0 - n0 * a.P) * a.stride;
        const int rows = min(a.TR, rho_end - rho0);
        // The band's pixels form one list (row-major); a wave's lane halves take
        // the two pixels of a pair and the pixel groups take alternate pairs.
        if constexpr (ODDQ) {
            // Odd rows: pairs straddle rows, so each lane finds its pixel's row
            // and column itself.  A pixel past the end reads the staged zero
            // that follows the dO band.
            const int npx = rows * a.Q;
            const int npairs = (npx + 1) >> 1;
#pragma unroll 2
            for (int pr = wave_p; pr < npairs; pr += G) {
                const int p = 2 * pr + h;
                const int pin = p < npx ? p : 0;
                const int trow = fast_div(pin, inv_Q);
                const int col = pin - trow * a.Q;
                const int rho = rho0 + trow;
                const int n = fast_div(rho, inv_P);
                const int oj = rho - n * a.P;
                const int ipos = (n * a.Hs + oj * a.stride - lam0) * a.LW + col * a.stride;
                const float bv = ldsO[b_lane + p * V];
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int s = 0; s < S; ++s) {
                        const float av = ldsI[a_lane + (ipos + r * a.LW + s) * V];
                        acc[r * S + s] =
                            __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[r * S + s], 0, 0, 0);
                    }
            }
        } else {
            // Even rows: pairs stay inside a row.  Each group walks a contiguous
            // run of pairs (half a row if the row has an even number of pairs,
            // else alternate rows), so with unit stride the input values of the
            // last filter columns are the next pair's first ones and are kept in
            // registers; the other operands of the next pair are read before this
            // pair's MFMAs issue.
            const bool halves = ((a.Q >> 1) & 1) == 0;
            const int row_first = halves ? 0 : wave_p, row_step = halves ? 1 : 2;
            const int ncol = halves ? (a.Q >> 1) : a.Q;  // pixels of a row this group takes
            const int col_first = halves ? wave_p * ncol : 0;
            const int nrow = rows > row_first ? (rows - row_first + row_step - 1) / row_step : 0;
            // rows [r0, r1) of this group's rows, columns [c0, c1) of its run (c0, c1 even)
            auto walk = [&](int r0, int r1, int c0, int c1) {
                if (c1 <= c0) return;
                for (int ri = r0; ri < r1; ++ri) {
                    const int trow = row_first + ri * row_step;
                    const int rho = rho0 + trow;
                    const int n = fast_div(rho, inv_P);
                    const int oj = rho - n * a.P;
                    const float *pi = ldsI + a_lane + ((n * a.Hs + oj - lam0) * a.LW + col_first + h) * V;
                    const float *po = ldsO + b_lane + (trow * a.Q + col_first + h) * V;
                    // (the window of the next pair starts two columns further: its first S-2
                    // values are this pair's last S-2, only the other two are read)
                    constexpr int KEEP = S > 2 ? S - 2 : 0;
                    float an[R][S], bn;
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int s = 0; s < S; ++s) an[r][s] = pi[(r * a.LW + c0 + s) * V];
                    bn = po[c0 * V];
#pragma unroll 2
                    for (int c = c0; c < c1; c += 2) {
                        float av[R][S];
                        const float bv = bn;
#pragma unroll
                        for (int r = 0; r < R; ++r)
#pragma unroll
                            for (int s = 0; s < S; ++s) av[r][s] = an[r][s];
                        // next pair (clamped at the end of the run: a harmless re-read, the
                        // values are not used)
                        const int cn = min(c + 2, c1 - 2);
#pragma unroll
                        for (int r = 0; r < R; ++r) {
#pragma unroll
                            for (int s = 0; s < KEEP; ++s) an[r][s] = av[r][s + 2];
#pragma unroll
                            for (int s = KEEP; s < S; ++s) an[r][s] = pi[(r * a.LW + cn + s) * V];
                        }
                        bn = po[cn * V];
#pragma unroll
                        for (int r = 0; r < R; ++r)
#pragma unroll
                            for (int s = 0; s < S; ++s)
                                acc[r * S + s] = __builtin_amdgcn_mfma_f32_32x32x2f32(
                                    av[r][s], bv, acc[r * S + s], 0, 0, 0);
                        // issue order: each of the next pair's reads behind an MFMA of this pair
#pragma unroll
                        for (int k = 0; k < R * S; ++k) {
                            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
                            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // LDS read
                            __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);  // VALU
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            };
            // the halves of this group's pixels: rows where it has several, else columns
            // (one copy of the loop: the two halves are two trips of an outer loop)
            const bool by_rows = nrow >= 2;
            const int rm = by_rows ? nrow >> 1 : nrow, cm = by_rows ? ncol : (ncol >> 1) & ~1;
#pragma nounroll
            for (int part = 0; part < 2; ++part) {
                if (part == 1 && more && wave_p == 1) fetch(rho0 + a.TR, buf ^ 1);
                const int r0 = part == 0 ? 0 : (by_rows ? rm : 0), r1 = part == 0 ? rm : nrow;
                const int c0 = part == 0 ? 0 : (by_rows ? 0 : cm), c1 = part == 0 ? cm : ncol;
                walk(r0, r1, c0, c1);
            }
        }
        wait_all_memory();
        __syncthreads();
    }

    // ---- the other pixel groups hand their sums to the first through LDS
    // (all staged bands have been consumed: the last barrier is behind us)
    f32x4 *xch = reinterpret_cast<f32x4 *>(lds) + (size_t)(wave % (WCC * WCK)) * NTAPS * 4 * 64 + lane;
    if constexpr (G > 2) {
        // group after group in a fixed order; the first group adds each in turn
#pragma unroll 1
        for (int g = 1; g < G; ++g) {
            if (wave_p == g) {
#pragma unroll
                for (int t = 0; t < NTAPS; ++t)
#pragma unroll
                    for (int vq = 0; vq < 4; ++vq) {
                        const f32x4 v = {acc[t][4 * vq + 0], acc[t][4 * vq + 1], acc[t][4 * vq + 2],
                                         acc[t][4 * vq + 3]};
                        xch[(t * 4 + vq) * 64] = v;
                    }
            }
            __syncthreads();
            if (wave_p == 0 && g < G - 1) {
#pragma unroll
                for (int t = 0; t < NTAPS; ++t)
#pragma unroll
                    for (int vq = 0; vq < 4; ++vq) {
                        const f32x4 v = xch[(t * 4 + vq) * 64];
                        acc[t][4 * vq + 0] += v[0];
                        acc[t][4 * vq + 1] += v[1];
                        acc[t][4 * vq + 2] += v[2];
                        acc[t][4 * vq + 3] += v[3];
                    }
            }
            if (g < G - 1) __syncthreads();
        }
        // (the last group's sums are still in the exchange buffer: added at the store below)
        if (wave_p != 0) return;
    } else if (wave_p == 1) {
#pragma unroll
        for (int t = 0; t < NTAPS; ++t)
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                const f32x4 v = {acc[t][4 * vq + 0], acc[t][4 * vq + 1], acc[t][4 * vq + 2],
                                 acc[t][4 * vq + 3]};
                xch[(t * 4 + vq) * 64] = v;
            }
    }
    if constexpr (G == 2) {
        __syncthreads();
        if (wave_p == 1) return;
    }

    // ---- write this split's partial dW tile: [split][cb][tap][k][c%V]
    const size_t copy = (size_t)a.Cb * NTAPS * a.Kp * V;
    float *dst = a.partial + (size_t)(a.copy0 + split) * copy;
    const int k = kb0 * V + k_lane;
#pragma unroll
    for (int t = 0; t < NTAPS; ++t)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
            const f32x4 o = xch[(t * 4 + vq) * 64];
            const int c = cb0 * V + wave_c * 32 + vq * 8 + h * 4;
            const int cb = c / V;
            if (k >= a.Kp || cb >= a.Cb) continue;
            const f32x4 v = {acc[t][4 * vq + 0] + o[0], acc[t][4 * vq + 1] + o[1],
                             acc[t][4 * vq + 2] + o[2], acc[t][4 * vq + 3] + o[3]};
            *reinterpret_cast<f32x4 *>(dst + (((size_t)cb * NTAPS + t) * a.Kp + k) * V) = v;
        }
}

bool upd_f32_bands_exists(int r, int s)
{
    // (not 7x1: its bands hold a single output row and the four-wave kernel measured faster)
    return (r == 3 && s == 3) || (r == 1 && (s == 3 || s == 7)) || (s == 1 && r == 3);
}

// Wave layouts: 0 = 2 x 2 channel waves (64 x 64 block of dW) x 2 pixel groups,
// 1 = 1 x 2 (32 x 64) x 4, 2 = 1 x 1 (32 x 32) x 8; layouts 1 and 2: 3x3, odd rows.
bool upd_f32_bands_layout_exists(int r, int s, int layout, bool odd_rows)
{
    if (layout == 0) return upd_f32_bands_exists(r, s);
    return (layout == 1 || layout == 2) && r == 3 && s == 3 && odd_rows;
}

// LDS bytes the in-workgroup exchange of the pixel groups needs: one buffer of all the
// taps' accumulators per channel-wave pair
size_t upd_f32_bands_exchange_bytes(int r, int s, int layout)
{
    const int pairs = layout == 0 ? 4 : layout == 1 ? 2 : 1;
    return (size_t)pairs * r * s * 4 * 64 * 16;
}

hipError_t launch_upd_f32_bands(int r, int s, int layout, const UpdArgs &a, size_t lds_bytes, int grid,
                                hipStream_t stream)
{
    typedef void (*fn_t)(const UpdArgs);
    fn_t fn = nullptr;
    const int odd = a.Q & 1;
    if (layout != 0) {
        if (!upd_f32_bands_layout_exists(r, s, layout, odd != 0)) return hipErrorInvalidDeviceFunction;
        fn = layout == 1 ? upd_f32_bands_kernel<3, 3, true, 1, 2> : upd_f32_bands_kernel<3, 3, true, 1, 1>;
        if (hipError_t err = ensure_dynamic_lds(reinterpret_cast<const void *>(fn), lds_bytes);
            err != hipSuccess)
            return err;
        hipLaunchKernelGGL(fn, dim3(grid), dim3(512), lds_bytes, stream, a);
        return hipGetLastError();
    }
#define BANDS_CASE(RR, SS) \
    if (r == RR && s == SS) fn = odd ? upd_f32_bands_kernel<RR, SS, true> : upd_f32_bands_kernel<RR, SS, false>;
    BANDS_CASE(3, 3)
    BANDS_CASE(1, 7)
    BANDS_CASE(1, 3)
    BANDS_CASE(3, 1)
#undef BANDS_CASE
    if (!fn) return hipErrorInvalidDeviceFunction;
    if (hipError_t err = ensure_dynamic_lds(reinterpret_cast<const void *>(fn), lds_bytes);
        err != hipSuccess)
        return err;
    hipLaunchKernelGGL(fn, dim3(grid), dim3(512), lds_bytes, stream, a);
    return hipGetLastError();
}

}  // namespace convmi
