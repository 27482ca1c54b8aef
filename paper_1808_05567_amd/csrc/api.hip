// C ABI of libconv_mi355x: descriptor validation and per-layer planning (done
// once at conv_create, the analogue of the dryrun phase of Section II-H),
// and the entry points that only enqueue kernels.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>
#include <unordered_map>

#include "conv_internal.h"

using namespace convmi;

namespace convmi {
hipError_t ensure_dynamic_lds(const void *kernel, size_t bytes)
{
    static std::mutex mu;
    static std::unordered_map<const void *, size_t> have;
    std::lock_guard<std::mutex> lock(mu);
    size_t &cur = have[kernel];
    if (bytes <= cur) return hipSuccess;
    const hipError_t err =
        hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (err == hipSuccess) cur = bytes;
    return err;
}
}  // namespace convmi

namespace {

struct IgemmPlan {
    bool ok = false;
    IgemmVariant v{};
    IgemmArgs a{};
    size_t lds = 0;
    int grid = 0;
};

struct BwdClass {  // one stride-parity class of the generic backward pass
    IgemmPlan p;
    WtXformArgs x{};
    WtMergeArgs m{};      // all classes in one launch (merged == true)
    bool merged = false;
    size_t ws_off = 0;
};

}  // namespace

struct conv_plan {
    conv_desc_t d;
    int pad_h = 0, pad_w = 0;  // zero padding per axis (d.pad is not used past conv_create)
    conv_info_t info;
    IgemmPlan fwd;
    size_t fwd_ws = 0;  // bytes of fp32 partial results if the forward reduction is split
    size_t fwd_stem_lds = 0;  // > 0: the plain forward pass runs on the resident-filter kernel (its LDS)
    // backward by data
    int bwd_mode = 0;  // 0 unsupported, 1 one launch (duality), 2 parity classes
    int n_bwd = 0;
    BwdClass bwd[16];
    size_t bwd_ws = 0;
    // weight update
    bool upd_ok = false;
    bool upd_c4 = false;   // few-channel formulation (one input channel block)
    bool upd_c4_bf16 = false; // bf16, one input channel block: (tap, channel) rows on the bf16 MFMA
    bool upd_rows = false; // bf16 row kernel (stride 1)
    int upd_bands_layout = 0;  // fp32 band kernel: 0 = 2x2 channel waves x 2 pixel groups, 1 = 1x2x4, 2 = 1x1x8
    bool upd_bands = false; // fp32 eight-wave band kernel
    bool upd_flat_bf16 = false; // bf16 1x1 eight-wave kernel on the flat pixel list (variant: urv)
    bool upd_flat = false;  // fp32 1x1 eight-wave kernel on the flat pixel list
    int upd_wb = 0;         //   its waves along the narrower tensor's channels
    bool upd_a_is_in = false; //   whether the wider tensor is the input
    UpdRowsVariant urv{};
    int upd_copies = 0;    // partial dW copies the reduce kernel sums
    UpdVariant uv{};
    int upd_row_launches = 1;  // > 1: one launch of a 1 x S kernel per filter row
    int upd_strips = 1;        // general kernels: strips of output columns, one launch each
    int upd_strip_w = 0;       // ... their width (the last may be narrower)
    UpdArgs ua{};
    size_t upd_lds = 0;
    int upd_grid = 0;
    size_t upd_ws = 0;
    // passes no tiled kernel fits run on the untiled direct kernels (no workspace)
    bool fwd_direct = false, bwd_direct = false, upd_direct = false;
    DirectArgs da{};
    // The minibatch in chunks of chunk_n images (the last chunk has the rest), each a plan of
    // its own run on its slice of the tensors: for tensors beyond the tiled kernels' 32-bit
    // byte offsets, or on request.  n_chunks == 0: none.
    int n_chunks = 0, chunk_n = 0;
    conv_plan *chunk = nullptr, *tail = nullptr;  // owned; tail: the last chunk if it is smaller
    bool fwd_chunked = false, bwd_chunked = false, upd_chunked = false;
    size_t chunk_ws = 0;  // the chunks' own workspace; the per-chunk dW results follow it
    ~conv_plan()
    {
        delete chunk;
        delete tail;
    }
};

namespace {

const int kMaxLds = 160 * 1024;

// Largest number of rows of the padded row space (image n occupies rows
// [n*Hs, (n+1)*Hs), output row oj of image n starts at n*Hs + oj*stride) that a
// band of TR consecutive linear output rows touches with an R-tall filter.
int max_band_rows(int N, int P, int TR, int Hs, int stride, int R)
{
    // A band's extent depends on the row it starts at within its image, rho0 % P, and those
    // repeat after at most P bands: the first P bands hold the maximum (the last band of the
    // row space can only be shorter than an earlier one of the same phase).
    const long long NP = (long long)N * P;
    const long long bands = std::min<long long>((NP + TR - 1) / TR, P);
    long long best = 0;
    for (long long b = 0; b < bands; ++b) {
        const long long rho0 = b * TR, rho1 = std::min(NP, rho0 + TR) - 1;
        const long long lam0 = (rho0 / P) * Hs + (rho0 % P) * stride;
        const long long lam1 = (rho1 / P) * Hs + (rho1 % P) * stride + R - 1;
        best = std::max(best, lam1 - lam0 + 1);
    }
    return (int)std::min<long long>(best, 1 << 30);
}

// One candidate plan of the implicit-GEMM kernel: `wk` waves along channels,
// dynamic LDS at most `lds_cap` bytes.  Returns ok=false if nothing fits.
IgemmPlan try_igemm(int dtype, int N, int Cb, int H, int W, int Kp, int P, int Q, int R, int S,
                    int stride, int pad_h, int pad_w, int OH, int OW, int ostr, int oy0, int ox0,
                    int zero_fill, const IgemmGeo &geo, int wk, int wm, int fk, int fm, size_t lds_cap,
                    int nb = 2, int npl_want = 0)
{
    IgemmPlan pl;
    // (columns of the result `cstride` input pixels apart, and `ostr_x` output pixels apart)
    const int cstride = geo.cstride > 0 ? geo.cstride : stride;
    const int ostr_x = geo.ostr_x > 0 ? geo.ostr_x : ostr;
    const int V = vlen_of(dtype);
    // (1x1, no padding: only the pixels that are read are staged -- valid where every output
    // pixel has its input pixel; a residue class of a strided backward pass can be one row or
    // column larger than its input, which then needs the zero rows of the padded row space)
    const bool sampled = (R == 1 && S == 1 && pad_h == 0 && pad_w == 0 && (P - 1) * stride < H &&
                          (Q - 1) * stride < W);

    int npl;
    if (R == 1 && S == 1)
        npl = (Cb % 4 == 0) ? 4 : 1;
    else
        npl = (Cb % 2 == 0) ? 2 : 1;
    if (npl_want > 0) {
        if (Cb % npl_want != 0) return pl;
        npl = npl_want;
    }
    // (eight waves: two groups of four, each staging its half of a step's planes)
    if (wk * wm == 8 && npl % 2 != 0) return pl;

    // (NT: threads of one staging group -- the input tile's chunks are dealt per group)
    const int TK = wk * fk * 32, TM = wm * fm * 32, NT = 256;
    const int nent = ((R * S * npl + 1) / 2) * 2;

    int ppt = -1;
    int TQ = std::min(Q, TM);
    int TR = std::max(1, TM / TQ);
    TR = std::min(TR, N * P);
    int Hs = 0, LW = 0, LR = 0;
    for (;; --TR) {
        if (TR < 1) return pl;
        if (sampled) {
            Hs = P;
            LW = TQ;
            LR = TR;
        } else {
            Hs = (P - 1) * stride + R;
            LW = (TQ - 1) * cstride + S;
            LR = max_band_rows(N, P, TR, Hs, stride, R);
        }
        const int need = ceil_div(LR * LW, NT);
        ppt = -1;
        for (int cand = need; cand <= 16; ++cand) {
            IgemmVariant v{dtype, wk, wm, fk, fm, npl, R, S, cand, nb};
            if (igemm_variant_exists(v)) {
                ppt = cand;
                break;
            }
        }
        // the plane pitch is a whole number of wave-level (64-lane) loads
        // (a single-step reduction never touches the second buffer)
        const size_t nbuf = ceil_div(Cb, npl) > 1 ? (size_t)nb : 1;
        const size_t lds = nbuf * ((size_t)nent * TK * 16 + (size_t)npl * ceil_div(LR * LW, 64) * 64 * 16);
        if (ppt > 0 && lds <= lds_cap) break;
    }

    IgemmArgs &a = pl.a;
    memset(&a, 0, sizeof(a));
    a.N = N; a.Cb = Cb; a.H = H; a.W = W; a.Kp = Kp; a.P = P; a.Q = Q;
    a.stride = stride; a.cstride = cstride; a.pad_h = pad_h; a.pad_w = pad_w;
    a.OH = OH; a.OW = OW; a.ostr = ostr; a.ostr_x = ostr_x; a.oy0 = oy0; a.ox0 = ox0; a.zero_fill = zero_fill;
    a.shuffle = 0; a.out_kb = Kp / V;
    a.ksplit = 1;
    a.scale = nullptr; a.bias = nullptr; a.resid = nullptr; a.relu = 0;
    a.TR = TR; a.TQ = TQ;
    a.n_qt = ceil_div(Q, TQ);
    a.n_mt = ceil_div(N * P, TR);
    a.n_kt = ceil_div(Kp, TK);
    a.Hs = Hs; a.LW = LW; a.LRW = LR * LW; a.PLS = ceil_div(LR * LW, 64) * 64;
    a.sampled = sampled ? 1 : 0;
    a.inv_P = 1.0f / (float)P; a.inv_Hs = 1.0f / (float)Hs;
    a.inv_LW = 1.0f / (float)LW; a.inv_TQ = 1.0f / (float)TQ;
    a.total = a.n_mt * a.n_qt * a.n_kt;
    {
        // Tiles over the XCDs (see the kernel): bytes from beyond the L2s are about
        // gk x input + (8/gk) x weights, provided an XCD's share of the weights (1/gk of
        // them) leaves room in its 4 MB L2 for the input tiles in flight.
        const double in_b = (double)N * Cb * (sampled ? (double)P * Q : (double)H * W) * 16.0;
        const double wt_b = (double)Cb * R * S * Kp * 16.0;
        int best_gk = 1;
        double best = 0;
        for (int gk = 1; gk <= 8; gk *= 2) {
            if (gk > a.n_kt) break;
            if (a.n_kt % gk != 0 && gk > 1) continue;
            double cost = gk * in_b + (8.0 / gk) * wt_b;
            if (wt_b / gk > 2.0e6) cost += 8.0 * in_b;  // the weights would not stay resident
            if (gk == 1 || cost < best) { best = cost; best_gk = gk; }
        }
        if (const char *env = getenv("CONVMI_IGEMM_GK")) {
            const int g = atoi(env);
            if ((g == 1 || g == 2 || g == 4 || g == 8) && g <= a.n_kt && a.n_kt % g == 0) best_gk = g;
        }
        a.gk = best_gk;
        a.kt_per = ceil_div(a.n_kt, a.gk);
        a.mq_per = ceil_div(a.n_mt * a.n_qt, 8 / a.gk);
        a.per_xcd = a.kt_per * a.mq_per;
    }
    a.n_stage = ceil_div(Cb, npl);
    a.st_per = a.n_stage;
    // (measured at N = 256, bf16, operands not in cache: 6 - 13 % on the forward pass of the deep
    // 1x1 layers, nothing lost elsewhere; CONVMI_IGEMM_ROT="rk,rm" overrides, a tuning aid)
    a.rot_k = 1;
    a.rot_m = 1;
    if (const char *env = getenv("CONVMI_IGEMM_ROT")) {
        int rk = 0, rm = 0;
        if (sscanf(env, "%d,%d", &rk, &rm) == 2 && rk >= 0 && rm >= 0) { a.rot_k = rk; a.rot_m = rm; }
    }
    pl.v = IgemmVariant{dtype, wk, wm, fk, fm, npl, R, S, ppt, nb};
    pl.lds = (a.n_stage > 1 ? nb : 1) * ((size_t)nent * TK * 16 + (size_t)npl * a.PLS * 16);
    pl.grid = a.per_xcd * 8;
    // 32-bit index guards (offsets are kept in 16-byte units / elements)
    // tensors are addressed with 32-bit byte offsets
    const double in_units = (double)N * Cb * H * W, out_units = (double)N * (Kp / V) * OH * OW;
    if (in_units * 16 > 4.0e9 || out_units * 16 > 4.0e9) return pl;
    // the kernels divide small indices through a float reciprocal, exact below 2^22
    if ((double)(N + 1) * std::max(Hs, P) >= 4.0e6 || a.LRW >= (1 << 22)) return pl;
    // ... and multiply row indices (image x channel block x row) as 24-bit integers
    if ((double)(N + 1) * std::max(Cb, Kp / V) * std::max(std::max(H, OH), Hs) >= 8.0e6) return pl;
    pl.ok = true;
    return pl;
}

// MFMA work a plan issues relative to the useful work: padded pixel slots of
// the tiles and padded channel rows both cost full MFMA time.
double igemm_waste(const IgemmPlan &p, int N, int P, int Q, int Kp)
{
    const double TM = p.v.wm * p.v.fm * 32.0, TK = p.v.wk * p.v.fk * 32.0;
    return (p.a.n_mt * p.a.n_qt * TM * p.a.n_kt * TK) / ((double)N * P * Q * Kp);
}

// Plan one launch of the implicit-GEMM kernel.
//   input tensor:  N x Cb blocks x H x W;  result extent P x Q;  A rows Kp.
// Candidates: 4 or 2 waves along channels, tile within half of the LDS (two
// workgroups per CU overlap each other's barriers and staging) or all of it.
// Preference: least wasted MFMA work, then two workgroups per CU, then the
// wider channel tile (fewer re-reads of the input tile).
IgemmPlan plan_igemm_tile(int dtype, int N, int Cb, int H, int W, int Kp, int P, int Q, int R, int S,
                          int stride, int pad_h, int pad_w, int OH, int OW, int ostr, int oy0, int ox0,
                          int zero_fill, const IgemmGeo &geo);

IgemmPlan plan_igemm(int dtype, int N, int Cb, int H, int W, int Kp, int P, int Q, int R, int S,
                     int stride, int pad_h, int pad_w, int OH, int OW, int ostr, int oy0, int ox0,
                     int zero_fill, const IgemmGeo &geo = IgemmGeo{})
{
    IgemmPlan p = plan_igemm_tile(dtype, N, Cb, H, W, Kp, P, Q, R, S, stride, pad_h, pad_w, OH, OW, ostr,
                                  oy0, ox0, zero_fill, geo);
    // One channel tile: every line of the input is staged by exactly one workgroup.  Loaded
    // non-temporally it does not displace the weights in the L2 nor settle in the last-level
    // cache on its way past.  The same with two channel tiles side by side on an XCD, as long as
    // every XCD walks all channel tiles (one channel group): the second reader still finds the
    // line (measured at N = 256: bf16 layer 6 forward -15 %, layer 11 backward -8 %, fp32 layers
    // 6 and 14 backward -3 %).  With several channel groups the XCDs of the other groups fetch
    // the same lines later, from the last-level cache: there the hint costs 8 - 17 % (layer 16).
    // (CONVMI_IGEMM_NT: 0 never, 1 wherever the variant exists, 2 one channel tile only -- tuning aids.)
    const char *env = getenv("CONVMI_IGEMM_NT");
    const int mode = env ? atoi(env) : -1;
    const bool want = mode == 0 ? false
                      : mode == 1 ? true
                      : mode == 2 ? p.a.n_kt == 1
                                  : (p.a.n_kt == 1 || (p.a.gk == 1 && p.a.kt_per <= 2));
    if (p.ok && want) {
        IgemmVariant v = p.v;
        v.nt = 1;
        if (igemm_variant_exists(v)) p.v = v;
    }
    return p;
}

IgemmPlan plan_igemm_tile(int dtype, int N, int Cb, int H, int W, int Kp, int P, int Q, int R, int S,
                          int stride, int pad_h, int pad_w, int OH, int OW, int ostr, int oy0, int ox0,
                          int zero_fill, const IgemmGeo &geo)
{
    IgemmPlan best;
    double best_cost = 0;
    const size_t caps[2] = {(size_t)kMaxLds / 2, (size_t)kMaxLds};
    struct Cand { int wk, wm, fk, fm; };
    // bf16: two channel fragments per wave halve the LDS reads per MFMA (one
    // fragment per wave cannot keep the bf16 matrix core fed from 128 B/clk of LDS)
    // (the last: 32 rows, for results with at most 32 channel rows)
    const Cand cands[6] = {{1, 4, 2, 4}, {2, 2, 2, 7}, {1, 4, 2, 7}, {4, 1, 1, 7}, {2, 2, 1, 7},
                           {1, 4, 1, 7}};
    for (int ci = 0; ci < 2; ++ci)
        for (const Cand &cd : cands) {
            if (cd.fk == 2 && dtype != CONV_BF16) continue;
            const int TK = cd.wk * cd.fk * 32;
            if (TK > 64 && Kp <= TK / 2) continue;
            if (TK == 32 && Kp > 96) continue;  // (three 32-row tiles at most: 80 rows waste less so)
            IgemmPlan c = try_igemm(dtype, N, Cb, H, W, Kp, P, Q, R, S, stride, pad_h, pad_w, OH, OW,
                                    ostr, oy0, ox0, zero_fill, geo, cd.wk, cd.wm, cd.fk, cd.fm, caps[ci]);
            if (!c.ok) continue;
            // one workgroup per CU loses roughly a fifth to exposed barriers/staging
            double cost = igemm_waste(c, N, P, Q, Kp) * (ci == 0 ? 1.0 : 1.2) *
                          (1.0 + 0.01 * (128 / TK));
            // rounds of workgroups over the 256 CUs: a last, partly filled round costs a full one
            const int slots = 256 * (ci == 0 ? 2 : 1);
            cost *= (double)(ceil_div(c.a.total, slots) * slots) / c.a.total;
            // one fragment per wave starves the bf16 matrix core of LDS bandwidth; it only
            // matters where the filter gives the layer enough reuse to be MFMA-bound
            if (dtype == CONV_BF16 && cd.fk == 1 && R * S > 1) cost *= 1.5;
            if (dtype == CONV_BF16 && cd.fk == 2 && R * S == 1) cost *= 1.5;
            if (!best.ok || cost < best_cost) {
                best = c;
                best_cost = cost;
            }
        }
    // Two cells per column (a strided backward pass into one channel block): the staged tile
    // is twice as wide per result column, and with two channel planes per step the band that
    // fits the LDS leaves a third of the pixel slots empty; one plane per step fits a full
    // band (measured on the 7x7 stride-2 layer at N = 256, fp32: 1.65 ms against 1.07 ms).
    if (geo.cstride > 1 && R * S > 1) {
        for (const Cand &cd : cands) {
            if (cd.fk == 2 && dtype != CONV_BF16) continue;
            if (cd.wk * cd.fk * 32 != 32 || Kp > 32) continue;
            IgemmPlan c = try_igemm(dtype, N, Cb, H, W, Kp, P, Q, R, S, stride, pad_h, pad_w, OH, OW,
                                    ostr, oy0, ox0, zero_fill, geo, cd.wk, cd.wm, cd.fk, cd.fm,
                                    (size_t)kMaxLds, 2, 1);
            if (c.ok && (!best.ok || igemm_waste(c, N, P, Q, Kp) < 0.9 * igemm_waste(best, N, P, Q, Kp)))
                best = c;
        }
    }
    // Tuning aid: CONVMI_IGEMM_CAND="wk,wm,fk,fm,nb,npl" asks for one kernel variant wherever it
    // exists and fits (npl 0: the default planes per step); unset in normal use.
    if (const char *env = getenv("CONVMI_IGEMM_CAND")) {
        int wk = 0, wm = 0, fk = 0, fm = 0, nb = 2, npl = 0;
        if (sscanf(env, "%d,%d,%d,%d,%d,%d", &wk, &wm, &fk, &fm, &nb, &npl) >= 4 && wk > 0 && wm > 0 &&
            fk > 0 && fm > 0 && (wk * wm == 4 || wk * wm == 8) && nb >= 2 && nb <= 5) {
            IgemmPlan c = try_igemm(dtype, N, Cb, H, W, Kp, P, Q, R, S, stride, pad_h, pad_w, OH, OW,
                                    ostr, oy0, ox0, zero_fill, geo, wk, wm, fk, fm, (size_t)kMaxLds, nb, npl);
            if (c.ok) return c;
        }
    }
    // bf16, eight waves (two per SIMD inside one workgroup, one workgroup per CU): a 256 x 256
    // tile for 1x1 filters (four MFMA rounds per step), 128 x 512 for 3x3.  One staged tile
    // feeds twice the MFMAs of two four-wave workgroups, which is what layers bound by the
    // rate at which a CU pulls tiles in from memory gain from (measured at N = 256: 5 - 12 %
    // on the 1x1 layers with at least 256 output rows and 128 input channels, 2 - 6 % on the
    // 28 x 28 and 14 x 14 3x3 layers).  Not for results narrower than the tile, and not where
    // the tiles would not fill the chip (there the four-wave tiles, or a split reduction, do).
    // ... except where the reduction is short (at most 256 channels) and the result wide: a
    // tile then spends as long on its first loads and its stores as on its MFMAs, and two
    // four-wave workgroups per CU with 128 x 256 tiles, which overlap each other's ends, are
    // 10 - 12 % faster than one eight-wave workgroup (measured on the 128 -> 512 and
    // 256 -> 1024 layers and the backward pass of 1024 -> 256).
    if (dtype == CONV_BF16 && best.ok && R * S == 1 && stride == 1 && ostr == 1 && Kp >= 512 &&
        Cb <= 32 && Cb % 4 == 0) {
        IgemmPlan c = try_igemm(dtype, N, Cb, H, W, Kp, P, Q, R, S, stride, pad_h, pad_w, OH, OW, ostr, oy0,
                                ox0, zero_fill, geo, 2, 2, 2, 4, (size_t)kMaxLds / 2, 2, 4);
        if (c.ok && c.a.total >= 300 && igemm_waste(c, N, P, Q, Kp) <= 1.1 * igemm_waste(best, N, P, Q, Kp))
            return c;
    }
    if (dtype == CONV_BF16 && best.ok) {
        IgemmPlan c;
        if (R * S == 1 && Kp >= 256 && Cb % 8 == 0)
            c = try_igemm(dtype, N, Cb, H, W, Kp, P, Q, R, S, stride, pad_h, pad_w, OH, OW, ostr, oy0,
                          ox0, zero_fill, geo, 4, 2, 2, 4, (size_t)kMaxLds, 2, 8);
        else if (R == 3 && S == 3 && stride == 1 && Kp >= 128 && Cb % 2 == 0)
            c = try_igemm(dtype, N, Cb, H, W, Kp, P, Q, R, S, stride, pad_h, pad_w, OH, OW, ostr, oy0,
                          ox0, zero_fill, geo, 2, 4, 2, 4, (size_t)kMaxLds, 2, 2);
        if (c.ok && c.a.total >= 150 && igemm_waste(c, N, P, Q, Kp) <= 1.1 * igemm_waste(best, N, P, Q, Kp))
            return c;
        // a result of one 32-row tile under a filter window (the merged classes of a strided
        // backward pass into one channel block): eight pixel waves, 32 x 1792; the band that
        // fits the LDS fills 7/8 of it and is still 13 % faster than four waves (conv1, N = 256)
        if (!c.ok && R * S > 1 && Kp <= 32 && Cb % 2 == 0 && geo.cstride <= 1) {
            c = try_igemm(dtype, N, Cb, H, W, Kp, P, Q, R, S, stride, pad_h, pad_w, OH, OW, ostr, oy0,
                          ox0, zero_fill, geo, 1, 8, 1, 7, (size_t)kMaxLds, 2, 2);
            if (c.ok && c.a.total >= 512 && igemm_waste(c, N, P, Q, Kp) <= 1.15 * igemm_waste(best, N, P, Q, Kp))
                return c;
        }
    }
    // bf16 1x1: a reduction step is two MFMA rounds, far shorter than a trip to memory; a
    // third buffer keeps the loads two steps ahead where it fits the same LDS budget
    if (dtype == CONV_BF16 && R * S == 1 && best.ok && best.a.n_stage >= 3) {
        const size_t cap = best.lds <= (size_t)kMaxLds / 2 ? (size_t)kMaxLds / 2 : (size_t)kMaxLds;
        IgemmPlan c = try_igemm(dtype, N, Cb, H, W, Kp, P, Q, R, S, stride, pad_h, pad_w, OH, OW, ostr,
                                oy0, ox0, zero_fill, geo, best.v.wk, best.v.wm, best.v.fk, best.v.fm, cap, 3);
        if (c.ok && c.a.total <= best.a.total) best = c;
    }
    // ... and where the tiles number no more than the CUs (a narrow result behind a deep
    // reduction: the 7x7 layers that narrow the channel count) a workgroup has its CU to itself
    // anyway: eight channel blocks per step then, four MFMA rounds between two barriers instead
    // of two and twice the bytes in flight (measured at N = 256: layer 20 forward 76 -> 55 us,
    // layer 19 backward 83 -> 60, layer 17 forward 64 -> 54; deeper rings change nothing).
    if (dtype == CONV_BF16 && R * S == 1 && best.ok && best.v.wk * best.v.wm == 4 && best.v.fk == 1 &&
        best.a.total <= 256 && Cb % 8 == 0 && Cb >= 32) {
        IgemmPlan c = try_igemm(dtype, N, Cb, H, W, Kp, P, Q, R, S, stride, pad_h, pad_w, OH, OW, ostr,
                                oy0, ox0, zero_fill, geo, best.v.wk, best.v.wm, best.v.fk, best.v.fm,
                                (size_t)kMaxLds, 2, 8);
        if (c.ok && c.a.total <= best.a.total) best = c;
    }
    return best;
}

void plan_bwd(conv_plan *p)
{
    const conv_desc_t &d = p->d;
    const conv_info_t &f = p->info;
    const int es = esize_of(d.dtype);
    p->bwd_mode = 0;
    p->n_bwd = 0;
    p->bwd_ws = 0;
    const int pad_h = p->pad_h, pad_w = p->pad_w;
    if (d.stride == 1 && pad_h <= d.R - 1 && pad_w <= d.S - 1) {
        BwdClass &b = p->bwd[0];
        b.p = plan_igemm(d.dtype, d.N, f.Kb, f.P, f.Q, f.Cp, d.H, d.W, d.R, d.S, 1, d.R - 1 - pad_h,
                         d.S - 1 - pad_w, d.H, d.W, 1, 0, 0, 0);
        b.x = WtXformArgs{nullptr, nullptr, f.Cb, f.Kb, f.Cp, f.Kp, d.R, d.S, d.R, d.S,
                          1, 0, 0, d.R, d.S};
        b.ws_off = 0;
        if (b.p.ok) {
            p->bwd_mode = 1;
            p->n_bwd = 1;
            p->bwd_ws = (size_t)f.Kb * d.R * d.S * f.Cp * f.vlen * es;
        }
        return;
    }
    if (d.R == 1 && d.S == 1 && pad_h == 0 && pad_w == 0) {
        BwdClass &b = p->bwd[0];
        b.p = plan_igemm(d.dtype, d.N, f.Kb, f.P, f.Q, f.Cp, f.P, f.Q, 1, 1, 1, 0, 0, d.H, d.W,
                         d.stride, 0, 0, 1);
        b.x = WtXformArgs{nullptr, nullptr, f.Cb, f.Kb, f.Cp, f.Kp, 1, 1, 1, 1, 1, 0, 0, 1, 1};
        b.ws_off = 0;
        if (b.p.ok) {
            p->bwd_mode = 1;
            p->n_bwd = 1;
            p->bwd_ws = (size_t)f.Kb * f.Cp * f.vlen * es;
        }
        return;
    }
    // Generic case: one stride-1 sub-convolution per residue class (py, px) of
    // the dI position modulo the stride, over the taps congruent to it.
    const int st = d.stride;
    if (st * st > 16) return;
    // dI with one channel block (conv1): the classes' sub-filters become the
    // rows of one filter over their common window, class (py, px) in channel
    // block py*st+px of the result, and the store interleaves the blocks into
    // the st x st cells of dI.  One launch, and st*st*vlen live rows per MFMA
    // instead of vlen.
    if (f.Cb == 1 && st * st * f.vlen <= 32 && st <= 4) {
        BwdClass &b = p->bwd[0];
        WtMergeArgs &m = b.m;
        memset(&m, 0, sizeof(m));
        int padU[2] = {0, 0}, win[2] = {1, 1};
        for (int ax = 0; ax < 2; ++ax) {
            const int F = ax == 0 ? d.R : d.S;
            const int pad_ax = ax == 0 ? pad_h : pad_w;
            int *sub = ax == 0 ? m.rsub : m.ssub, *roff = ax == 0 ? m.roff : m.soff;
            int *sh = ax == 0 ? m.rsh : m.ssh;
            int padc[4];
            for (int pp = 0; pp < st; ++pp) {
                const int ro = (pp + pad_ax) % st;
                sub[pp] = ro < F ? ceil_div(F - ro, st) : 0;
                roff[pp] = ro;
                padc[pp] = std::max(sub[pp], 1) - 1 - (pp + pad_ax) / st;
                padU[ax] = pp == 0 ? padc[pp] : std::max(padU[ax], padc[pp]);
            }
            for (int pp = 0; pp < st; ++pp) {
                sh[pp] = padU[ax] - padc[pp];
                win[ax] = std::max(win[ax], std::max(sub[pp], 1) + sh[pp]);
            }
        }
        // Where the classes fill only half of an MFMA's 32 rows (fp32, stride 2), a column of
        // the result stands for TWO cells side by side: 32 live rows, half the columns, and a
        // window one tap wider (cell e of the pair reads its taps e columns to the right).
        // (CONVMI_BWD_CELLS=1 keeps one cell per column: a tuning aid.)
        int cells = (2 * st * st * f.vlen <= 32 && ceil_div(d.W, st) >= 2) ? 2 : 1;
        if (const char *env = getenv("CONVMI_BWD_CELLS"); env && atoi(env) == 1) cells = 1;
        const int Hc = ceil_div(d.H, st), Wc = ceil_div(d.W, st);
        for (; cells >= 1 && padU[0] >= 0 && padU[1] >= 0; --cells) {
            m.Kb = f.Kb; m.Kp = f.Kp; m.R = d.R; m.S = d.S; m.R2 = win[0]; m.S2 = win[1] + cells - 1;
            m.st = st; m.cells = cells;
            IgemmGeo geo;
            geo.cstride = cells;
            geo.ostr_x = cells * st;
            b.p = plan_igemm(d.dtype, d.N, f.Kb, f.P, f.Q, cells * st * st * f.vlen, Hc, ceil_div(Wc, cells),
                             m.R2, m.S2, 1, padU[0], padU[1], d.H, d.W, st, 0, 0, 0, geo);
            if (b.p.ok) {
                b.p.a.shuffle = 1;
                b.p.a.out_kb = 1;
                b.merged = true;
                b.ws_off = 0;
                p->bwd_mode = 3;
                p->n_bwd = 1;
                p->bwd_ws = (size_t)f.Kb * m.R2 * m.S2 * cells * st * st * f.vlen * f.vlen * es;
                return;
            }
        }
    }
    const int R2 = ceil_div(d.R, st), S2 = ceil_div(d.S, st);
    size_t off = 0;
    int n = 0;
    for (int py = 0; py < st; ++py)
        for (int px = 0; px < st; ++px) {
            const int ry = (py + pad_h) % st, rx = (px + pad_w) % st;
            const int Rsub = ry < d.R ? ceil_div(d.R - ry, st) : 0;
            const int Ssub = rx < d.S ? ceil_div(d.S - rx, st) : 0;
            const int dy0 = (py + pad_h) / st, dx0 = (px + pad_w) / st;
            const int Hsub = py < d.H ? ceil_div(d.H - py, st) : 0;
            const int Wsub = px < d.W ? ceil_div(d.W - px, st) : 0;
            if (Hsub == 0 || Wsub == 0) continue;
            BwdClass &b = p->bwd[n];
            // With no tap in the class the sub-filter is all zero and the
            // launch writes zeros, which is what Algorithm 6 leaves there.
            const int Re = std::max(Rsub, 1), Se = std::max(Ssub, 1);
            // the class's own sub-filter extent where a kernel exists for it, else
            // the common extent with zero taps
            int R2c = Re, S2c = Se;
            b.p = plan_igemm(d.dtype, d.N, f.Kb, f.P, f.Q, f.Cp, Hsub, Wsub, R2c, S2c, 1,
                             Re - 1 - dy0, Se - 1 - dx0, d.H, d.W, st, py, px, 0);
            if (!b.p.ok) {
                R2c = R2;
                S2c = S2;
                b.p = plan_igemm(d.dtype, d.N, f.Kb, f.P, f.Q, f.Cp, Hsub, Wsub, R2c, S2c, 1,
                                 Re - 1 - dy0, Se - 1 - dx0, d.H, d.W, st, py, px, 0);
            }
            if (!b.p.ok) return;
            b.x = WtXformArgs{nullptr, nullptr, f.Cb, f.Kb, f.Cp, f.Kp, d.R, d.S, R2c, S2c,
                              st, ry, rx, Rsub, Ssub};
            if (Rsub == 0 || Ssub == 0) { b.x.Rsub = 0; b.x.Ssub = 0; }
            b.ws_off = off;
            off += (size_t)f.Kb * R2c * S2c * f.Cp * f.vlen * es;
            ++n;
        }
    p->bwd_mode = 2;
    p->n_bwd = n;
    p->bwd_ws = off;
}

// Weight update, bf16, at most 4 input channels: (tap, channel) rows on the bf16 MFMA.
bool plan_upd_c4_bf16(conv_plan *p)
{
    const conv_desc_t &d = p->d;
    const conv_info_t &f = p->info;
    const int pad_h = p->pad_h, pad_w = p->pad_w;
    const bool bf16 = d.dtype == CONV_BF16;
    if (bf16 && d.C <= 4 && upd_c4_bf16_exists(d.R, d.S)) {
        // one input channel block, bf16: (tap, channel) rows on the bf16 MFMA, eight waves,
        // two LDS buffers holding the bands as they sit in HBM
        auto plan_c4_bf16 = [&]() -> bool {
            const int NPO = 8;  // planes of 8 output channels
            const int NP = d.N * f.P;
            UpdArgs &a = p->ua;
            memset(&a, 0, sizeof(a));
            a.N = d.N; a.Cb = 1; a.H = d.H; a.W = d.W; a.Kb = f.Kb; a.Kp = f.Kp; a.P = f.P; a.Q = f.Q;
            a.R = d.R; a.S = d.S; a.stride = d.stride; a.pad = pad_h; a.pad_w = pad_w;
            a.tap0 = 0; a.ntaps_all = d.R * d.S;
            a.q0 = 0; a.Qpitch = f.Q; a.copy0 = 0;
            a.runs = ceil_div(f.Q, 8);
            const int RP = a.runs * 8;
            a.Hs = (f.P - 1) * d.stride + d.R;
            // a lane addresses up to 7 pixels past the first pixel of its run's last window
            a.LW = std::max(d.W + 2 * pad_w, d.stride * (RP - 1) + 8);
            int TR = std::min(NP, 16);
            for (;; --TR) {
                if (TR < 1) return false;
                const int LR = max_band_rows(d.N, f.P, TR, a.Hs, d.stride, d.R);
                a.LRW = LR * a.LW;
                a.PLS_in = ceil_div(a.LRW, 64) * 64;
                // (+4 pixels: the two planes a 16-lane transposing read touches start 64
                // bytes apart in the 256-byte bank row)
                a.PLS_out = ceil_div(TR * RP + 8, 64) * 64 + 4;
                p->upd_lds = 2 * ((size_t)a.PLS_in + (size_t)NPO * a.PLS_out) * 16;
                if (p->upd_lds <= (size_t)kMaxLds) break;
            }
            p->upd_lds = std::max(p->upd_lds, (size_t)16 * 1024);  // the accumulator exchange
            a.TR = TR;
            a.n_ct = 1;
            a.n_kt = ceil_div(f.Kp, 64);
            int splits = std::max(1, 256 / a.n_kt);  // one workgroup per CU, one round
            splits = std::max(splits, ceil_div(NP * f.Q, 1 << 17));
            int rps = ceil_div(ceil_div(NP, splits), TR) * TR;
            splits = ceil_div(NP, rps);
            a.rows_per_split = rps;
            a.splits = splits;
            a.sampled = 0;
            a.total = a.n_kt * splits;
            a.per_xcd = ceil_div(a.total, 8);
            if ((double)(d.N + 1) * std::max(a.Hs, std::max(d.H, f.P * f.Kb)) >= 4.0e6 ||
                a.LRW >= (1 << 22) || TR * RP + 8 >= (1 << 22) || (double)d.N * d.H * d.W * 16 >= 4.0e9 ||
                (double)d.N * f.Kp * f.P * f.Q * 2 >= 4.0e9)
                return false;
            p->upd_grid = a.per_xcd * 8;
            p->upd_copies = splits;
            p->upd_ws = (size_t)p->upd_copies * f.dwt_bytes;
            p->upd_c4_bf16 = true;
            p->upd_ok = true;
            return true;
        };
        if (plan_c4_bf16()) return true;
    }
    return false;
}

// Weight update, at most 4 input channels, fp32 MFMA (fp32 tensors, or bf16 widened into LDS).
bool plan_upd_c4(conv_plan *p)
{
    const conv_desc_t &d = p->d;
    const conv_info_t &f = p->info;
    const int pad_h = p->pad_h, pad_w = p->pad_w;
    const bool bf16 = d.dtype == CONV_BF16;
    const bool square_pad = pad_h == pad_w;  // the filter-specific kernels take one pad
    if (d.C <= 4 && square_pad && ((d.R == 7 && d.S == 7) || (d.R == 3 && d.S == 3))) {
        // (a plan that does not fit leaves the layer to the general kernels)
        auto plan_c4 = [&]() -> bool {
            // one input channel block: filter-row formulation, eight waves, two LDS buffers
            const int NPO = 16;
            const int Qp = (f.Q + 1) & ~1;
            const int NP = d.N * f.P;
            UpdArgs &a = p->ua;
            memset(&a, 0, sizeof(a));
            a.N = d.N; a.Cb = 1; a.H = d.H; a.W = d.W; a.Kb = f.Kb; a.Kp = f.Kp; a.P = f.P; a.Q = f.Q;
            a.R = d.R; a.S = d.S; a.stride = d.stride; a.pad = pad_h; a.pad_w = pad_w;
            a.tap0 = 0; a.ntaps_all = d.R * d.S;
            a.live_ch = d.C;
            int TR = std::min(NP, std::max(1, 256 / Qp));
            for (;; --TR) {
                if (TR < 1) return false;
                a.Hs = (f.P - 1) * d.stride + d.R;
                // a lane reads up to 8 pixels (32 floats) past the pair's first pixel
                a.LW = std::max((Qp - 1) * d.stride + 8, d.W + 2 * pad_w);
                const int LR = max_band_rows(d.N, f.P, TR, a.Hs, d.stride, d.R);
                a.LRW = LR * a.LW;
                // whole wave-level loads of 64 positions; the dO plane pitch is 1 (mod 8) pixels
                a.PLS_in = ceil_div(a.LRW, 64) * 64 + 8;
                a.PLS_out = ceil_div(TR * Qp, 64) * 64 + 1;
                p->upd_lds = 2 * ((size_t)a.PLS_in + (size_t)NPO * a.PLS_out) * 16;
                if (p->upd_lds <= (size_t)kMaxLds) break;
            }
            a.TR = TR;
            a.n_ct = 1;
            a.n_kt = ceil_div(f.Kp, 64);  // 64 output channels per workgroup
            // (bf16 tensors: the staged band must fit the kernel's register staging)
            if (bf16 && (a.PLS_in - 8 > 8 * 512 || 8 * TR * Qp > 4 * 512)) return false;
            // one workgroup per CU, one round
            int splits = std::max(1, 256 / a.n_kt);
            splits = std::max(splits, ceil_div(NP * f.Q, 1 << 17));  // chains of at most 2^15 pixels
            int rps = ceil_div(ceil_div(NP, splits), TR) * TR;
            splits = ceil_div(NP, rps);
            a.rows_per_split = rps;
            a.splits = splits;
            a.sampled = 0;
            a.total = a.n_kt * splits;
            a.per_xcd = ceil_div(a.total, 8);
            if ((double)(d.N + 1) * std::max(a.Hs, std::max(d.H, f.P * f.Kb)) >= 8.0e6 ||
                a.LRW >= (1 << 22) || 8 * TR * Qp >= (1 << 22) || (double)d.N * d.H * d.W * 16 >= 4.0e9 ||
                (double)d.N * f.Kp * f.P * f.Q * 4 >= 4.0e9)
                return false;
            p->upd_grid = a.per_xcd * 8;
            p->upd_copies = splits;
            p->upd_ws = (size_t)p->upd_copies * f.dwt_bytes;
            p->upd_c4 = true;
            p->upd_ok = true;
            return true;
        };
        if (plan_c4()) return true;
    }
    return false;
}

// Weight update, fp32 1x1 without padding: flat pixel list, eight waves.
bool plan_upd_flat_f32(conv_plan *p)
{
    const conv_desc_t &d = p->d;
    const conv_info_t &f = p->info;
    const int pad_h = p->pad_h, pad_w = p->pad_w;
    const bool sampled = (d.R == 1 && d.S == 1 && pad_h == 0 && pad_w == 0);
    const bool bf16 = d.dtype == CONV_BF16;
    if (!bf16 && sampled) {
        // fp32 1x1: 256 channels of the wider tensor x up to 256 of the other per workgroup,
        // the pixel list split so that one round of workgroups fills the chip
        // (the wider side, but the input wherever it has 256 channels: partial dW keeps 4
        // input channels together, which the rows of an accumulator tile store as 16 bytes)
        const bool a_is_in = f.Cp >= f.Kp || f.Cp >= 256;
        const int chA = a_is_in ? f.Cp : f.Kp, chB = a_is_in ? f.Kp : f.Cp;
        const double npix = (double)d.N * f.P * f.Q;
        const int plA = a_is_in ? f.Cb : f.Kb, plB = a_is_in ? f.Kb : f.Cb;
        if (chA >= 256 && chB >= 32 && npix < 4.0e6 &&
            (double)(d.N + 1) * std::max(f.Cb, f.Kb) < 8.0e6 && (double)d.H * d.W < 8.0e6 &&
            (double)d.N * f.Cp * d.H * d.W * 4 < 4.0e9 && (double)d.N * f.Kp * f.P * f.Q * 4 < 4.0e9) {
            const int wb = chB >= 192 ? 4 : chB >= 96 ? 2 : 1, wp = 4 / wb, BP = 32;
            UpdArgs &a = p->ua;
            memset(&a, 0, sizeof(a));
            a.N = d.N; a.Cb = f.Cb; a.H = d.H; a.W = d.W; a.Kb = f.Kb; a.Kp = f.Kp; a.P = f.P; a.Q = f.Q;
            a.R = 1; a.S = 1; a.stride = d.stride; a.pad = 0; a.pad_w = 0; a.tap0 = 0; a.ntaps_all = 1;
            const int n_at = ceil_div(plA, 64), n_bt = ceil_div(plB, 16 * wb);
            a.n_ct = a_is_in ? n_at : n_bt;
            a.n_kt = a_is_in ? n_bt : n_at;
            const int tiles = n_at * n_bt;
            const int np = (int)npix;
            int splits = std::max(1, 256 / tiles);
            splits = std::max(splits, ceil_div(np, 1 << 16));
            const int pps = ceil_div(ceil_div(np, splits), BP) * BP;
            splits = ceil_div(np, pps);
            a.rows_per_split = pps;
            a.splits = splits;
            a.sampled = 1;
            a.total = tiles * splits;
            a.per_xcd = ceil_div(a.total, 8);
            p->upd_wb = wb;
            p->upd_a_is_in = a_is_in;
            p->upd_lds = upd_f32_1x1_lds_bytes(wb);
            p->upd_grid = a.per_xcd * 8;
            p->upd_copies = splits;
            p->upd_ws = (size_t)p->upd_copies * f.dwt_bytes;
            p->upd_flat = true;
            (void)wp;
            p->upd_ok = true;
            return true;
        }
    }
    return false;
}

// Weight update, bf16 1x1 without padding: flat pixel list.
bool plan_upd_flat_bf16(conv_plan *p)
{
    const conv_desc_t &d = p->d;
    const conv_info_t &f = p->info;
    const int pad_h = p->pad_h, pad_w = p->pad_w;
    const bool sampled = (d.R == 1 && d.S == 1 && pad_h == 0 && pad_w == 0);
    const bool bf16 = d.dtype == CONV_BF16;
    if (bf16 && sampled && (double)d.N * f.P * f.Q < 4.0e6 &&
        (double)(d.N + 1) * std::max(f.Cb, f.Kb) < 8.0e6 && (double)d.H * d.W < 8.0e6 &&
        (double)d.N * f.Cp * d.H * d.W * 2 < 4.0e9 && (double)d.N * f.Kp * f.P * f.Q * 2 < 4.0e9) {
        // bf16 1x1: the dW block that moves the fewest bytes.  The input is staged once per
        // output-channel block and dO once per input-channel block (re-reads that the L2
        // mostly serves: weight 1/2; with stride 2 only every other pixel of a fetched line
        // is used), and the pixel list is split so that one round of workgroups fills the
        // chip, each split writing a partial dW that the reduce kernel reads back (HBM both
        // ways).  Fitted to the update times of the 14x14 and 7x7 layers at N = 256 under every
        // block shape: a 128 x 256 block there beats 256 x 256 by 5 - 12 % (half the partial
        // copies), except where dW itself is the largest tensor (1024 -> 2048).
        static const UpdRowsVariant kFlat[9] = {
            {1, 1, 4, 2, 1, 2, 4}, {1, 1, 2, 2, 2, 2, 4}, {1, 1, 1, 2, 4, 2, 4},
            {1, 1, 4, 1, 2, 2, 4}, {1, 1, 2, 1, 4, 2, 4}, {1, 1, 2, 2, 2, 1, 2},
            {1, 1, 4, 1, 2, 2, 2}, {1, 1, 2, 1, 4, 2, 2}, {1, 1, 2, 2, 2, 1, 1}};
        UpdRowsVariant rv{};
        bool have = false;
        double best = 0;
        for (const UpdRowsVariant &c : kFlat) {
            if (!upd_bf16_1x1_variant_exists(c)) continue;
            const int TC = c.wc * c.fc * 32, TK = c.wk * c.fk * 32;
            const int n_ct = ceil_div(f.Cp, TC), n_kt = ceil_div(f.Kp, TK);
            const double staged = (double)f.in_bytes / d.stride * n_kt + (double)f.out_bytes * n_ct;
            const double copies = 2.0 * std::max(1, 256 / (n_ct * n_kt)) * (double)f.dwt_bytes;
            const double cost = (0.5 * staged + copies) * (1.0 + 1e-4 * (TC + TK));
            if (!have || cost < best) { rv = c; best = cost; have = true; }
        }
        // (a tuning aid: CONVMI_UPD_FLAT="wc,wk,wp,fc,fk" asks for one variant)
        if (const char *env = getenv("CONVMI_UPD_FLAT")) {
            UpdRowsVariant c{1, 1, 0, 0, 0, 0, 0};
            if (sscanf(env, "%d,%d,%d,%d,%d", &c.wc, &c.wk, &c.wp, &c.fc, &c.fk) == 5 &&
                upd_bf16_1x1_variant_exists(c)) {
                rv = c;
                have = true;
            }
        }
        if (have) {
            const int TC = rv.wc * rv.fc * 32, TK = rv.wk * rv.fk * 32, BP = 64;
            UpdArgs &a = p->ua;
            memset(&a, 0, sizeof(a));
            a.N = d.N; a.Cb = f.Cb; a.H = d.H; a.W = d.W; a.Kb = f.Kb; a.Kp = f.Kp; a.P = f.P; a.Q = f.Q;
            a.R = 1; a.S = 1; a.stride = d.stride; a.pad = 0; a.pad_w = 0; a.tap0 = 0; a.ntaps_all = 1;
            a.n_ct = ceil_div(f.Cp, TC);
            a.n_kt = ceil_div(f.Kp, TK);
            const int tiles = a.n_ct * a.n_kt;
            const int np = d.N * f.P * f.Q;
            int splits = std::max(1, 256 / tiles);
            splits = std::max(splits, ceil_div(np, 1 << 16));
            const int pps = ceil_div(ceil_div(np, splits), BP) * BP;
            splits = ceil_div(np, pps);
            a.rows_per_split = pps;
            a.splits = splits;
            a.sampled = 1;
            a.total = tiles * splits;
            a.per_xcd = ceil_div(a.total, 8);
            p->urv = rv;
            p->upd_lds = upd_bf16_1x1_lds_bytes(rv);
            p->upd_grid = a.per_xcd * 8;
            p->upd_copies = splits;
            p->upd_ws = (size_t)p->upd_copies * f.dwt_bytes;
            p->upd_flat_bf16 = true;
            p->upd_ok = true;
            return true;
        }
    }
    return false;
}

// Weight update, bf16 row kernel (8-pixel runs).
bool plan_upd_rows(conv_plan *p)
{
    const conv_desc_t &d = p->d;
    const conv_info_t &f = p->info;
    const int pad_h = p->pad_h, pad_w = p->pad_w;
    const bool sampled = (d.R == 1 && d.S == 1 && pad_h == 0 && pad_w == 0);
    const bool bf16 = d.dtype == CONV_BF16;
    // (this kernel takes the two pads separately)
    const bool rows_strided = d.stride > 1 && d.R == 3 && d.S == 3;
    const bool rows_5x5 = d.stride == 1 && d.R == 5 && d.S == 5;  // one launch per filter row
    const bool rows_rs = !sampled && (rows_strided || rows_5x5 ||
                         (d.stride == 1 &&
                          ((d.R == 3 && d.S == 3) || (d.R == 1 && (d.S == 3 || d.S == 7)) ||
                           (d.S == 1 && (d.R == 3 || d.R == 7)))));
    const int rows_R = rows_5x5 ? 1 : d.R;  // filter rows a launch of the row kernel serves
    if (bf16 && (rows_rs || sampled)) {
        // bf16 row kernel: 8-pixel runs, filter-column shifts in registers.
        // 3x3: all nine taps in the wave (144 accumulators).  1x1: the layer is bound by
        // HBM, so take the channel tile that re-reads the least (input is read once per
        // output-channel tile, dO once per input-channel tile), then the smaller tile.
        static const UpdRowsVariant k1x1[7] = {{1, 1, 2, 2, 2, 1, 1}, {1, 1, 2, 4, 1, 1, 1},
                                               {1, 1, 4, 2, 1, 1, 1}, {1, 1, 2, 4, 1, 1, 2},
                                               {1, 1, 4, 2, 1, 2, 1}, {1, 1, 2, 4, 1, 2, 2},
                                               {1, 1, 4, 2, 1, 2, 2}};
        UpdRowsVariant rv{};
        bool have = false;
        if (rows_rs) {
            // 64 x 128 channels, or 64 x 64 with two wave groups along the pixels
            rv = f.Kp <= 64 ? UpdRowsVariant{rows_R, d.S, 2, 2, 2, 1, 1, 0} : UpdRowsVariant{rows_R, d.S, 2, 4, 1, 1, 1, 0};
            rv.strided = rows_strided ? 1 : 0;
            have = upd_rows_variant_exists(rv);
        } else {
            double best = 0;
            for (const UpdRowsVariant &c : k1x1) {
                if (!upd_rows_variant_exists(c)) continue;
                const int TC = c.wc * c.fc * 32, TK = c.wk * c.fk * 32;
                const double bytes = (double)f.in_bytes * ceil_div(f.Kp, TK) +
                                     (double)f.out_bytes * ceil_div(f.Cp, TC);
                const double cost = bytes * (1.0 + 1e-4 * (TC + TK));
                if (!have || cost < best) { rv = c; best = cost; have = true; }
            }
        }
        if (have) {
            const int TC = rv.wc * rv.fc * 32, TK = rv.wk * rv.fk * 32, NPI = TC / 8, NPO = TK / 8;
            const int NP = d.N * f.P;
            UpdArgs &a = p->ua;
            memset(&a, 0, sizeof(a));
            a.N = d.N; a.Cb = f.Cb; a.H = d.H; a.W = d.W; a.Kb = f.Kb; a.Kp = f.Kp; a.P = f.P; a.Q = f.Q;
            a.R = rows_R; a.S = d.S; a.stride = d.stride; a.pad = pad_h; a.pad_w = pad_w;
            a.tap0 = 0; a.ntaps_all = d.R * d.S;
            a.q0 = 0; a.Qpitch = f.Q; a.copy0 = 0;
            a.sampled = sampled ? 1 : 0;
            const int lst = rows_strided ? d.stride : 1;  // input pixels per output pixel in a band
            a.Hs = sampled ? f.P : (f.P - 1) * lst + rows_R;
            // a lane reads a window of whole 4-pixel groups covering a run and its S-1 shifts
            const int win = (8 + d.S - 1 + 3) / 4 * 4;
            // Rows too wide for two bands in the LDS are cut into up to four strips of whole
            // 8-pixel runs, one launch per strip; beyond that the general kernel takes over.
            int TR = 0, Qs = f.Q;
            for (int ns = 1; ns <= 4 && TR < 1; ++ns) {
                Qs = ns == 1 ? f.Q : ceil_div(ceil_div(f.Q, ns), 8) * 8;
                if (ns > 1 && (sampled || Qs * (ns - 1) >= f.Q)) continue;
                a.runs = ceil_div(Qs, 8);
                const int RP = a.runs * 8;
                a.LW = sampled ? RP : std::max(ns == 1 ? d.W + 2 * pad_w : 0, RP + win - 8);
                if (rows_strided) a.LW = std::max(ns == 1 ? d.W + 2 * pad_w : 0, lst * (RP - 1) + d.S);
                for (TR = std::min(NP, 64); TR >= 1; --TR) {
                    const int LR = sampled ? TR : max_band_rows(d.N, f.P, TR, a.Hs, lst, rows_R);
                    a.LRW = LR * a.LW;
                    a.PLS_in = ceil_div(a.LRW, 64) * 64 + 4;
                    a.PLS_out = ceil_div(TR * RP + 8, 64) * 64 + 4;
                    p->upd_lds = 2 * ((size_t)NPI * a.PLS_in + (size_t)NPO * a.PLS_out) * 16;
                    if (p->upd_lds <= (size_t)kMaxLds) break;
                }
            }
            const int n_strips = ceil_div(f.Q, Qs);
            a.Q = Qs;
            if (TR >= 1) {
                a.TR = TR;
                a.n_ct = ceil_div(f.Cb, NPI);
                a.n_kt = ceil_div(f.Kb, NPO);
                const int tiles = a.n_ct * a.n_kt;
                // one workgroup per CU
                int splits = std::max(1, 256 / tiles);
                splits = std::max(splits, ceil_div(NP * f.Q, 1 << 15));
                int rps = ceil_div(ceil_div(NP, splits), TR) * TR;
                splits = ceil_div(NP, rps);
                a.rows_per_split = rps;
                a.splits = splits;
                a.total = tiles * splits;
                a.per_xcd = ceil_div(a.total, 8);
                if ((double)(d.N + 1) * std::max(a.Hs, f.P) < 4.0e6 &&
                    (double)d.N * f.Cp * d.H * d.W * 2 < 4.0e9 &&
                    (double)d.N * f.Kp * f.P * f.Q * 2 < 4.0e9) {
                    p->urv = rv;
                    p->upd_grid = a.per_xcd * 8;
                    p->upd_copies = splits * rv.wp * n_strips;
                    p->upd_ws = (size_t)p->upd_copies * f.dwt_bytes;
                    p->upd_strips = n_strips;
                    p->upd_strip_w = Qs;
                    p->upd_row_launches = rows_R == d.R ? 1 : d.R;
                    p->upd_rows = true;
                    p->upd_ok = true;
                    return true;
                }
            }
        }
    }
    return false;
}

// Weight update, fp32 band kernel.
bool plan_upd_bands(conv_plan *p)
{
    const conv_desc_t &d = p->d;
    const conv_info_t &f = p->info;
    const int pad_h = p->pad_h, pad_w = p->pad_w;
    const bool sampled = (d.R == 1 && d.S == 1 && pad_h == 0 && pad_w == 0);
    const bool bf16 = d.dtype == CONV_BF16;
    // (this kernel takes the two pads separately)
    // (stride > 1: its odd-row path only, which addresses every pixel on its own)
    if (!bf16 && !sampled && upd_f32_bands_exists(d.R, d.S)) {
        // fp32 band kernel: 64 x 64 channel tile, one workgroup per CU, the LDS holds two
        // bands; the pixel range is split so that one round of workgroups fills the chip.
        // Layers with at most 32 channels on the input side (and on both) take 32 x 64
        // (32 x 32) blocks of dW with four (eight) pixel groups where every strip has odd rows.
        // (65 to 96 input channels: three 32-channel blocks waste less than two of 64)
        const int want = f.Cp <= 32 ? (f.Kp <= 32 ? 2 : 1) : (f.Cp > 64 && f.Cp <= 96 ? 1 : 0);
        int layout = upd_f32_bands_layout_exists(d.R, d.S, want, true) ? want : 0;
        const int NP = d.N * f.P;
        UpdArgs &a = p->ua;
        memset(&a, 0, sizeof(a));
        a.N = d.N; a.Cb = f.Cb; a.H = d.H; a.W = d.W; a.Kb = f.Kb; a.Kp = f.Kp; a.P = f.P; a.Q = f.Q;
        a.R = d.R; a.S = d.S; a.stride = d.stride; a.pad = pad_h; a.pad_w = pad_w;
        a.tap0 = 0; a.ntaps_all = d.R * d.S;
        a.Hs = (f.P - 1) * d.stride + d.R;
        a.q0 = 0; a.Qpitch = f.Q; a.copy0 = 0;
        size_t lds = 0;
        // Rows too wide for two bands in the LDS are cut into up to four strips of output
        // columns, one launch per strip; beyond that the general kernel takes over.
        int TR = 0, Qs = f.Q, n_strips = 1, NPI = 16, NPO = 16;
        for (int attempt = 0; attempt < 2 && TR < 1; ++attempt) {
        if (attempt == 1) {
            if (layout == 0) break;
            layout = 0;  // no odd strips: the 64 x 64 layout
        }
        NPI = layout == 0 ? 16 : 8;
        NPO = layout == 2 ? 8 : 16;
        for (n_strips = 1; n_strips <= 4; ++n_strips) {
            Qs = ceil_div(f.Q, n_strips);
            if (ceil_div(f.Q, Qs) != n_strips) continue;
            const int q_last = f.Q - (n_strips - 1) * Qs;
            if ((layout != 0 || d.stride > 1) && ((Qs & 1) == 0 || (q_last & 1) == 0)) continue;
            a.LW = (Qs - 1) * d.stride + d.S;
            if (n_strips == 1) a.LW = std::max(a.LW, d.W + 2 * pad_w);
            // (rows with an odd number of pixel pairs are shared out whole: even bands)
            auto rows_whole = [](int q) { return (q % 2 == 0) && ((q / 2) % 2 == 1); };
            const bool by_rows = rows_whole(Qs) || rows_whole(q_last);
            for (TR = std::min(NP, 64); TR >= 1; --TR) {
                if (by_rows && TR > 1 && (TR & 1)) continue;
                const int LR = max_band_rows(d.N, f.P, TR, a.Hs, d.stride, d.R);
                a.LRW = LR * a.LW;
                a.PLS_in = ceil_div(a.LRW, 64) * 64 + 1;
                a.PLS_out = ceil_div(TR * Qs + 1, 64) * 64 + 1;  // the band and one zero pixel
                lds = 2 * ((size_t)NPI * a.PLS_in + (size_t)NPO * a.PLS_out) * 16;
                if (lds <= (size_t)kMaxLds) break;
            }
            if (TR >= 1) break;
        }
        }
        // (strided: bands of a single output row lose to the four-wave kernel)
        if (d.stride > 1 && TR < 2) TR = 0;
        const size_t xch = upd_f32_bands_exchange_bytes(d.R, d.S, layout);
        a.Q = Qs;
        // (the band kernel addresses both tensors with 32-bit byte offsets)
        if (TR >= 1 && (double)(d.N + 1) * a.Hs < 4.0e6 && a.LRW < (1 << 22) &&
            (double)f.in_bytes < 4.0e9 && (double)f.out_bytes < 4.0e9) {
            a.TR = TR;
            a.n_ct = ceil_div(f.Cb, NPI);
            a.n_kt = ceil_div(f.Kb, NPO);
            const int tiles = a.n_ct * a.n_kt;
            int splits = std::max(1, 256 / tiles);
            splits = std::max(splits, ceil_div(NP * f.Q, 1 << 16));  // chains of at most 2^15 pixels
            int rps = ceil_div(ceil_div(NP, splits), TR) * TR;
            splits = ceil_div(NP, rps);
            a.rows_per_split = rps;
            a.splits = splits;
            a.sampled = 0;
            a.total = tiles * splits;
            a.per_xcd = ceil_div(a.total, 8);
            p->upd_lds = std::max(lds, xch);
            p->upd_grid = a.per_xcd * 8;
            p->upd_copies = splits * n_strips;
            p->upd_ws = (size_t)p->upd_copies * f.dwt_bytes;
            p->upd_strips = n_strips;
            p->upd_strip_w = Qs;
            p->upd_bands_layout = layout;
            p->upd_bands = true;
            p->upd_ok = true;
            return true;
        }
    }
    return false;
}

// Weight update, general four-wave kernels (any remaining filter the kernels cover).
void plan_upd_general(conv_plan *p)
{
    const conv_desc_t &d = p->d;
    const conv_info_t &f = p->info;
    const int pad_h = p->pad_h, pad_w = p->pad_w;
    const bool sampled = (d.R == 1 && d.S == 1 && pad_h == 0 && pad_w == 0);
    const bool bf16 = d.dtype == CONV_BF16;
    // General kernels.  3x3 and 1x1 in one launch; any other filter with S in {1, 3, 5, 7} as
    // one launch of the 1 x S kernel per filter row r (run with pad_h - r rows of padding,
    // writing taps [r*S, (r+1)*S) of the partial copies).
    // filter rows one launch serves: all of them for 3x3 and the one-column filters
    const bool whole = (d.R == 3 && d.S == 3) || (d.S == 1 && (d.R == 3 || d.R == 7));
    const int kR = whole ? d.R : 1;
    UpdVariant v{};
    if (d.R == 1 && d.S == 1)
        v = bf16 ? UpdVariant{CONV_BF16, 1, 1, 2, 2, 2, 2, 8, 8}
                 : UpdVariant{CONV_F32, 1, 1, 2, 2, f.Cp > 64 ? 2 : 1, f.Kp > 64 ? 2 : 1, 4, 4};
    else if (whole || d.S == 1 || d.S == 3 || d.S == 5 || d.S == 7)
        v = bf16 ? UpdVariant{CONV_BF16, kR, d.S, 2, 2, 1, 2, 8, 8}
                 : UpdVariant{CONV_F32, kR, d.S, 2, 2, 1, 1, 1, 4};
    else
        return;
    if (kR == 1 && d.S == 1 && d.R > 1)  // (other one-column filters: the 1x1 kernel per row)
        v = bf16 ? UpdVariant{CONV_BF16, 1, 1, 2, 2, 2, 2, 8, 8}
                 : UpdVariant{CONV_F32, 1, 1, 2, 2, f.Cp > 64 ? 2 : 1, f.Kp > 64 ? 2 : 1, 4, 4};
    if (!upd_variant_exists(v)) return;
    p->upd_row_launches = kR == d.R ? 1 : d.R;
    const int V = f.vlen;
    const int TC = v.wc * v.fc * 32, TK = v.wk * v.fk * 32, NPI = TC / V, NPO = TK / V, NT = 256;
    // fp32 pairs pixels along a row (row pitch rounded up to even, zero padded);
    // bf16 walks the band's pixels linearly in steps of 16.
    // (1x1 without padding: both bands are flat pixel lists, no row padding needed,
    // but a band must hold an even number of pixels)
    // A row wider than a band can hold is cut into strips of Qs output columns, one launch
    // (and one set of partial copies) per strip.
    int Qs = f.Q, Qp = 0, n_strips = 1;
    const int NP = d.N * f.P;
    // staged pixels a band may hold (see the staging maps of the two kernels)
    const int max_px_in = bf16 ? v.ppt_in * NT / NPI : NT / v.ppt_in;
    const int max_px_out = bf16 ? v.ppt_out * NT / NPO : NT / v.ppt_out;
    // fp32 tiles are kept below half of the LDS so that two workgroups share a CU
    const size_t lds_cap = bf16 ? (size_t)kMaxLds : (size_t)kMaxLds / 2;
    int TR = 0, Hs = 0, LW = 0, LR = 0, npxO = 0;
    for (n_strips = 1; TR < 1; ++n_strips) {
        if (n_strips > f.Q) return;
        Qs = ceil_div(f.Q, n_strips);
        if (ceil_div(f.Q, Qs) != n_strips) continue;
        const int q_last = f.Q - (n_strips - 1) * Qs;  // width of the last strip
        Qp = (bf16 || sampled) ? Qs : ((Qs + 1) & ~1);
        for (TR = std::min(NP, std::max(1, max_px_out / Qp)); TR >= 1; --TR) {
            if (sampled) { Hs = f.P; LW = Qp; LR = TR; }
            else {
                Hs = (f.P - 1) * d.stride + kR;
                LW = (Qp - 1) * d.stride + d.S;
                if (n_strips == 1) LW = std::max(LW, d.W + 2 * pad_w);
                LR = max_band_rows(d.N, f.P, TR, Hs, d.stride, kR);
            }
            if (!bf16 && sampled && TR > 1 && ((TR * Qp) % 2 != 0 || (TR * q_last) % 2 != 0)) continue;
            npxO = bf16 ? ceil_div(TR * Qp, 16) * 16 : TR * Qp;
            const size_t lds_est = ((size_t)NPI * (LR * LW + 16) + (size_t)NPO * (npxO + 16)) * 16;
            if (LR * LW <= max_px_in && npxO <= max_px_out && lds_est <= lds_cap) break;
        }
        if (TR >= 1) break;
    }
    p->upd_strips = n_strips;
    p->upd_strip_w = Qs;
    UpdArgs &a = p->ua;
    memset(&a, 0, sizeof(a));
    a.N = d.N; a.Cb = f.Cb; a.H = d.H; a.W = d.W; a.Kb = f.Kb; a.Kp = f.Kp; a.P = f.P; a.Q = Qs;
    a.R = kR; a.S = d.S; a.stride = d.stride; a.pad = pad_h; a.pad_w = pad_w;
    a.tap0 = 0; a.ntaps_all = d.R * d.S;
    a.q0 = 0; a.Qpitch = f.Q; a.copy0 = 0;
    a.TR = TR;
    a.n_ct = ceil_div(f.Cb, NPI);
    a.n_kt = ceil_div(f.Kb, NPO);
    const int tiles = a.n_ct * a.n_kt;
    // two rounds of two workgroups per CU (measured better than one round: the tail is
    // shorter), and no accumulation
    // chain longer than about 2^15 pixels
    const int target = 1024;
    int splits = std::max(1, (target + tiles / 2) / tiles);
    splits = std::max(splits, ceil_div(NP * f.Q, 1 << 15));
    int rps = ceil_div(ceil_div(NP, splits), TR) * TR;
    splits = ceil_div(NP, rps);
    a.rows_per_split = rps;
    a.splits = splits;
    a.Hs = Hs; a.LW = LW; a.LRW = LR * LW; a.Qp = Qp;
    if (bf16) {
        // plane pitch = 8 (mod 16) pixels: the two channel planes a 16-lane
        // transposing read touches sit half an LDS row apart
        a.PLS_in = ((a.LRW + 15) / 16) * 16 + 8;
        a.PLS_out = ((npxO + 15) / 16) * 16 + 8;
    } else {
        // plane pitch = 1 (mod 8) pixels: the 8 channel blocks a 32-lane group
        // reads land in different LDS banks
        a.PLS_in = ((a.LRW + 7) / 8) * 8 + 1;
        a.PLS_out = ((npxO + 7) / 8) * 8 + 1;
    }
    a.sampled = sampled ? 1 : 0;
    a.total = tiles * splits;
    a.per_xcd = ceil_div(a.total, 8);
    p->uv = v;
    p->upd_lds = ((size_t)NPI * a.PLS_in + (size_t)NPO * a.PLS_out) * 16;
    if (p->upd_lds > (size_t)kMaxLds) return;
    // the kernels divide linear row indices through a float reciprocal, exact below 2^22
    if ((double)(d.N + 1) * std::max(a.Hs, f.P) >= 4.0e6) return;
    p->upd_grid = a.per_xcd * 8;
    p->upd_copies = splits * n_strips;
    p->upd_ws = (size_t)splits * n_strips * f.dwt_bytes;
    p->upd_ok = true;
}

void plan_upd(conv_plan *p)
{
    p->upd_ok = false;
    p->upd_ws = 0;
    p->upd_row_launches = 1;
    p->upd_strips = 1;
    p->upd_c4 = false;
    p->upd_c4_bf16 = false;
    p->upd_flat = false;
    p->upd_flat_bf16 = false;
    p->upd_rows = false;
    p->upd_bands = false;
    // the kernels written for a family of layers first, each declining what it does not fit
    if (!(plan_upd_c4_bf16(p) || plan_upd_c4(p) || plan_upd_flat_f32(p) || plan_upd_flat_bf16(p) ||
          plan_upd_rows(p) || plan_upd_bands(p)))
        plan_upd_general(p);
    // Partial copies that dwarf the tensors themselves (very wide rows cut into many strips,
    // under a filter with thousands of channels): no tiled plan; the direct kernel needs no
    // workspace.
    const double cap = std::max(2.0 * ((double)p->info.in_bytes + (double)p->info.out_bytes), 8.0e9);
    if (p->upd_ok && (double)p->upd_ws > cap) {
        p->upd_ok = false;
        p->upd_ws = 0;
    }
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" {

const char *conv_status_str(conv_status_t s)
{
    switch (s) {
        case CONV_OK: return "ok";
        case CONV_EINVAL: return "invalid argument";
        case CONV_EUNSUPPORTED: return "unsupported problem";
        case CONV_EWORKSPACE: return "workspace missing or too small";
        case CONV_ELAUNCH: return "kernel launch failed";
        case CONV_ESCRATCH: return "problem needs more scratch than the library's static buffer holds";
    }
    return "unknown status";
}

conv_status_t conv_create(const conv_desc_t *desc, conv_handle_t *out)
{
    if (!desc) return CONV_EINVAL;
    return conv_create_rect(desc, desc->pad, desc->pad, out);
}

namespace {
bool all_tiled(const conv_plan *q) { return q->fwd.ok && q->bwd_mode != 0 && q->upd_ok; }
conv_status_t create_plan(const conv_desc_t *desc, int32_t pad_h, int32_t pad_w, int32_t max_images,
                          conv_handle_t *out);
}  // namespace

conv_status_t conv_create_rect(const conv_desc_t *desc, int32_t pad_h, int32_t pad_w, conv_handle_t *out)
{
    return create_plan(desc, pad_h, pad_w, 0, out);
}

conv_status_t conv_create_chunked(const conv_desc_t *desc, int32_t pad_h, int32_t pad_w,
                                  int32_t max_images, conv_handle_t *out)
{
    if (max_images < 1) return CONV_EINVAL;
    return create_plan(desc, pad_h, pad_w, max_images, out);
}

namespace {
// max_images: > 0: no launch covers more images; 0: chunks only where the tensors need them;
// < 0: never (the plan of a chunk)
conv_status_t create_plan(const conv_desc_t *desc, int32_t pad_h, int32_t pad_w, int32_t max_images,
                          conv_handle_t *out)
{
    if (!desc || !out) return CONV_EINVAL;
    *out = nullptr;
    const conv_desc_t &d = *desc;
    if (d.N < 1 || d.C < 1 || d.K < 1 || d.H < 1 || d.W < 1 || d.R < 1 || d.S < 1 || d.stride < 1 ||
        pad_h < 0 || pad_w < 0)
        return CONV_EINVAL;
    if (d.dtype != CONV_F32 && d.dtype != CONV_BF16) return CONV_EINVAL;
    // Everything below this point is computed in int; the extents are bounded here, in
    // 64-bit, so that no later product or sum can leave the range.
    const long long Hp = (long long)d.H + 2LL * pad_h, Wp = (long long)d.W + 2LL * pad_w;
    if (Hp < d.R || Wp < d.S) return CONV_EINVAL;
    const int kMaxExtent = 1 << 24, kMaxSmall = 1 << 16;
    if (d.N > kMaxExtent || d.C > kMaxExtent || d.K > kMaxExtent || d.H > kMaxExtent ||
        d.W > kMaxExtent || d.R > kMaxSmall || d.S > kMaxSmall || d.stride > kMaxSmall ||
        pad_h > kMaxSmall || pad_w > kMaxSmall)
        return CONV_EUNSUPPORTED;
    {
        const int V = vlen_of(d.dtype);
        const double Cp = (double)ceil_div(d.C, V) * V, Kp = (double)ceil_div(d.K, V) * V;
        const double P = (double)((Hp - d.R) / d.stride + 1), Q = (double)((Wp - d.S) / d.stride + 1);
        const double kMaxElems = 549755813888.0;  // 2^39 elements per activation tensor
        if ((double)d.N * Cp * d.H * d.W > kMaxElems || (double)d.N * Kp * P * Q > kMaxElems ||
            Cp * Kp * d.R * d.S > 2147483647.0)
            return CONV_EUNSUPPORTED;
    }

    conv_plan *p = new (std::nothrow) conv_plan();
    if (!p) return CONV_EINVAL;
    p->d = d;
    p->d.pad = pad_h;
    p->pad_h = pad_h;
    p->pad_w = pad_w;
    conv_info_t &f = p->info;
    memset(&f, 0, sizeof(f));
    f.P = (d.H + 2 * pad_h - d.R) / d.stride + 1;
    f.Q = (d.W + 2 * pad_w - d.S) / d.stride + 1;
    f.vlen = vlen_of(d.dtype);
    f.Cb = ceil_div(d.C, f.vlen);
    f.Kb = ceil_div(d.K, f.vlen);
    f.Cp = f.Cb * f.vlen;
    f.Kp = f.Kb * f.vlen;
    const size_t es = esize_of(d.dtype);
    f.in_bytes = (size_t)d.N * f.Cp * d.H * d.W * es;
    f.out_bytes = (size_t)d.N * f.Kp * f.P * f.Q * es;
    f.wt_bytes = (size_t)f.Cp * d.R * d.S * f.Kp * es;
    f.dwt_bytes = (size_t)f.Cp * d.R * d.S * f.Kp * sizeof(float);

    // The tiled planners index rows, staged tiles and channel blocks with int products; they
    // are only asked where those stay far inside the range (the kernels' own limits -- exact
    // float reciprocals below 2^22, 24-bit multiplies -- are tighter still and checked by each
    // planner).  Anything else runs on the untiled kernels, or in chunks of the minibatch.
    const bool tiled_domain = (long long)(d.N + 1) * std::max<long long>(Hp, f.P) < (1LL << 24) &&
                              Wp < (1 << 15) && f.Cp < (1 << 20) && f.Kp < (1 << 20) &&
                              d.R <= 64 && d.S <= 64 && d.stride <= 64;
    p->fwd_ws = 0;
    if (tiled_domain) {
        p->fwd = plan_igemm(d.dtype, d.N, f.Cb, d.H, d.W, f.Kp, f.P, f.Q, d.R, d.S, d.stride, pad_h,
                            pad_w, f.P, f.Q, 1, 0, 0, 0);
        // Few tiles and a long reduction (small minibatch, inference): split the reduction
        // over more workgroups, fp32 partial results in the workspace, summed in a fixed order.
        if (p->fwd.ok && p->fwd.a.total <= 128 && p->fwd.a.n_stage >= 4) {
            IgemmArgs &a = p->fwd.a;
            const int want = std::min(a.n_stage / 2, std::max(1, 512 / a.total));
            if (want >= 2) {
                a.st_per = ceil_div(a.n_stage, want);
                a.ksplit = ceil_div(a.n_stage, a.st_per);
                a.per_xcd = ceil_div(a.total * a.ksplit, 8);
                p->fwd.grid = a.per_xcd * 8;
                p->fwd_ws = (size_t)a.ksplit * d.N * f.Kp * f.P * f.Q * sizeof(float);
            }
        }
        // A first layer (one channel block in, one reduction step, one channel tile): resident
        // workgroups that keep the filter in LDS and prefetch the next input tile.
        // (CONVMI_STEM=0 keeps one workgroup per tile: a tuning aid.)
        p->fwd.a.live_ch = f.Cb == 1 ? std::min(d.C, vlen_of(d.dtype)) : vlen_of(d.dtype);
        p->fwd_stem_lds = 0;
        if (p->fwd.ok) {
            const char *env = getenv("CONVMI_STEM");
            const size_t need = igemm_stem_lds(p->fwd.v, p->fwd.a);
            if (need > 0 && need <= (size_t)kMaxLds && !(env && atoi(env) == 0)) p->fwd_stem_lds = need;
            // (CONVMI_STEM_WG=n: at most n workgroups per XCD, so that small inputs too give a
            // workgroup several tiles to walk: for tests of that path)
            if (const char *cap = getenv("CONVMI_STEM_WG"); cap && atoi(cap) > 0) p->fwd.a.jstep = atoi(cap);
        }
        plan_bwd(p);
        plan_upd(p);
    }
    // A pass without a tiled plan falls to the direct kernels (any filter, stride and pad).
    if (direct_fits(d.dtype, d.N, f.Cb, f.Kb, d.H, d.W, f.P, f.Q, d.R, d.S)) {
        p->fwd_direct = !p->fwd.ok;
        p->bwd_direct = p->bwd_mode == 0;
        p->upd_direct = !p->upd_ok;
        DirectArgs &a = p->da;
        a = DirectArgs{};
        a.N = d.N; a.Cb = f.Cb; a.Kb = f.Kb; a.H = d.H; a.W = d.W; a.P = f.P; a.Q = f.Q;
        a.R = d.R; a.S = d.S; a.stride = d.stride; a.pad_h = pad_h; a.pad_w = pad_w;
        if (p->fwd_direct) p->fwd_ws = 0;
        if (p->bwd_direct) p->bwd_ws = 0;
        if (p->upd_direct) {
            p->upd_ws = 0;
            p->upd_copies = 1;  // dW is written once, by the kernel itself
        }
    }
    f.upd_splits = (p->upd_ok || p->upd_direct) ? p->upd_copies : 0;
    f.workspace_bytes = std::max(std::max(p->bwd_ws, p->upd_ws), p->fwd_ws);

    // Chunks of the minibatch.  On request: every pass.  Otherwise only for tensors of 4 GB
    // and more, which the tiled kernels' 32-bit byte offsets do not reach, or minibatches
    // whose linear row indices pass the kernels' exact-division range: the fewest equal
    // chunks whose plans are all tiled, for the passes that would else run untiled.
    int nc = 0;
    const bool forced = max_images > 0;
    if (forced) {
        if (max_images < d.N) nc = max_images;
    } else if (max_images == 0 && d.N >= 2 && !all_tiled(p) &&
               ((double)std::max(f.in_bytes, f.out_bytes) >= 4.0e9 ||
                (double)(d.N + 1) * std::max(d.H + 2 * pad_h, f.P) * std::max(f.Cb, f.Kb) >= 4.0e6)) {
        // (if one image alone has no tiled plan, no chunk has)
        conv_desc_t d1 = d;
        d1.N = 1;
        conv_handle_t q1 = nullptr;
        const bool any = create_plan(&d1, pad_h, pad_w, -1, &q1) == CONV_OK && all_tiled(q1);
        delete q1;
        for (int k = 2; any && k <= 64 && k <= d.N && nc == 0; ++k) {
            conv_desc_t dd = d;
            dd.N = ceil_div(d.N, k);
            conv_handle_t q = nullptr;
            if (create_plan(&dd, pad_h, pad_w, -1, &q) != CONV_OK) break;
            if (all_tiled(q)) nc = dd.N;
            delete q;
        }
    }
    if (nc > 0) {
        conv_desc_t dd = d;
        dd.N = nc;
        const int n_chunks = ceil_div(d.N, nc), rest = d.N - (n_chunks - 1) * nc;
        conv_status_t st = create_plan(&dd, pad_h, pad_w, -1, &p->chunk);
        if (st == CONV_OK && rest != nc) {
            dd.N = rest;
            st = create_plan(&dd, pad_h, pad_w, -1, &p->tail);
        }
        if (st != CONV_OK) {
            delete p;
            return st;
        }
        p->n_chunks = n_chunks;
        p->chunk_n = nc;
        p->fwd_chunked = forced || !p->fwd.ok;
        p->bwd_chunked = forced || p->bwd_mode == 0;
        p->upd_chunked = forced || !p->upd_ok;
        if (p->fwd_chunked) p->fwd_direct = false, p->fwd_ws = 0;
        if (p->bwd_chunked) p->bwd_direct = false, p->bwd_ws = 0;
        if (p->upd_chunked) p->upd_direct = false, p->upd_ws = 0;
        const size_t sub = std::max(p->chunk->info.workspace_bytes,
                                    p->tail ? p->tail->info.workspace_bytes : (size_t)0);
        p->chunk_ws = (sub + 255) / 256 * 256;
        const size_t need = p->chunk_ws + (p->upd_chunked ? (size_t)n_chunks * f.dwt_bytes : 0);
        if (p->upd_chunked) f.upd_splits = n_chunks;  // one dW per chunk, summed in chunk order
        f.workspace_bytes = std::max(f.workspace_bytes, need);
    }
    *out = p;
    return CONV_OK;
}
}  // namespace

conv_status_t conv_destroy(conv_handle_t h)
{
    if (!h) return CONV_EINVAL;
    delete h;
    return CONV_OK;
}

conv_status_t conv_query(conv_handle_t h, conv_info_t *info)
{
    if (!h || !info) return CONV_EINVAL;
    *info = h->info;
    return CONV_OK;
}

conv_status_t conv_fwd_fused(conv_handle_t h, const void *in, const void *wt, void *out,
                             const float *bias, const void *residual, int32_t relu, void *ws,
                             void *stream)
{
    return conv_fwd_fused_norm(h, in, wt, out, nullptr, bias, residual, relu, ws, stream);
}

conv_status_t conv_fwd_fused_norm(conv_handle_t h, const void *in, const void *wt, void *out,
                                  const float *scale, const float *bias, const void *residual,
                                  int32_t relu, void *ws, void *stream)
{
    if (!h || !in || !wt || !out) return CONV_EINVAL;
    if (!aligned16(in) || !aligned16(wt) || !aligned16(out) || !aligned16(ws) || !aligned16(bias) ||
        !aligned16(residual) || !aligned16(scale))
        return CONV_EINVAL;
    if (h->fwd_chunked) {
        const size_t in_img = h->info.in_bytes / h->d.N, out_img = h->info.out_bytes / h->d.N;
        for (int c = 0; c < h->n_chunks; ++c) {
            conv_plan *q = (c == h->n_chunks - 1 && h->tail) ? h->tail : h->chunk;
            const size_t n0 = (size_t)c * h->chunk_n;
            const conv_status_t st = conv_fwd_fused_norm(
                q, static_cast<const char *>(in) + n0 * in_img, wt, static_cast<char *>(out) + n0 * out_img,
                scale, bias, residual ? static_cast<const char *>(residual) + n0 * out_img : nullptr, relu,
                ws, stream);
            if (st != CONV_OK) return st;
        }
        return CONV_OK;
    }
    if (h->fwd_direct) {
        DirectArgs a = h->da;
        a.x = in;
        a.wt = wt;
        a.y = out;
        a.scale = scale;
        a.bias = bias;
        a.resid = residual;
        a.relu = relu != 0;
        return launch_direct_fwd(h->d.dtype, a, (hipStream_t)stream) == hipSuccess ? CONV_OK : CONV_ELAUNCH;
    }
    if (!h->fwd.ok) return CONV_EUNSUPPORTED;
    IgemmArgs a = h->fwd.a;
    const bool split = a.ksplit > 1;
    if (split && !ws) return CONV_EWORKSPACE;
    a.in = in;
    a.wt = wt;
    a.out = split ? ws : out;
    // a split reduction applies the operators where the partial results are summed
    a.scale = split ? nullptr : scale;
    a.bias = split ? nullptr : bias;
    a.resid = split ? nullptr : residual;
    a.relu = split ? 0 : (relu != 0);
    hipError_t e;
    // (bf16 with fused operators: the resident-filter kernel's phases are a few microseconds
    // long there, and the residual's round trips do not fit into them -- 0.49 ms against 0.38
    // on the general kernel for layer 1 of Table I; in fp32 it is 0.64 against 0.89)
    const bool fused_ops = scale || bias || residual || relu;
    if (h->fwd_stem_lds && !(fused_ops && h->d.dtype == CONV_BF16))
        e = launch_igemm_stem(h->fwd.v, a, h->fwd_stem_lds, (hipStream_t)stream);
    else
        e = launch_igemm(h->fwd.v, a, h->fwd.lds, h->fwd.grid, (hipStream_t)stream);
    if (e == hipSuccess && split)
        e = launch_split_reduce(h->d.dtype, static_cast<const float *>(ws), out,
                                (size_t)h->d.N * h->info.Kp * h->info.P * h->info.Q, a.ksplit, scale,
                                bias, residual, relu != 0, h->info.P * h->info.Q, h->info.Kb,
                                (hipStream_t)stream);
    return e == hipSuccess ? CONV_OK : CONV_ELAUNCH;
}

conv_status_t conv_fwd(conv_handle_t h, const void *in, const void *wt, void *out, void *ws,
                       void *stream)
{
    return conv_fwd_fused(h, in, wt, out, nullptr, nullptr, 0, ws, stream);
}

conv_status_t conv_bwd_data(conv_handle_t h, const void *dout, const void *wt, void *din, void *ws,
                            void *stream)
{
    if (!h || !dout || !wt || !din) return CONV_EINVAL;
    if (!aligned16(dout) || !aligned16(wt) || !aligned16(din) || !aligned16(ws)) return CONV_EINVAL;
    if (h->bwd_chunked) {
        const size_t in_img = h->info.in_bytes / h->d.N, out_img = h->info.out_bytes / h->d.N;
        for (int c = 0; c < h->n_chunks; ++c) {
            conv_plan *q = (c == h->n_chunks - 1 && h->tail) ? h->tail : h->chunk;
            const size_t n0 = (size_t)c * h->chunk_n;
            const conv_status_t st =
                conv_bwd_data(q, static_cast<const char *>(dout) + n0 * out_img, wt,
                              static_cast<char *>(din) + n0 * in_img, ws, stream);
            if (st != CONV_OK) return st;
        }
        return CONV_OK;
    }
    if (h->bwd_direct) {
        DirectArgs a = h->da;
        a.x = dout;
        a.wt = wt;
        a.y = din;
        return launch_direct_bwd(h->d.dtype, a, (hipStream_t)stream) == hipSuccess ? CONV_OK : CONV_ELAUNCH;
    }
    if (h->bwd_mode == 0) return CONV_EUNSUPPORTED;
    if (!ws) return CONV_EWORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    for (int i = 0; i < h->n_bwd; ++i) {
        const BwdClass &b = h->bwd[i];
        void *wt2 = static_cast<char *>(ws) + b.ws_off;
        if (b.merged) {
            WtMergeArgs m = b.m;
            m.src = wt;
            m.dst = wt2;
            if (launch_wt_merge(h->d.dtype, m, s) != hipSuccess) return CONV_ELAUNCH;
        } else {
            WtXformArgs x = b.x;
            x.src = wt;
            x.dst = wt2;
            if (launch_wt_xform(h->d.dtype, x, s) != hipSuccess) return CONV_ELAUNCH;
        }
        IgemmArgs a = b.p.a;
        a.in = dout;
        a.wt = wt2;
        a.out = din;
        if (launch_igemm(b.p.v, a, b.p.lds, b.p.grid, s) != hipSuccess) return CONV_ELAUNCH;
    }
    return CONV_OK;
}

conv_status_t conv_upd(conv_handle_t h, const void *in, const void *dout, void *dwt, void *ws,
                       void *stream)
{
    if (!h || !in || !dout || !dwt) return CONV_EINVAL;
    if (!aligned16(in) || !aligned16(dout) || !aligned16(dwt) || !aligned16(ws)) return CONV_EINVAL;
    if (h->upd_chunked) {
        // dW of chunk c goes to slot c behind the chunks' own workspace; the slots are then
        // summed in chunk order
        if (!ws) return CONV_EWORKSPACE;
        const size_t in_img = h->info.in_bytes / h->d.N, out_img = h->info.out_bytes / h->d.N;
        char *slots = static_cast<char *>(ws) + h->chunk_ws;
        for (int c = 0; c < h->n_chunks; ++c) {
            conv_plan *q = (c == h->n_chunks - 1 && h->tail) ? h->tail : h->chunk;
            const size_t n0 = (size_t)c * h->chunk_n;
            const conv_status_t st =
                conv_upd(q, static_cast<const char *>(in) + n0 * in_img,
                         static_cast<const char *>(dout) + n0 * out_img,
                         slots + (size_t)c * h->info.dwt_bytes, ws, stream);
            if (st != CONV_OK) return st;
        }
        if (launch_upd_reduce(reinterpret_cast<const float *>(slots), static_cast<float *>(dwt),
                              h->info.dwt_bytes / sizeof(float), h->n_chunks,
                              (hipStream_t)stream) != hipSuccess)
            return CONV_ELAUNCH;
        return CONV_OK;
    }
    if (h->upd_direct) {
        DirectArgs a = h->da;
        a.x = in;
        a.wt = dout;
        a.y = dwt;
        return launch_direct_upd(h->d.dtype, a, (hipStream_t)stream) == hipSuccess ? CONV_OK : CONV_ELAUNCH;
    }
    if (!h->upd_ok) return CONV_EUNSUPPORTED;
    if (!ws) return CONV_EWORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    UpdArgs a = h->ua;
    a.in = in;
    a.dout = dout;
    a.partial = static_cast<float *>(ws);
    hipError_t e = hipSuccess;
    if (h->upd_flat_bf16)
        e = launch_upd_bf16_1x1(h->urv, a, h->upd_grid, s);
    else if (h->upd_flat)
        e = launch_upd_f32_1x1(h->upd_wb, h->upd_a_is_in, a, h->upd_grid, s);
    else if (h->upd_c4_bf16)
        e = launch_upd_c4_bf16(h->d.R, h->d.S, a, h->upd_lds, h->upd_grid, s);
    else if (h->upd_c4)
        e = launch_upd_c4(h->d.dtype, h->d.R, h->d.S, a, h->upd_lds, h->upd_grid, s);
    else if (h->upd_rows)
        for (int st = 0; st < h->upd_strips && e == hipSuccess; ++st) {
            a.q0 = st * h->upd_strip_w;
            a.Q = std::min(h->upd_strip_w, h->info.Q - a.q0);
            a.copy0 = st * a.splits * h->urv.wp;
            for (int r = 0; r < h->upd_row_launches && e == hipSuccess; ++r) {
                // (one launch, or filter row r of a taller filter: its taps, its share of
                // the padding)
                a.pad = h->pad_h - r;
                a.tap0 = r * h->d.S * (h->upd_row_launches > 1 ? 1 : 0);
                e = launch_upd_rows(h->urv, a, h->upd_lds, h->upd_grid, s);
            }
        }
    else if (h->upd_bands)
        for (int st = 0; st < h->upd_strips && e == hipSuccess; ++st) {
            a.q0 = st * h->upd_strip_w;
            a.Q = std::min(h->upd_strip_w, h->info.Q - a.q0);
            a.copy0 = st * a.splits;
            e = launch_upd_f32_bands(h->d.R, h->d.S, h->upd_bands_layout, a, h->upd_lds, h->upd_grid, s);
        }
    else
        for (int st = 0; st < h->upd_strips && e == hipSuccess; ++st) {
            // strip st of the output columns; a narrower last strip of a flat (unpadded
            // 1x1) band is its own row pitch
            a.q0 = st * h->upd_strip_w;
            a.Q = std::min(h->upd_strip_w, h->info.Q - a.q0);
            a.copy0 = st * a.splits;
            if (a.sampled) {
                a.Qp = a.Q;
                a.LW = a.Q;
                a.LRW = a.TR * a.Q;
            }
            for (int r = 0; r < h->upd_row_launches && e == hipSuccess; ++r) {
                // (one launch, or filter row r of a taller filter: its taps, its share of
                // the padding)
                a.pad = h->pad_h - r;
                a.tap0 = r * h->d.S * (h->upd_row_launches > 1 ? 1 : 0);
                e = launch_upd(h->uv, a, h->upd_lds, h->upd_grid, s);
            }
        }
    if (e != hipSuccess) return CONV_ELAUNCH;
    if (launch_upd_reduce(a.partial, static_cast<float *>(dwt), h->info.dwt_bytes / sizeof(float),
                          h->upd_copies, s) != hipSuccess)
        return CONV_ELAUNCH;
    return CONV_OK;
}

namespace {
// bytes of workspace a pass of this plan reads or writes
static size_t pass_ws_bytes(const conv_plan *h, int pass)
{
    const bool chunked = pass == 0 ? h->fwd_chunked : pass == 1 ? h->bwd_chunked : h->upd_chunked;
    if (chunked) {
        size_t need = h->chunk ? pass_ws_bytes(h->chunk, pass) : 0;
        if (h->tail) need = std::max(need, pass_ws_bytes(h->tail, pass));
        if (pass == 2) need = h->chunk_ws + (size_t)h->n_chunks * h->info.dwt_bytes;
        return need;
    }
    return pass == 0 ? h->fwd_ws : pass == 1 ? h->bwd_ws : h->upd_ws;
}
}  // namespace

conv_status_t conv_fwd_ws(conv_handle_t h, const void *in, const void *wt, void *out, void *ws,
                          size_t ws_bytes, void *stream)
{
    if (!h) return CONV_EINVAL;
    if (ws_bytes < pass_ws_bytes(h, 0)) return CONV_EWORKSPACE;
    return conv_fwd(h, in, wt, out, ws, stream);
}

conv_status_t conv_bwd_data_ws(conv_handle_t h, const void *dout, const void *wt, void *din,
                               void *ws, size_t ws_bytes, void *stream)
{
    if (!h) return CONV_EINVAL;
    if (ws_bytes < pass_ws_bytes(h, 1)) return CONV_EWORKSPACE;
    return conv_bwd_data(h, dout, wt, din, ws, stream);
}

conv_status_t conv_upd_ws(conv_handle_t h, const void *in, const void *dout, void *dwt, void *ws,
                          size_t ws_bytes, void *stream)
{
    if (!h) return CONV_EINVAL;
    if (ws_bytes < pass_ws_bytes(h, 2)) return CONV_EWORKSPACE;
    return conv_upd(h, in, dout, dwt, ws, stream);
}

// ---------------------------------------------------------------------------
// Backward by data for callers that cannot allocate: the transformed weights live in a
// file-scope device array instead of a caller-provided workspace.
// ---------------------------------------------------------------------------
namespace {
constexpr size_t kScratchBytes = (size_t)16 << 20;
constexpr int kMaxDevices = 64;
}  // namespace
// Every GPU the library runs on holds its own copy of this array, at its own address, until
// the process ends.  In host code the name is only a handle for hipGetSymbolAddress.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {
// Device address of `scratch` on the current device (looked up once per device), or null.
static void *scratch_of_current_device()
{
    static std::mutex mu;
    static void *ptr_of[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr_of[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        ptr_of[dev] = ptr;
    }
    return ptr_of[dev];
}
}  // namespace

conv_status_t conv_bwd_data_noalloc(conv_handle_t h, const void *dout, const void *wt, void *din,
                                    void *stream)
{
    if (!h || !dout || !wt || !din) return CONV_EINVAL;
    if (pass_ws_bytes(h, 1) > kScratchBytes) return CONV_ESCRATCH;
    void *ptr = scratch_of_current_device();
    if (!ptr) return CONV_ELAUNCH;
    return conv_bwd_data(h, dout, wt, din, ptr, stream);
}

size_t conv_noalloc_scratch_bytes(void) { return kScratchBytes; }

#define CHECK_PACK_ARGS(h, a, b)                                  \
    if (!(h) || !(a) || !(b)) return CONV_EINVAL;                 \
    if (!aligned16(a) || !aligned16(b)) return CONV_EINVAL;

conv_status_t conv_pack_in(conv_handle_t h, const void *nchw, void *blk, void *stream)
{
    CHECK_PACK_ARGS(h, nchw, blk);
    const conv_desc_t &d = h->d;
    return launch_pack_act(d.dtype, nchw, blk, d.N, d.C, d.H, d.W, (hipStream_t)stream) == hipSuccess
               ? CONV_OK : CONV_ELAUNCH;
}
conv_status_t conv_pack_out(conv_handle_t h, const void *nkpq, void *blk, void *stream)
{
    CHECK_PACK_ARGS(h, nkpq, blk);
    const conv_desc_t &d = h->d;
    return launch_pack_act(d.dtype, nkpq, blk, d.N, d.K, h->info.P, h->info.Q,
                           (hipStream_t)stream) == hipSuccess ? CONV_OK : CONV_ELAUNCH;
}
conv_status_t conv_pack_wt(conv_handle_t h, const void *kcrs, void *blk, void *stream)
{
    CHECK_PACK_ARGS(h, kcrs, blk);
    const conv_desc_t &d = h->d;
    return launch_pack_wt(d.dtype, kcrs, blk, d.K, d.C, d.R, d.S, (hipStream_t)stream) == hipSuccess
               ? CONV_OK : CONV_ELAUNCH;
}
conv_status_t conv_unpack_in(conv_handle_t h, const void *blk, void *nchw, void *stream)
{
    CHECK_PACK_ARGS(h, blk, nchw);
    const conv_desc_t &d = h->d;
    return launch_unpack_act(d.dtype, blk, nchw, d.N, d.C, d.H, d.W, (hipStream_t)stream) == hipSuccess
               ? CONV_OK : CONV_ELAUNCH;
}
conv_status_t conv_unpack_out(conv_handle_t h, const void *blk, void *nkpq, void *stream)
{
    CHECK_PACK_ARGS(h, blk, nkpq);
    const conv_desc_t &d = h->d;
    return launch_unpack_act(d.dtype, blk, nkpq, d.N, d.K, h->info.P, h->info.Q,
                             (hipStream_t)stream) == hipSuccess ? CONV_OK : CONV_ELAUNCH;
}
conv_status_t conv_unpack_wt(conv_handle_t h, const void *blk, void *kcrs, void *stream)
{
    CHECK_PACK_ARGS(h, blk, kcrs);
    const conv_desc_t &d = h->d;
    return launch_unpack_wt(d.dtype, blk, kcrs, d.K, d.C, d.R, d.S, h->info.vlen,
                            (hipStream_t)stream) == hipSuccess ? CONV_OK : CONV_ELAUNCH;
}
conv_status_t conv_unpack_dwt(conv_handle_t h, const void *blk_f32, void *kcrs_f32, void *stream)
{
    CHECK_PACK_ARGS(h, blk_f32, kcrs_f32);
    const conv_desc_t &d = h->d;
    return launch_unpack_wt(CONV_F32, blk_f32, kcrs_f32, d.K, d.C, d.R, d.S, h->info.vlen,
                            (hipStream_t)stream) == hipSuccess ? CONV_OK : CONV_ELAUNCH;
}

conv_status_t conv_describe(conv_handle_t h, int32_t pass, char *buf, size_t buflen)
{
    if (!h || !buf || buflen == 0) return CONV_EINVAL;
    buf[0] = 0;
    if ((pass == 0 && h->fwd_chunked) || (pass == 1 && h->bwd_chunked) || (pass == 2 && h->upd_chunked)) {
        const int n = snprintf(buf, buflen, "chunks=%d images=%d: ", h->n_chunks, h->chunk_n);
        if (n < 0 || (size_t)n >= buflen) return CONV_EINVAL;
        return conv_describe(h->chunk, pass, buf + n, buflen - n);
    }
    if ((pass == 0 && h->fwd_direct) || (pass == 1 && h->bwd_direct) || (pass == 2 && h->upd_direct)) {
        const DirectArgs &a = h->da;
        const int V = h->info.vlen;
        // (the kernels stride over what a capped grid of 2^22 workgroups does not reach)
        const size_t grid = std::min<size_t>(
            pass == 0   ? ((size_t)a.N * a.Kb * a.P * a.Q * V + 255) / 256
            : pass == 1 ? ((size_t)a.N * a.Cb * a.H * a.W * V + 255) / 256
                        : (size_t)a.Cb * a.R * a.S * a.Kb,
            (size_t)1 << 22);
        snprintf(buf, buflen, "direct dt=%d RS=%dx%d stride=%d threads=256 grid=%zu lds=%d launches=1",
                 (int)h->d.dtype, a.R, a.S, a.stride, grid, pass == 2 ? 4 * V * V * 4 : 0);
        return CONV_OK;
    }
    if (pass == 0 || pass == 1) {
        const IgemmPlan *p = pass == 0 ? &h->fwd : &h->bwd[0].p;
        if (pass == 1 && h->bwd_mode == 0) return CONV_EUNSUPPORTED;
        if (!p->ok) return CONV_EUNSUPPORTED;
        snprintf(buf, buflen,
                 "igemm dt=%d waves=%dx%d frags=%dx%d npl=%d nt=%d RS=%dx%d ppt=%d TR=%d TQ=%d tiles=%d "
                 "(m=%d q=%d k=%d) xcd_kgroups=%d grid=%d lds=%zu stages=%d ksplit=%d launches=%d",
                 p->v.dtype, p->v.wk, p->v.wm, p->v.fk, p->v.fm, p->v.npl, p->v.nt, p->v.r, p->v.s, p->v.ppt,
                 p->a.TR, p->a.TQ, p->a.total, p->a.n_mt, p->a.n_qt, p->a.n_kt, p->a.gk, p->grid, p->lds,
                 p->a.n_stage, p->a.ksplit, pass == 0 ? 1 : h->n_bwd);
        if (pass == 0 && h->fwd_stem_lds) {
            const size_t n = strlen(buf);
            snprintf(buf + n, buflen - n, " resident_filter_lds=%zu", h->fwd_stem_lds);
        }
        return CONV_OK;
    }
    if (pass == 2) {
        if (!h->upd_ok) return CONV_EUNSUPPORTED;
        if (h->upd_flat_bf16) {
            snprintf(buf, buflen,
                     "upd_1x1 dt=1 waves=%dx%dx%d frags=%dx%d pixels/split=%d splits=%d tiles=%dx%d "
                     "grid=%d lds=%zu",
                     h->urv.wc, h->urv.wk, h->urv.wp, h->urv.fc, h->urv.fk, h->ua.rows_per_split,
                     h->ua.splits, h->ua.n_ct, h->ua.n_kt, h->upd_grid, h->upd_lds);
            return CONV_OK;
        }
        if (h->upd_flat) {
            snprintf(buf, buflen,
                     "upd_1x1 dt=0 waves=2x%dx%d tile=256x%d (%s) pixels/split=%d splits=%d tiles=%dx%d "
                     "grid=%d lds=%zu",
                     h->upd_wb, 4 / h->upd_wb, 64 * h->upd_wb, h->upd_a_is_in ? "in x out" : "out x in",
                     h->ua.rows_per_split, h->ua.splits, h->ua.n_ct, h->ua.n_kt, h->upd_grid,
                     h->upd_lds);
            return CONV_OK;
        }
        if (h->upd_c4 || h->upd_c4_bf16) {
            snprintf(buf, buflen,
                     "upd_c4 dt=%d mfma=%s RS=%dx%d waves=2x4 TR=%d splits=%d rows/split=%d ktiles=%d grid=%d lds=%zu",
                     (int)h->d.dtype, h->upd_c4_bf16 ? "bf16" : "f32", h->d.R, h->d.S, h->ua.TR, h->ua.splits, h->ua.rows_per_split, h->ua.n_kt,
                     h->upd_grid, h->upd_lds);
            return CONV_OK;
        }
        if (h->upd_rows) {
            snprintf(buf, buflen,
                     "upd_rows dt=1 RS=%dx%d waves=%dx%dx%d frags=%dx%d TR=%d runs=%d splits=%d "
                     "rows/split=%d tiles=%dx%d grid=%d lds=%zu launches=%d",
                     h->d.R, h->d.S, h->urv.wc, h->urv.wk, h->urv.wp, h->urv.fc, h->urv.fk, h->ua.TR,
                     h->ua.runs, h->ua.splits, h->ua.rows_per_split, h->ua.n_ct, h->ua.n_kt,
                     h->upd_grid, h->upd_lds, h->upd_strips * h->upd_row_launches);
            return CONV_OK;
        }
        if (h->upd_bands) {
            snprintf(buf, buflen,
                     "upd_bands dt=0 RS=%dx%d waves=%s frags=1x1 TR=%d splits=%d rows/split=%d "
                     "tiles=%dx%d grid=%d lds=%zu launches=%d",
                     h->d.R, h->d.S,
                     h->upd_bands_layout == 0 ? "2x2x2" : h->upd_bands_layout == 1 ? "1x2x4" : "1x1x8",
                     h->ua.TR, h->ua.splits, h->ua.rows_per_split, h->ua.n_ct,
                     h->ua.n_kt, h->upd_grid, h->upd_lds, h->upd_strips);
            return CONV_OK;
        }
        snprintf(buf, buflen,
                 "upd dt=%d RS=%dx%d waves=%dx%d frags=%dx%d TR=%d splits=%d rows/split=%d "
                 "tiles=%dx%d grid=%d lds=%zu launches=%d",
                 h->uv.dtype, h->uv.r, h->uv.s, h->uv.wc, h->uv.wk, h->uv.fc, h->uv.fk, h->ua.TR,
                 h->ua.splits, h->ua.rows_per_split, h->ua.n_ct, h->ua.n_kt, h->upd_grid,
                 h->upd_lds, h->upd_row_launches * h->upd_strips);
        return CONV_OK;
    }
    return CONV_EINVAL;
}

}  // extern "C"
