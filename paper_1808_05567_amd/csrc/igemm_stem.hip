// Forward pass of a first layer: ONE input channel block (three colour channels padded to a
// block), a tall filter, at most one tile of output channels -- the whole reduction of a
// tile is a single staged step of R*S taps (Algorithm 1 with C_b = 1; Section II-B keeps the
// blocked layout for it, Section II-H replays a fixed stream of microkernel calls).
//
// The general kernel gives such a layer one workgroup per tile: it stages the filter and the
// input tile, waits, computes, stores, and ends, and with the filter (R*S x 64 rows) and the
// tall input tile both in LDS only one workgroup fits a CU, so nothing overlaps anything.
// Here a workgroup is resident for the whole launch and walks its share of the tiles:
//   * the filter is staged ONCE per workgroup and stays in LDS (it is the same for every
//     tile: one channel block in, one channel tile out);
//   * its eight waves are two groups of four with an input buffer each, and the groups take
//     turns: while one runs the MFMAs of a tile, the other stores its results of the tile
//     before, forms the addresses of its next tile and stages it.  Only the MFMA phases
//     are left on the critical path; with four waves all of that is serial, and in bf16 the
//     MFMAs are the smaller part of a tile's time.
// Per tile that halves the bytes pulled into LDS and takes the load latency off the path.
//
//   * with stride 2 a staged row is kept de-interleaved, its even columns first, then its odd
//     ones: the 32 lanes of an MFMA operand read, which take 32 consecutive RESULT columns
//     of one tap, then read 32 consecutive 16-byte chunks instead of every other one (a
//     two-way bank conflict on every such read, and these layers are bound by LDS reads
//     in bf16).
//
// Tile geometry, MFMA operand layout and the store are those of the general kernel's
// one-plane path (same IgemmArgs, same order of the sum: results are bit-identical).
#include <algorithm>
#include <map>
#include <mutex>
#include <tuple>

#include "igemm_kernel.h"

namespace convmi {

template <int DT, int WK, int WM, int FK, int FM, int R, int S, int PPT, int NCH>
__global__ __launch_bounds__(512, 1) void igemm_stem_kernel(const IgemmArgs a)
{
    using E_ = Elem<DT>;
    constexpr int V = E_::V;
    static_assert(WK * WM == 4, "two groups of four waves");
    constexpr int TK = WK * FK * 32;
    constexpr int NTAPS = R * S;
    constexpr int NENT = ((NTAPS + 1) / 2) * 2;  // taps per tile, even (the filler tap is zero)
    constexpr int WCH = NENT * TK;               // 16-byte weight chunks
    constexpr int WPT = (WCH + 511) / 512;       // ... per thread, all eight waves loading
    constexpr int WBYTES = WCH * 16;

    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int ibytes = a.PLS * 16;
    unsigned char *const wb = lds;  // the filter; the two groups' input buffers follow

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave8 = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave8 >> 2;  // the wave's group
    const int wave = wave8 & 3;  // ... and its place in it
    const int h = lane >> 5;
    const int l32 = lane & 31;
    const int wave_k = wave % WK;
    const int wave_m = wave / WK;
    const int wave_chunk = wave * 64;
    unsigned char *const ib = lds + WBYTES + grp * ibytes;  // this group's input tile

    // Tiles of XCD x: pixel tiles x * mq_per + j, j = 0 .. (one channel tile).  This workgroup
    // takes j = j0, j0 + jstep, ...: `ntiles` of them, its k-th tile being tile_of(k).
    const int xcd = blockIdx.x & 7;
    const int j0 = blockIdx.x >> 3;
    const int j_end = min(a.mq_per, a.n_mt * a.n_qt - xcd * a.mq_per);
    const int ntiles = j0 < j_end ? (j_end - j0 + a.jstep - 1) / a.jstep : 0;
    if (ntiles == 0) return;  // (the whole workgroup)
    auto tile_of = [&](int k) { return xcd * a.mq_per + j0 + k * a.jstep; };

    const int NP = a.N * a.P;
    const float inv_P = a.inv_P, inv_Hs = a.inv_Hs, inv_LW = a.inv_LW, inv_TQ = a.inv_TQ;
    const size_t in_bytes = (size_t)a.N * a.H * a.W * 16;
    const rsrc_t rsrc_in = make_rsrc(a.in, 0, in_bytes);
    // (a.LW is the pitch of a staged row; with stride 2 the launch makes it even)
    const bool deint = a.stride == 2;
    const int half = a.LW >> 1;

    // Stage the input tile of pixel tile `rest` into this group's buffer (as the general
    // kernel does: 16-byte loads that write straight into LDS, out-of-range lanes are zeros).
    auto issue_input = [&](int rest) {
        const int qt = rest % a.n_qt, mt = rest / a.n_qt;
        const int q0 = qt * a.TQ, rho0 = mt * a.TR;
        const int n0 = fast_div(rho0, inv_P);
        const int lam0 = n0 * a.Hs + (rho0 - n0 * a.P) * a.stride;
#pragma unroll
        for (int i = 0; i < PPT; ++i) {
            const int c0 = min(i * 256 + wave_chunk, a.PLS - 64);
            const int p = c0 + lane;
            unsigned off = kOutOfRange;
            if (p < a.LRW) {
                const int row = fast_div(p, inv_LW);
                const int x = p - mul24(row, a.LW);
                // (stride 2: position x of a staged row holds column 2 (x mod half) + x / half)
                const int col = deint ? ((x >= half ? x - half : x) * 2 + (x >= half ? 1 : 0)) : x;
                const int lam = lam0 + row;
                const int n = fast_div(lam, inv_Hs);
                const int ih = lam - mul24(n, a.Hs) - a.pad_h;
                const int iw = q0 * a.stride - a.pad_w + col;
                if (n < a.N && ih >= 0 && ih < a.H && iw >= 0 && iw < a.W)
                    off = (unsigned)(mul24(mul24(n, a.H) + ih, a.W) + iw) * 16u;
            }
            load_to_lds_16(rsrc_in, off, 0u, ib + c0 * 16);
        }
    };

    // the filter, once, by all eight waves; group 0 also stages the first tile
    {
        const size_t wt_bytes = (size_t)NTAPS * a.Kp * 16;
        const rsrc_t rsrc_wt = make_rsrc(a.wt, 0, wt_bytes);
#pragma unroll
        for (int i = 0; i < WPT; ++i) {
            const int c0 = min(i * 512 + wave8 * 64, WCH - 64);
            const int w = c0 + lane;
            const int tap = w / TK;
            const int k = w - tap * TK;
            const unsigned off = (tap < NTAPS && k < a.Kp) ? (unsigned)(mul24(tap, a.Kp) + k) * 16u : kOutOfRange;
            load_to_lds_16(rsrc_wt, off, 0u, wb + c0 * 16);
        }
    }
    if (grp == 0) issue_input(tile_of(0));
    wait_all_memory();
    __syncthreads();

    const size_t oplane = (size_t)a.OH * a.OW * 16;
    const size_t out_bytes = (size_t)a.N * a.out_kb * oplane;
    const rsrc_t ro = make_rsrc(a.out, 0, out_bytes);
    const int a_base = (h * TK + wave_k * FK * 32 + l32) * 16;

    // The groups take turns, a barrier of the whole workgroup between the phases.  In phase ph
    // group ph mod 2 runs the MFMAs of the workgroup's tile ph out of its own buffer, while the
    // other group stages tile ph + 1 into its buffer (which it has just finished with), stores
    // its results of tile ph - 1 and waits for the loads to land.  The accumulators stay in registers
    // from a group's compute phase to its store phase.
    f32x16 acc[FK][FM];
    for (int ph = 0; ph <= ntiles; ++ph) {
        if (grp == (ph & 1)) {
            if (ph < ntiles) {
                const int rest = tile_of(ph);
                const int qt = rest % a.n_qt, mt = rest / a.n_qt;
                const int q0 = qt * a.TQ, rho0 = mt * a.TR;
                const int n0 = fast_div(rho0, inv_P);
                const int lam0 = n0 * a.Hs + (rho0 - n0 * a.P) * a.stride;
                int bpos[FM];
#pragma unroll
                for (int f = 0; f < FM; ++f) {
                    const int m = (wave_m * FM + f) * 32 + l32;
                    const int trow = fast_div(m, inv_TQ);
                    const int tcol = m - mul24(trow, a.TQ);
                    const int rho = rho0 + trow;
                    const bool ok = trow < a.TR && rho < NP && (q0 + tcol) < a.Q;
                    const int n = fast_div(rho, inv_P);
                    const int oj = rho - mul24(n, a.P);
                    const int pos = ok ? mul24(mul24(n, a.Hs) + mul24(oj, a.stride) - lam0, a.LW) +
                                             (deint ? tcol : mul24(tcol, a.stride))
                                       : 0;
                    bpos[f] = pos * 16;
                }
#pragma unroll
                for (int i = 0; i < FK; ++i)
#pragma unroll
                    for (int f = 0; f < FM; ++f)
#pragma unroll
                        for (int t = 0; t < 16; ++t) acc[i][f][t] = 0.0f;

                // One channel block: the two lane halves take two taps; the operands of tap
                // pair q+1 are read before the MFMAs of pair q issue.
                auto read_pair = [&](int q, u32x4(&af)[FK], u32x4(&bf)[FM]) {
                    const int t0 = 2 * q;
                    const int t1 = (2 * q + 1 < NTAPS) ? 2 * q + 1 : NTAPS - 1;
                    // (tap column s of a de-interleaved row: half s mod 2, position s / 2 further on)
                    const int x0 = deint ? ((t0 % S) & 1) * half + ((t0 % S) >> 1) : (t0 % S);
                    const int x1 = deint ? ((t1 % S) & 1) * half + ((t1 % S) >> 1) : (t1 % S);
                    const int off0 = ((t0 / S) * a.LW + x0) * 16;
                    const int off1 = ((t1 / S) * a.LW + x1) * 16;
                    const int toff = h ? off1 : off0;
#pragma unroll
                    for (int i = 0; i < FK; ++i)
                        af[i] = *reinterpret_cast<const u32x4 *>(wb + a_base + (2 * q * TK + 32 * i) * 16);
#pragma unroll
                    for (int f = 0; f < FM; ++f)
                        bf[f] = *reinterpret_cast<const u32x4 *>(ib + bpos[f] + toff);
                };
                u32x4 ac[FK], bc[FM];
                read_pair(0, ac, bc);
#pragma unroll
                for (int q = 0; q < NENT / 2; ++q) {
                    u32x4 an[FK], bn[FM];
                    if (q + 1 < NENT / 2) read_pair(q + 1, an, bn);
#pragma unroll
                    for (int i = 0; i < FK; ++i)
#pragma unroll
                        for (int f = 0; f < FM; ++f) E_::template mma<NCH>(ac[i], bc[f], acc[i][f]);
                    // Issue order of the round: one MFMA, then one LDS read of the next pair's
                    // operands, and so on (left to itself the compiler reads each operand
                    // right before the MFMA that takes it, and waits for it there).
                    constexpr int NMFMA = FK * FM * E_::template mfmas_per_operand<NCH>;
#pragma unroll
                    for (int k = 0; k < NMFMA; ++k) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // LDS read
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    if (q + 1 < NENT / 2) {
#pragma unroll
                        for (int i = 0; i < FK; ++i) ac[i] = an[i];
#pragma unroll
                        for (int f = 0; f < FM; ++f) bc[f] = bn[f];
                    }
                }
                // (every LDS read of this phase has returned before the barrier)
                wait_all_memory();
            }
        } else {
            // (this group read its buffer last in phase ph - 1: the barrier since then has
            // passed.  The loads go out before the stores: they have the longer way.)
            if (ph + 1 < ntiles) issue_input(tile_of(ph + 1));
            if (ph >= 1) {
                // Store tile ph - 1: per group of 8 channel rows only the scalar offset (the
                // channel block) changes.
                const int rest = tile_of(ph - 1);
                const int qt = rest % a.n_qt, mt = rest / a.n_qt;
                const int q0 = qt * a.TQ, rho0 = mt * a.TR;
                const unsigned lane_off = (V == 4) ? (unsigned)h * (unsigned)oplane : (unsigned)h * 8u;
                unsigned ooff[FM];  // byte offset of the lane's pixel (and lane half) in channel block 0
#pragma unroll
                for (int f = 0; f < FM; ++f) {
                    const int m = (wave_m * FM + f) * 32 + l32;
                    const int trow = fast_div(m, inv_TQ);
                    const int tcol = m - mul24(trow, a.TQ);
                    const int rho = rho0 + trow;
                    const bool ok = trow < a.TR && rho < NP && (q0 + tcol) < a.Q;
                    const int n = fast_div(rho, inv_P);
                    const int oj = rho - mul24(n, a.P);
                    ooff[f] = ok ? (unsigned)(mul24(mul24(mul24(n, a.out_kb), a.OH) + oj, a.OW) + q0 + tcol) * 16u +
                                       lane_off
                                 : kOutOfRange;
                }
                // L() of Algorithm 4 on the finished accumulators, as in the general kernel: scale,
                // bias, residual, ReLU.  The residual values of a row group are all requested
                // before the first store of the group (the residual may be the output itself).
                const bool fused = a.scale != nullptr || a.bias != nullptr || a.resid != nullptr || a.relu != 0;
                const rsrc_t rres = make_rsrc(a.resid ? a.resid : a.out, 0, out_bytes);
#pragma unroll
                for (int i = 0; i < FK; ++i) {
#pragma unroll
                    for (int vq = 0; vq < 4; ++vq) {
                        const int krow0 = (wave_k * FK + i) * 32 + vq * 8;  // + 4*h for this lane
                        if (krow0 >= a.Kp) continue;                       // wave-uniform
                        const unsigned skip = (unsigned)(krow0 / V) * (unsigned)oplane;
                        // (fp32: the upper lane half's block may lie beyond the last channel block)
                        const bool upper_dead = (V == 4) && krow0 + 4 >= a.Kp;  // wave-uniform
                        if (!fused) {
#pragma unroll
                            for (int f = 0; f < FM; ++f)
                                E_::template store4<CONVMI_OUT_POLICY>(
                                    ro, (upper_dead && h) ? kOutOfRange : ooff[f], skip, acc[i][f][4 * vq + 0],
                                    acc[i][f][4 * vq + 1], acc[i][f][4 * vq + 2], acc[i][f][4 * vq + 3]);
                            continue;
                        }
                        const bool rows_live = krow0 + 4 * h < a.Kp;
                        float b4[4] = {0.f, 0.f, 0.f, 0.f}, s4[4] = {1.f, 1.f, 1.f, 1.f};
                        if (a.bias && rows_live) {
                            const f32x4 b = *reinterpret_cast<const f32x4 *>(a.bias + krow0 + 4 * h);
                            b4[0] = b[0]; b4[1] = b[1]; b4[2] = b[2]; b4[3] = b[3];
                        }
                        if (a.scale && rows_live) {
                            const f32x4 g = *reinterpret_cast<const f32x4 *>(a.scale + krow0 + 4 * h);
                            s4[0] = g[0]; s4[1] = g[1]; s4[2] = g[2]; s4[3] = g[3];
                        }
                        float r4[FM][4];
#pragma unroll
                        for (int f = 0; f < FM; ++f)
#pragma unroll
                            for (int t = 0; t < 4; ++t) r4[f][t] = 0.0f;
                        if (a.resid) {
#pragma unroll
                            for (int f = 0; f < FM; ++f)
                                E_::load4(rres, rows_live ? ooff[f] : kOutOfRange, skip, r4[f]);
                        }
#pragma unroll
                        for (int f = 0; f < FM; ++f) {
                            float o4[4];
#pragma unroll
                            for (int t = 0; t < 4; ++t) {
                                o4[t] = acc[i][f][4 * vq + t] * s4[t] + r4[f][t] + b4[t];
                                if (a.relu) o4[t] = fmaxf(o4[t], 0.0f);
                            }
                            E_::template store4<CONVMI_OUT_POLICY>(ro, rows_live ? ooff[f] : kOutOfRange, skip,
                                                                   o4[0], o4[1], o4[2], o4[3]);
                        }
                    }
                }
            }
            wait_all_memory();
        }
        __syncthreads();
    }
}

namespace {

struct StemEntry {
    int dtype, wk, wm, fk, fm, r, s, ppt, nch;
    igemm_fn_t fn;
};
#define STEM_ENTRY(DT, WK, WM, FK, FM, R, S, PPT, NCH) \
    {DT, WK, WM, FK, FM, R, S, PPT, NCH, igemm_stem_kernel<DT, WK, WM, FK, FM, R, S, PPT, NCH>}
StemEntry g_stem[] = {
    // 7x7, stride 2 over 224 x 224 (112 result columns, four result rows per tile); nch: the
    // channel slots that get an MFMA of their own (fp32; three for an RGB input)
    STEM_ENTRY(CONV_F32, 2, 2, 1, 7, 7, 7, 12, 3),
    STEM_ENTRY(CONV_F32, 2, 2, 1, 7, 7, 7, 12, 4),
    STEM_ENTRY(CONV_BF16, 2, 2, 1, 7, 7, 7, 12, 8),
};

// The instantiation for variant v whose MFMAs cover `live_ch` channel slots with the fewest.
const StemEntry *find_stem(const IgemmVariant &v, int live_ch)
{
    if (v.npl != 1 || v.nb != 2) return nullptr;
    if (live_ch <= 0) live_ch = vlen_of(v.dtype);  // (not stated: all of them)
    const StemEntry *best = nullptr;
    for (const StemEntry &e : g_stem)
        if (e.dtype == v.dtype && e.wk == v.wk && e.wm == v.wm && e.fk == v.fk && e.fm == v.fm &&
            e.r == v.r && e.s == v.s && e.ppt == v.ppt && e.nch >= live_ch && (!best || e.nch < best->nch))
            best = &e;
    return best;
}

// Workgroups of `kernel` (threads, dynamic LDS) that one XCD holds at a time on the current
// device; asked of the runtime once per kernel, LDS size and device.
hipError_t resident_per_xcd(const void *kernel, int threads, size_t lds_bytes, int *out)
{
    static std::mutex mu;
    static std::map<std::tuple<int, const void *, size_t>, int> known;
    int dev = 0;
    if (hipError_t err = hipGetDevice(&dev); err != hipSuccess) return err;
    std::lock_guard<std::mutex> lock(mu);
    const auto key = std::make_tuple(dev, kernel, lds_bytes);
    auto it = known.find(key);
    if (it == known.end()) {
        int per_cu = 0, cus = 0;
        if (hipError_t err = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, lds_bytes);
            err != hipSuccess)
            return err;
        if (hipError_t err = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
            err != hipSuccess)
            return err;
        if (per_cu < 1 || cus < 8) return hipErrorInvalidConfiguration;
        it = known.emplace(key, per_cu * (cus / 8)).first;
    }
    *out = it->second;
    return hipSuccess;
}

}  // namespace

// The kernel's staged-tile geometry: the plan's, with an even row pitch where the stride is 2
// (rows are kept de-interleaved: even columns, then odd ones).
static IgemmArgs stem_geometry(const IgemmArgs &a)
{
    IgemmArgs b = a;
    if (a.stride == 2 && (a.LW & 1)) {
        const int rows = a.LRW / a.LW;
        b.LW = a.LW + 1;
        b.LRW = rows * b.LW;
        b.PLS = (b.LRW + 63) / 64 * 64;
        b.inv_LW = 1.0f / (float)b.LW;
    }
    return b;
}

// LDS the resident-filter kernel needs for plan (v, a): the filter and two input tiles; 0 if
// the plan is not one it serves (one channel block in, one reduction step, one channel tile,
// plain result geometry) or no instantiation exists.
size_t igemm_stem_lds(const IgemmVariant &v, const IgemmArgs &a)
{
    const StemEntry *e = find_stem(v, a.live_ch);
    if (!e) return 0;
    if (a.Cb != 1 || a.n_stage != 1 || a.n_kt != 1 || a.ksplit != 1 || a.sampled || a.shuffle || a.zero_fill ||
        a.ostr != 1 || a.ostr_x != 1 || a.cstride != a.stride || a.oy0 != 0 || a.ox0 != 0 || a.gk != 1 ||
        a.kt_per != 1)
        return 0;
    const int TK = v.wk * v.fk * 32;
    const int nent = ((v.r * v.s + 1) / 2) * 2;
    const IgemmArgs b = stem_geometry(a);
    if (b.PLS > v.ppt * 256) return 0;  // (the even row pitch no longer fits the loads per thread)
    return (size_t)nent * TK * 16 + 2 * (size_t)b.PLS * 16;
}

// The launch: as many workgroups as stay resident, each walking every jstep-th tile of its XCD.
hipError_t launch_igemm_stem(const IgemmVariant &v, const IgemmArgs &a, size_t lds_bytes, hipStream_t stream)
{
    const StemEntry *e = find_stem(v, a.live_ch);
    if (!e) return hipErrorInvalidDeviceFunction;
    const void *fn = reinterpret_cast<const void *>(e->fn);
    if (hipError_t err = ensure_dynamic_lds(fn, lds_bytes); err != hipSuccess) return err;
    int resident = 0;
    if (hipError_t err = resident_per_xcd(fn, 512, lds_bytes, &resident); err != hipSuccess) return err;
    IgemmArgs b = stem_geometry(a);
    b.jstep = std::min(a.mq_per, resident);
    if (a.jstep > 0) b.jstep = std::min(b.jstep, a.jstep);  // (a cap from the plan: see conv_create)
    hipLaunchKernelGGL(e->fn, dim3(8 * b.jstep), dim3(512), lds_bytes, stream, b);
    return hipGetLastError();
}

}  // namespace convmi
