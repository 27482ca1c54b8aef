// The implicit-GEMM convolution kernel template and its table-entry type, shared by
// the translation units that instantiate it (square ResNet-style filters in one,
// rectangular Inception-style filters in another, so that they compile in parallel).
#pragma once
#include <type_traits>

#include "conv_internal.h"

// Cache policy of the stores of a result that is written once, in whole 16-byte (fp32) or
// paired 8-byte (bf16) blocks, and not read again by this pass: non-temporal (measured at
// N = 256: bf16 forward passes 6 % faster in total, up to 18 % on the strided 1x1 layers).
// Scattering stores (strided backward: 8- or 16-byte pieces with zeros written in between)
// keep the default policy -- written non-temporally their partial lines reach memory one
// by one, twice as slow -- and so do the partial results of a split reduction, which the
// reduce kernel reads back at once.
#ifndef CONVMI_OUT_POLICY
#define CONVMI_OUT_POLICY 2
#endif

namespace convmi {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int DT>
struct Elem;

template <>
struct Elem<CONV_F32> {
    static constexpr int V = 4;
    static constexpr int ES = 4;
    // One 16-byte operand per lane carries 4 reduction indices; lanes 0-31 and
    // 32-63 hold different channel blocks, so four 32x32x2 MFMAs consume it.
    // NCH: channel slots of the operand's block that can be non-zero (a first layer with
    // three channels pads the fourth slot with zeros on both sides: its MFMA adds nothing).
    template <int NCH = 4>
    static __device__ __forceinline__ void mma(const u32x4 &a, const u32x4 &b, f32x16 &c)
    {
#pragma unroll
        for (int t = 0; t < NCH; ++t)
            c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[t]), __uint_as_float(b[t]),
                                                     c, 0, 0, 0);
    }
    template <int NCH>
    static constexpr int mfmas_per_operand = NCH;
    // Load 4 consecutive channels of one pixel (zeros if byte_off is out of range).
    static __device__ __forceinline__ void load4(rsrc_t r, unsigned byte_off, unsigned uniform_off,
                                                 float (&x)[4])
    {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, uniform_off, 0);
#pragma unroll
        for (int t = 0; t < 4; ++t) x[t] = __uint_as_float(v[t]);
    }
    // Store 4 consecutive channels of one pixel (dropped if byte_off is out of range).
    template <int POLICY = 0>
    static __device__ __forceinline__ void store4(rsrc_t r, unsigned byte_off, unsigned uniform_off,
                                                  float x0, float x1, float x2, float x3)
    {
        u32x4 v = {__float_as_uint(x0), __float_as_uint(x1), __float_as_uint(x2),
                   __float_as_uint(x3)};
        __builtin_amdgcn_raw_buffer_store_b128(v, r, byte_off, uniform_off, POLICY);
        // A 16-byte buffer store reads its data registers over several cycles.  The compiler
        // guards a VALU write to them right behind the store only where the store has no
        // scalar offset; with one (as here) it places the write directly behind the store,
        // and on gfx950 the first data register of the last lanes of each 16-lane group was
        // then stored with the new value (seen as sporadic wrong partial results).  Two
        // wait states pinned behind the store close the window.
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_nop 1");
        __builtin_amdgcn_sched_barrier(0);
    }
};

static __device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 p = {(__bf16)lo, (__bf16)hi};  // round to nearest even
    return __builtin_bit_cast(unsigned, p);
}

template <>
struct Elem<CONV_BF16> {
    static constexpr int V = 8;
    static constexpr int ES = 2;
    // (one MFMA takes all eight channel slots of the block, live or not)
    template <int NCH = 8>
    static __device__ __forceinline__ void mma(const u32x4 &a, const u32x4 &b, f32x16 &c)
    {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                    __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
    template <int NCH>
    static constexpr int mfmas_per_operand = 1;
    static __device__ __forceinline__ void load4(rsrc_t r, unsigned byte_off, unsigned uniform_off,
                                                 float (&x)[4])
    {
        const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(r, byte_off, uniform_off, 0);
        x[0] = __uint_as_float(v[0] << 16);
        x[1] = __uint_as_float(v[0] & 0xFFFF0000u);
        x[2] = __uint_as_float(v[1] << 16);
        x[3] = __uint_as_float(v[1] & 0xFFFF0000u);
    }
    template <int POLICY = 0>
    static __device__ __forceinline__ void store4(rsrc_t r, unsigned byte_off, unsigned uniform_off,
                                                  float x0, float x1, float x2, float x3)
    {
        u32x2 v = {pack_bf16x2(x0, x1), pack_bf16x2(x2, x3)};
        __builtin_amdgcn_raw_buffer_store_b64(v, r, byte_off, uniform_off, POLICY);
    }
};

// NB: LDS buffers of the staging ring (2 = double buffering; more = the loads run further ahead)
// NTI: 1 = the input tile is loaded non-temporally.  For plans with a single channel tile, where
// every input line is read by exactly one workgroup: such lines then leave the L2 first and
// are not kept in the last-level cache, instead of pushing out the weights and the output
// lines on their way to memory (measured at N = 256, bf16, backward pass of the 1x1 layers
// that widen the channel count: 25 - 35 % faster).
// (Register budget: two workgroups per CU for the four-wave tiles of at most 128 accumulator
// registers; a 7x7 filter alone fills most of a CU's LDS, so those run one per CU anyway.)
template <int DT, int WK, int WM, int FK, int FM, int NPL, int R, int S, int PPT, int NB = 2, int NTI = 0>
__global__ __launch_bounds__(WK *WM * 64, ((WK * WM == 4 && FK * FM * 16 <= 128 && R * S < 49) ? 2 : 1)) void igemm_kernel(const IgemmArgs a)
{
    using E_ = Elem<DT>;
    constexpr int V = E_::V;
    constexpr int NT = WK * WM * 64;
    // Four or eight waves.  Eight waves are two groups of four for the staging of the input
    // tile: each group brings in its own half of a step's channel planes, with the chunk
    // bookkeeping of a four-wave workgroup.  (Two waves per SIMD inside ONE workgroup share
    // one staged tile: half the bytes pulled into LDS per flop of two four-wave workgroups.)
    static_assert(NT == 256 || NT == 512, "four or eight waves");
    constexpr int NG = NT / 256;
    static_assert(NPL % NG == 0, "every wave group stages whole planes");
    constexpr int NPLG = NPL / NG;  // planes a wave group stages per step
    constexpr int TK = WK * FK * 32;
    constexpr int NTAPS = R * S;
    constexpr int NENT = ((NTAPS * NPL + 1) / 2) * 2;  // reduction entries per step, even
    constexpr int WCH = NENT * TK;                     // 16-byte weight chunks per step
    constexpr int WPT = (WCH + NT - 1) / NT;
    constexpr int WBYTES = WCH * 16;  // a multiple of 64 chunks: whole wave-level loads
    static_assert(NPL == 1 || NPL % 2 == 0, "planes per step: 1 or even");

    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int ibytes = NPL * a.PLS * 16;
    const int bufbytes = WBYTES + ibytes;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    // (the wave index is the same in all lanes: tell the compiler, so that everything
    // derived from it lives in scalar registers and store offsets need no per-lane loop)
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5;
    const int l32 = lane & 31;
    const int wave_k = wave % WK;
    const int wave_m = wave / WK;

    // Workgroup -> tile.  Hardware deals consecutive workgroup ids round-robin over the 8
    // XCDs, each with an L2 of its own.  The tiles are dealt to the XCDs as a grid of gk
    // channel groups x 8/gk pixel groups: an XCD works through its pixel tiles one after the
    // other, all of its channel tiles of a pixel tile side by side (the staged input tile is
    // fetched from beyond the L2 once per XCD that needs it), while its share of the weights,
    // 1/gk of them, stays resident in its L2 for the whole launch.  The planner picks gk so
    // that the bytes fetched from beyond the L2s, gk x input + (8/gk) x weights, are least.
    const int bid = blockIdx.x;
    int sp = 0, kt, rest;
    if (a.ksplit > 1) {
        // reduction split (few tiles): copy sp of tile lin % total, tiles in plain order
        const int lin = (bid & 7) * a.per_xcd + (bid >> 3);
        if (lin >= a.total * a.ksplit) return;
        sp = lin / a.total;
        const int tile = lin - sp * a.total;
        kt = tile % a.n_kt;
        rest = tile / a.n_kt;
    } else {
        const int x = bid & 7, j = bid >> 3;
        const int kg = x % a.gk, mg = x / a.gk;
        const int mql = j / a.kt_per;
        kt = kg * a.kt_per + (j - mql * a.kt_per);
        rest = mg * a.mq_per + mql;
        if (kt >= a.n_kt || mql >= a.mq_per || rest >= a.n_mt * a.n_qt) return;
    }
    const int sbeg = sp * a.st_per;                  // its first reduction step ...
    const int nst = min(a.n_stage - sbeg, a.st_per);  // ... and how many (at least one)
    const int qt = rest % a.n_qt;
    const int mt = rest / a.n_qt;
    // Workgroups that share a staged tile -- the channel tiles of one pixel tile share its input,
    // the pixel tiles of one channel tile its weights -- run side by side.  If they all walked the
    // reduction in the same order they would all ask for the same lines at the same moment and
    // all wait for the one fetch from beyond the L2; started at different steps, one of them
    // fetches a line and the others find it resident.  (The order of a sum changes with the
    // tile, not from run to run.)
    const int rot = (int)(((unsigned)kt * (unsigned)a.rot_k + (unsigned)rest * (unsigned)a.rot_m) % (unsigned)nst);
    const int k0 = kt * TK;
    const int q0 = qt * a.TQ;
    const int rho0 = mt * a.TR;
    const int NP = a.N * a.P;
    const float inv_P = a.inv_P, inv_Hs = a.inv_Hs, inv_LW = a.inv_LW, inv_TQ = a.inv_TQ;
    const int n0 = fast_div(rho0, inv_P);
    const int lam0 = n0 * a.Hs + (rho0 - n0 * a.P) * a.stride;
    const int HW = a.H * a.W;

    // Staging: 16-byte buffer loads that write straight into LDS (lane i of a
    // wave lands at base + 16*i), so no registers, VALU work or LDS-write
    // instructions are spent on it.  Padding (outside the image, beyond the
    // channel count, the odd filler entry, the tail of a plane's last
    // wave-level load) is out of range and arrives as zeros.  Per step only the
    // scalar offset moves; the per-lane offsets never change.
    //
    // A plane is PLS chunks (a multiple of 64), the weights of a step WCH
    // chunks (also one).  Load i of a wave covers chunks [c, c + 64) with
    // c = min(i*NT + 64*wave, size - 64): where the waves' shares are ragged the
    // surplus loads repeat the last chunk group (same bytes to the same place),
    // which keeps the staging code free of branches.
    const int wave_chunk = wave * 64;
    const int grp = wave >> 2;               // staging group of this wave
    const int grp_chunk = (wave & 3) * 64;   // its first chunk within the group's share
    const size_t in_bytes = (size_t)a.N * a.Cb * HW * 16;
    const size_t wt_bytes = (size_t)a.Cb * NTAPS * a.Kp * 16;
    const rsrc_t rsrc_in = make_rsrc(a.in, 0, in_bytes);
    const rsrc_t rsrc_wt = make_rsrc(a.wt, 0, wt_bytes);
    unsigned g_off[PPT];  // per-thread source byte offsets of the staged input pixels (plane 0)
    unsigned w_off[WPT];  // ... and of the staged weights (channel block 0)
    // Load number l of a step: the input loads (plane-major) come first, then the weights.
    constexpr int NLOADS = NPLG * PPT + WPT;
    auto fetch_one = [&](int st, int l) {
        // (the workgroup's reduction starts at step rot and wraps round: see IgemmArgs::rot_k)
        int sr = st + rot;
        if (sr >= nst) sr -= nst;
        const int cb0 = (sbeg + sr) * NPL;
        unsigned char *wb = lds + (st % NB) * bufbytes;
        unsigned char *ib = wb + WBYTES;
        if (l < NPLG * PPT) {
            const int j = l / PPT, i = l - j * PPT;
            const int pl = grp * NPLG + j;
            load_to_lds_16<NTI ? 2 : 0>(rsrc_in, g_off[i], (unsigned)(cb0 + pl) * (unsigned)HW * 16u,
                           ib + (pl * a.PLS + min(i * 256 + grp_chunk, a.PLS - 64)) * 16);
        } else {
            const int i = l - NPLG * PPT;
            load_to_lds_16(rsrc_wt, w_off[i], (unsigned)cb0 * (unsigned)(NTAPS * a.Kp) * 16u,
                           wb + min(i * NT + wave_chunk, WCH - 64) * 16);
        }
    };
    auto fetch = [&](int st) {
#pragma unroll
        for (int l = 0; l < NLOADS; ++l) fetch_one(st, l);
    };
    // The offsets are formed once per tile, and each load of the tile's FIRST step goes out as
    // soon as its offset is known: the weights first (their offsets are the cheaper ones), so
    // that the first bytes are on their way while the rest of the address arithmetic runs (a
    // tall filter's tile has nine to twelve input positions per thread, 2 - 3 us of it).
#pragma unroll
    for (int i = 0; i < WPT; ++i) {
        const int w = min(i * NT + wave_chunk, WCH - 64) + lane;
        unsigned off = kOutOfRange;
        const int e = w / TK;
        const int k = w - e * TK;
        const int tap = e / NPL;
        const int pl = e - tap * NPL;
        if (tap < NTAPS && k0 + k < a.Kp)
            off = (unsigned)(mul24(pl * NTAPS + tap, a.Kp) + k0 + k) * 16u;
        w_off[i] = off;
        fetch_one(0, NPLG * PPT + i);
    }
#pragma unroll
    for (int i = 0; i < PPT; ++i) {
        const int p = min(i * 256 + grp_chunk, a.PLS - 64) + lane;
        unsigned off = kOutOfRange;
        if (p < a.LRW) {
            const int row = fast_div(p, inv_LW);
            const int col = p - mul24(row, a.LW);
            int n, ih, iw;
            bool ok;
            if (a.sampled) {
                const int rho = rho0 + row;
                n = fast_div(rho, inv_P);
                ih = mul24(rho - mul24(n, a.P), a.stride);
                iw = mul24(q0 + col, a.stride);
                ok = rho < NP && (q0 + col) < a.Q;
            } else {
                const int lam = lam0 + row;
                n = fast_div(lam, inv_Hs);
                ih = lam - mul24(n, a.Hs) - a.pad_h;
                iw = q0 * a.cstride - a.pad_w + col;
                ok = n < a.N && ih >= 0 && ih < a.H && iw >= 0 && iw < a.W;
            }
            if (ok) off = (unsigned)(mul24(mul24(mul24(n, a.Cb), a.H) + ih, a.W) + iw) * 16u;
        }
        g_off[i] = off;
#pragma unroll
        for (int j = 0; j < NPLG; ++j) fetch_one(0, j * PPT + i);
    }
    // All of this wave's staging loads have landed in LDS and all of its LDS reads are done.
    auto staged = [&]() { wait_all_memory(); };

    // ---- per-lane pixel bookkeeping for the B fragments and the epilogue
    int bpos[FM];
    unsigned obyte[FM];  // byte offset of the lane's pixel in output channel block 0
    const int Kb_out = a.out_kb;
#pragma unroll
    for (int j = 0; j < FM; ++j) {
        const int m = (wave_m * FM + j) * 32 + l32;
        const int trow = fast_div(m, inv_TQ);
        const int tcol = m - mul24(trow, a.TQ);
        const int rho = rho0 + trow;
        const bool ok = trow < a.TR && rho < NP && (q0 + tcol) < a.Q;
        const int n = fast_div(rho, inv_P);
        const int oj = rho - mul24(n, a.P);
        int pos = a.sampled ? m
                            : mul24(mul24(n, a.Hs) + mul24(oj, a.stride) - lam0, a.LW) +
                                  mul24(tcol, a.cstride);
        if (!ok) pos = 0;
        // lane halves read two channel planes, or (one plane per step) two taps
        bpos[j] = ((NPL == 1 ? 0 : h) * a.PLS + pos) * 16;
        obyte[j] = ok ? (unsigned)(mul24(mul24(mul24(n, Kb_out), a.OH) + mul24(oj, a.ostr) + a.oy0,
                                         a.OW) +
                                   mul24(q0 + tcol, a.ostr_x) + a.ox0) * 16u
                      : kOutOfRange;
    }
    const int a_base = (h * TK + wave_k * FK * 32 + l32) * 16;

    f32x16 acc[FK][FM];
#pragma unroll
    for (int i = 0; i < FK; ++i)
#pragma unroll
        for (int j = 0; j < FM; ++j)
#pragma unroll
            for (int t = 0; t < 16; ++t) acc[i][j][t] = 0.0f;

    // (step 0's loads went out above) the other steps of the first NB-1; step 0 must have
    // landed before anyone reads it
#pragma unroll
    for (int d = 1; d < NB - 1; ++d)
        if (d < nst) fetch(d);
    staged();
    __syncthreads();

    if constexpr (NPL == 1) {
        static_assert(NB == 2, "the one-plane path is double buffered");
        // One channel block per step: the two lane halves take two taps.
        for (int st = 0; st < nst; ++st) {
            if (st + 1 < nst) fetch(st + 1);
            const unsigned char *wb = lds + (st & 1) * bufbytes;
            const unsigned char *ib = wb + WBYTES;
            // (the operands of tap pair q+1 are read before the MFMAs of pair q issue)
            auto read_pair = [&](int q, u32x4(&af)[FK], u32x4(&bf)[FM]) {
                const int t0 = 2 * q;
                const int t1 = (2 * q + 1 < NTAPS) ? 2 * q + 1 : NTAPS - 1;
                const int off0 = ((t0 / S) * a.LW + (t0 % S)) * 16;
                const int off1 = ((t1 / S) * a.LW + (t1 % S)) * 16;
                const int toff = h ? off1 : off0;
#pragma unroll
                for (int i = 0; i < FK; ++i)
                    af[i] = *reinterpret_cast<const u32x4 *>(wb + a_base + (2 * q * TK + 32 * i) * 16);
#pragma unroll
                for (int j = 0; j < FM; ++j)
                    bf[j] = *reinterpret_cast<const u32x4 *>(ib + bpos[j] + toff);
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
                    for (int j = 0; j < FM; ++j) E_::mma(ac[i], bc[j], acc[i][j]);
                // Issue order of the round: one MFMA, then one LDS read of the next pair's
                // operands, and so on (left to itself the compiler reads each operand right
                // before the MFMA that takes it, into one register set, and waits there).
                constexpr int NMFMA1 = FK * FM * (DT == CONV_F32 ? 4 : 1);
#pragma unroll
                for (int k = 0; k < NMFMA1; ++k) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // LDS read
                }
                __builtin_amdgcn_sched_barrier(0);
                if (q + 1 < NENT / 2) {
#pragma unroll
                    for (int i = 0; i < FK; ++i) ac[i] = an[i];
#pragma unroll
                    for (int j = 0; j < FM; ++j) bc[j] = bn[j];
                }
            }
            staged();
            __syncthreads();
        }
    } else {
        // A step is NQ MFMA rounds (tap x plane pair).  The operands of round
        // q+1 are read from LDS into a second register set while the MFMAs of
        // round q issue.  The next step's staging loads all issue in round 0
        // and are awaited before the LAST round, together with this wave's final
        // reads of the current buffer; after that barrier the last round already
        // reads the next step's first operands, and the buffer just left is free
        // for the loads of the step after.
        constexpr int NQ = NTAPS * (NPL / 2);
        static_assert(NQ >= 2, "a step needs two MFMA rounds");
        u32x4 ac[FK], bc[FM];
        auto read_round = [&](int buf, int q, u32x4(&af)[FK], u32x4(&bf)[FM]) {
            const unsigned char *wb = lds + buf * bufbytes;
            const unsigned char *ib = wb + WBYTES;
            const int tap = q / (NPL / 2), pp = q - tap * (NPL / 2);
            const int toff = ((tap / S) * a.LW + (tap % S) + 2 * pp * a.PLS) * 16;
#pragma unroll
            for (int i = 0; i < FK; ++i)
                af[i] = *reinterpret_cast<const u32x4 *>(wb + a_base + (2 * q * TK + 32 * i) * 16);
#pragma unroll
            for (int j = 0; j < FM; ++j)
                bf[j] = *reinterpret_cast<const u32x4 *>(ib + bpos[j] + toff);
        };
        // With NB > 2 buffers the loads of step st+NB-1 issue during step st and a
        // step waits only for the loads of the step that follows it: a wave's
        // loads complete in order, so "all but the newest (NB-2)*NLOADS" is that.
        // Near the end, when nothing further is issued, it waits for everything.
        constexpr int AHEAD = NB - 1;
        constexpr int LEAVE = (NB - 2) * NLOADS;
        static_assert(LEAVE <= 63, "outstanding loads exceed the counter");
        // s_waitcnt: vmcnt(LEAVE) lgkmcnt(0), export counter untouched
        constexpr int WAIT_PARTIAL = (LEAVE & 15) | ((LEAVE >> 4) << 14) | (7 << 4) | (0 << 8);
        auto step = [&](int st, auto more_tag, auto issue_tag) {
            constexpr bool MORE = decltype(more_tag)::value;    // a step follows
            constexpr bool ISSUE = decltype(issue_tag)::value;  // step st+AHEAD exists
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                u32x4 an[FK], bn[FM];
                if (q + 1 < NQ)
                    read_round(st % NB, q + 1, an, bn);
                else if (MORE)
                    read_round((st + 1) % NB, 0, an, bn);
                if (ISSUE && q == 0) fetch(st + AHEAD);
#pragma unroll
                for (int i = 0; i < FK; ++i)
#pragma unroll
                    for (int j = 0; j < FM; ++j) E_::mma(ac[i], bc[j], acc[i][j]);
                // Issue order of the round: one MFMA, then an LDS read or a
                // staging load, and so on, instead of all reads first.
                constexpr int NMFMA = FK * FM * (DT == CONV_F32 ? 4 : 1);
#pragma unroll
                for (int k = 0; k < NMFMA; ++k) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // LDS read
                    __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);  // staging loads
                }
                __builtin_amdgcn_sched_barrier(0);
                if (MORE && q == NQ - 2) {
                    if (ISSUE && NB > 2)
                        __builtin_amdgcn_s_waitcnt(WAIT_PARTIAL);
                    else
                        staged();
                    __syncthreads();
                }
                if (q + 1 < NQ || MORE) {
#pragma unroll
                    for (int i = 0; i < FK; ++i) ac[i] = an[i];
#pragma unroll
                    for (int j = 0; j < FM; ++j) bc[j] = bn[j];
                }
            }
        };
        read_round(0, 0, ac, bc);
        int st = 0;
        for (; st + AHEAD < nst; ++st) step(st, std::true_type{}, std::true_type{});
        for (; st + 1 < nst; ++st) step(st, std::true_type{}, std::false_type{});
        step(st, std::false_type{}, std::false_type{});
    }

    // ---- epilogue: each lane owns, per fragment, one pixel and 4x4 channels.
    // The channel block of a store is wave-uniform, so it rides in the scalar
    // offset; the per-lane offset is the pixel's.
    const size_t oplane = (size_t)a.OH * a.OW * 16;
    const size_t out_bytes = (size_t)a.N * Kb_out * oplane;
    if (a.ksplit > 1) {
        // partial result of this reduction split: fp32, the output tensor's element
        // order (so for bf16 every byte offset doubles), copy sp
        constexpr unsigned SC = (V == 8) ? 2u : 1u;
        const rsrc_t rp = make_rsrc(static_cast<char *>(a.out) + (size_t)sp * out_bytes * SC, 0,
                                    out_bytes * SC);
#pragma unroll
        for (int i = 0; i < FK; ++i) {
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                const int krow0 = k0 + (wave_k * FK + i) * 32 + vq * 8;
                if (krow0 >= a.Kp) continue;
                const unsigned skip = (unsigned)(krow0 / V) * (unsigned)oplane;
                const unsigned lane_off = (V == 4) ? (unsigned)h * (unsigned)oplane : (unsigned)h * 8u;
#pragma unroll
                for (int j = 0; j < FM; ++j) {
                    const bool live = obyte[j] != kOutOfRange && krow0 + 4 * h < a.Kp;
                    Elem<CONV_F32>::store4(rp, live ? (obyte[j] + lane_off) * SC : kOutOfRange, skip * SC,
                                           acc[i][j][4 * vq + 0], acc[i][j][4 * vq + 1],
                                           acc[i][j][4 * vq + 2], acc[i][j][4 * vq + 3]);
                }
            }
        }
        return;
    }
    const rsrc_t ro = make_rsrc(a.out, 0, out_bytes);
    if (a.scale != nullptr || a.bias != nullptr || a.resid != nullptr || a.relu != 0) {
        // L() of Algorithm 4 on the finished accumulators: scale, bias, residual, ReLU (forward
        // pass: plain store geometry).  The residual values of a row group are all
        // requested before the first of them is used, and before any store of the group
        // (the residual may be the output buffer itself).
        const rsrc_t rres = make_rsrc(a.resid ? a.resid : a.out, 0, out_bytes);
#pragma unroll
        for (int i = 0; i < FK; ++i) {
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                const int krow0 = k0 + (wave_k * FK + i) * 32 + vq * 8;  // + 4*h for this lane
                if (krow0 >= a.Kp) continue;                            // wave-uniform
                const bool rows_live = krow0 + 4 * h < a.Kp;
                float b4[4] = {0.f, 0.f, 0.f, 0.f};
                if (a.bias && rows_live) {
                    const f32x4 b = *reinterpret_cast<const f32x4 *>(a.bias + krow0 + 4 * h);
                    b4[0] = b[0]; b4[1] = b[1]; b4[2] = b[2]; b4[3] = b[3];
                }
                float s4[4] = {1.f, 1.f, 1.f, 1.f};
                if (a.scale && rows_live) {
                    const f32x4 g = *reinterpret_cast<const f32x4 *>(a.scale + krow0 + 4 * h);
                    s4[0] = g[0]; s4[1] = g[1]; s4[2] = g[2]; s4[3] = g[3];
                }
                const unsigned skip = (unsigned)(krow0 / V) * (unsigned)oplane;
                const unsigned lane_off = (V == 4) ? (unsigned)h * (unsigned)oplane : (unsigned)h * 8u;
                float r4[FM][4];
#pragma unroll
                for (int j = 0; j < FM; ++j)
#pragma unroll
                    for (int t = 0; t < 4; ++t) r4[j][t] = 0.0f;
                if (a.resid) {
#pragma unroll
                    for (int j = 0; j < FM; ++j) {
                        const bool live = obyte[j] != kOutOfRange && rows_live;
                        E_::load4(rres, live ? obyte[j] + lane_off : kOutOfRange, skip, r4[j]);
                    }
                }
#pragma unroll
                for (int j = 0; j < FM; ++j) {
                    const bool live = obyte[j] != kOutOfRange && rows_live;
                    float o4[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        o4[t] = acc[i][j][4 * vq + t] * s4[t] + r4[j][t] + b4[t];
                        if (a.relu) o4[t] = fmaxf(o4[t], 0.0f);
                    }
                    E_::template store4<CONVMI_OUT_POLICY>(ro, live ? obyte[j] + lane_off : kOutOfRange, skip,
                                                           o4[0], o4[1], o4[2], o4[3]);
                }
            }
        }
        return;
    }
    if (!a.shuffle && !a.zero_fill) {
        // Plain store: the lane's byte offsets (pixel, lane half) are formed once; per group
        // of 8 channel rows only the scalar offset (the channel block) changes.
        const unsigned lane_off = (V == 4) ? (unsigned)h * (unsigned)oplane : (unsigned)h * 8u;
        unsigned ooff[FM];
#pragma unroll
        for (int j = 0; j < FM; ++j) ooff[j] = obyte[j] != kOutOfRange ? obyte[j] + lane_off : kOutOfRange;
#pragma unroll
        for (int i = 0; i < FK; ++i) {
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                const int krow0 = k0 + (wave_k * FK + i) * 32 + vq * 8;  // + 4*h for this lane
                if (krow0 >= a.Kp) continue;                            // wave-uniform
                const unsigned skip = (unsigned)(krow0 / V) * (unsigned)oplane;
                // (fp32: the upper lane half's block may lie beyond the last channel block)
                const bool upper_dead = (V == 4) && krow0 + 4 >= a.Kp;  // wave-uniform
                if (!upper_dead) {
#pragma unroll
                    for (int j = 0; j < FM; ++j)
                        E_::template store4<CONVMI_OUT_POLICY>(ro, ooff[j], skip, acc[i][j][4 * vq + 0], acc[i][j][4 * vq + 1],
                                   acc[i][j][4 * vq + 2], acc[i][j][4 * vq + 3]);
                } else {
#pragma unroll
                    for (int j = 0; j < FM; ++j)
                        E_::template store4<CONVMI_OUT_POLICY>(ro, h ? kOutOfRange : ooff[j], skip, acc[i][j][4 * vq + 0],
                                   acc[i][j][4 * vq + 1], acc[i][j][4 * vq + 2], acc[i][j][4 * vq + 3]);
                }
            }
        }
        return;
    }
    // Scattering store (strided backward): position of the lane's result pixels in the
    // output tensor, recomputed here rather than kept in registers across the main loop.
    int sy[FM], sx[FM];
#pragma unroll
    for (int j = 0; j < FM; ++j) {
        const int m = (wave_m * FM + j) * 32 + l32;
        const int trow = fast_div(m, inv_TQ);
        const int tcol = m - mul24(trow, a.TQ);
        const int rho = rho0 + trow;
        const int n = fast_div(rho, inv_P);
        sy[j] = mul24(rho - mul24(n, a.P), a.ostr) + a.oy0;
        sx[j] = mul24(q0 + tcol, a.ostr_x) + a.ox0;
    }
#pragma unroll
    for (int i = 0; i < FK; ++i) {
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
            const int krow0 = k0 + (wave_k * FK + i) * 32 + vq * 8;  // + 4*h for this lane
            if (krow0 >= a.Kp) continue;                            // wave-uniform
            // fp32: 8 rows = blocks 2*q (h=0) and 2*q+1 (h=1); bf16: one block, halves by h
            // Shuffle mode: the lane's channel block is a position of the ostr x ostr_x cell.
            const int blk = krow0 / V + (V == 4 ? h : 0);
            const int cy = blk / a.ostr_x, cx = blk - cy * a.ostr_x;
            const unsigned skip = a.shuffle ? 0u : (unsigned)(krow0 / V) * (unsigned)oplane;
            const unsigned lane_off =
                a.shuffle ? (unsigned)(cy * a.OW + cx) * 16u + (V == 4 ? 0u : (unsigned)h * 8u)
                          : ((V == 4) ? (unsigned)h * (unsigned)oplane : (unsigned)h * 8u);
#pragma unroll
            for (int j = 0; j < FM; ++j) {
                // (fp32: the upper lane half's block may lie beyond the last channel block)
                bool live = obyte[j] != kOutOfRange && krow0 + 4 * h < a.Kp;
                if (a.shuffle) live = live && sy[j] + cy < a.OH && sx[j] + cx < a.OW;
                const unsigned off = live ? obyte[j] + lane_off : kOutOfRange;
                E_::store4(ro, off, skip, acc[i][j][4 * vq + 0], acc[i][j][4 * vq + 1],
                           acc[i][j][4 * vq + 2], acc[i][j][4 * vq + 3]);
                if (a.zero_fill) {
                    for (int dy = 0; dy < a.ostr; ++dy)
                        for (int dx = 0; dx < a.ostr_x; ++dx) {
                            if ((dy | dx) == 0) continue;
                            const bool in = live && sy[j] + dy < a.OH && sx[j] + dx < a.OW;
                            E_::store4(ro, in ? off + (unsigned)(dy * a.OW + dx) * 16u : kOutOfRange,
                                       skip, 0.f, 0.f, 0.f, 0.f);
                        }
                }
            }
        }
    }
}


typedef void (*igemm_fn_t)(const IgemmArgs);
struct IgemmEntry {
    IgemmVariant v;
    igemm_fn_t fn;
};

#define IGEMM_ENTRY_NB_NT(DT, WK, WM, FK, FM, NPL, R, S, PPT, NB, NT)          \
    {                                                                            \
        {DT, WK, WM, FK, FM, NPL, R, S, PPT, NB, NT},                            \
            igemm_kernel<DT, WK, WM, FK, FM, NPL, R, S, PPT, NB, NT>             \
    }
#define IGEMM_ENTRY_NB(DT, WK, WM, FK, FM, NPL, R, S, PPT, NB) \
    IGEMM_ENTRY_NB_NT(DT, WK, WM, FK, FM, NPL, R, S, PPT, NB, 0)
#define IGEMM_ENTRY(DT, WK, WM, FK, FM, NPL, R, S, PPT) \
    IGEMM_ENTRY_NB(DT, WK, WM, FK, FM, NPL, R, S, PPT, 2)


// Entries of the rectangular-filter translation unit.
IgemmEntry *igemm_rect_entries(int *count);

}  // namespace convmi
