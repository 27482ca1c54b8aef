// Weight-gradient update (Algorithm 8 of the paper, with padding) for bf16
// tensors on MFMA, fp32 accumulation and output -- the kernel for stride-1
// layers (and for 1x1 layers of any stride, whose input is staged sampled).
//
//   dW[k,c,r,s] = sum over (n,oj,oi) of I[n,c,oj-pad+r,oi-pad+s] * dO[n,k,oj,oi]
//
// M = input channels, N = output channels, reduction = pixels; one 32x32
// accumulator tile per filter tap, all taps of the tile resident in the wave
// (the register-resident dW block of Algorithm 9).
//
// The MFMA takes 8 consecutive reduction indices (pixels) per lane while the
// blocked layout keeps 8 channels of one pixel together: the transpose the paper
// pays for up front on Knights Mill (Section III-B).  Here the bands stay in LDS
// exactly as they sit in HBM ([plane][pixel][8 channels]) and gfx950's
// transposing LDS read hands each lane four consecutive pixels of its channel.
//
// The reduction walks 8-pixel runs along output rows; the two lane halves of a
// step take two different runs.  For one filter row r a lane reads a window of
// 12 consecutive input pixels of its channel once and forms the operands of the
// S taps from it in registers (a tap one pixel to the right is the same data
// shifted by 16 bits): the staged input row is read once per filter row, not
// once per tap.
//
// Staging is by buffer loads straight into a double-buffered LDS band (padding
// and band tails are out-of-range lanes and arrive as zeros); the next band
// streams in while the current one is consumed.  Grid = (split of the linear
// output-row range) x (channel tiles); every split writes a private partial dW
// and the reduce kernel sums them in a fixed order.  Waves that share a channel
// tile but take different runs (WP > 1) write private copies as well.
#include "conv_internal.h"

namespace convmi {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// STRIDED: filters larger than 1x1 with stride > 1.  Consecutive output pixels are then
// `stride` input pixels apart, so a tap's operand is not a shifted window any more; the
// transposing read takes a per-lane address, and the lanes of a group simply address
// pixels stride*(q+j) + s: two reads per tap instead of a shared window per filter row.
template <int R, int S, int WC, int WK, int WP, int FC, int FK, bool STRIDED = false>
__global__ __launch_bounds__(WC *WK *WP * 64) void upd_rows_bf16_kernel(const UpdArgs a)
{
    constexpr int V = 8;
    constexpr int NT = WC * WK * WP * 64;
    constexpr int NTAPS = R * S;
    constexpr int TC = WC * FC * 32;
    constexpr int TK = WK * FK * 32;
    constexpr int NPI = TC / V;
    constexpr int NPO = TK / V;
    constexpr int WIN = (8 + S - 1 + 3) / 4;  // 4-pixel reads covering a run plus S-1 shifts
    static_assert(NT == 256 || NT == 512, "four or eight waves");
    // Two waves per SIMD need the accumulators to fit the 256 AGPRs outright:
    // above that the compiler shuttles tiles between register files every step.
    static_assert(NTAPS * FC * FK * 16 <= 256, "accumulators must fit the AGPRs");
    static_assert(S <= 9, "window of at most four 4-pixel reads");

    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int ibytes = NPI * a.PLS_in * 16;
    const int obytes = NPO * a.PLS_out * 16;
    const int bufbytes = ibytes + obytes;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // (uniform: kept in a scalar register)
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);  // the same, known to be uniform
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

    const int NP = a.N * a.P;
    const int rho_begin = split * a.rows_per_split;
    const int rho_end = min(NP, rho_begin + a.rows_per_split);
    const int RP = a.runs * 8;              // staged dO row pitch (pixels), zero padded beyond Q
    const int npxO = a.TR * RP + 8;         // ... plus one all-zero run for idle lane halves
    const int HW = a.H * a.W, PQ = a.P * a.Qpitch;
    const int gap = a.sampled ? 0 : a.Hs - a.P;  // staged rows between images (stride 1)
    const int lst = STRIDED ? a.stride : 1;      // input pixels per output pixel in the staged band
    const float inv_LW = 1.0f / (float)a.LW, inv_Hs = 1.0f / (float)a.Hs;
    const float inv_RP = 1.0f / (float)RP, inv_P = 1.0f / (float)a.P;
    const float inv_runs = 1.0f / (float)a.runs;
    const size_t in_bytes = (size_t)a.N * a.Cb * HW * 16;
    const size_t out_bytes = (size_t)a.N * a.Kb * PQ * 16;
    const rsrc_t rsrc_in = make_rsrc(a.in, 0, in_bytes);
    const rsrc_t rsrc_out = make_rsrc(a.dout, 0, out_bytes);

    // Stage the bands of linear output rows [rho0, rho0 + TR) into buffer `buf`.
    auto fetch = [&](int rho0, int buf) {
        unsigned char *ib = lds + buf * bufbytes;
        unsigned char *ob = ib + ibytes;
        const int n0 = fast_div(rho0, inv_P);
        const int lam0 = n0 * a.Hs + (rho0 - n0 * a.P) * lst;
        // Positions are staged in whole wave-level loads (64 chunks); the plane pitch is
        // that count plus 4 pixels, so that the two planes a 16-lane transposing read
        // touches start 64 bytes apart in the 256-byte bank row.
        constexpr int NW = NT / 64;
        const int cov_in = (a.LRW + 63) & ~63, cov_out = (npxO + 63) & ~63;
        // byte offset of staged input position p / dO position p in channel block 0
        auto in_off = [&](int p) -> unsigned {
            if (p >= a.LRW) return kOutOfRange;
            const int row = fast_div(p, inv_LW);
            const int col = p - row * a.LW;
            int n, ih, iw;
            bool ok;
            if (a.sampled) {
                const int rho = rho0 + row;
                n = fast_div(rho, inv_P);
                ih = (rho - n * a.P) * a.stride;
                iw = (a.q0 + col) * a.stride;
                ok = rho < rho_end && col < a.Q;
            } else {
                const int lam = lam0 + row;
                n = fast_div(lam, inv_Hs);
                ih = lam - n * a.Hs - a.pad;
                iw = col + a.q0 * lst - a.pad_w;
                ok = n < a.N && ih >= 0 && ih < a.H && iw >= 0 && iw < a.W;
            }
            return ok ? (unsigned)((n * a.Cb * a.H + ih) * a.W + iw) * 16u : kOutOfRange;
        };
        auto out_off = [&](int p) -> unsigned {
            if (p >= a.TR * RP) return kOutOfRange;
            const int trow = fast_div(p, inv_RP);
            const int col = p - trow * RP;
            const int rho = rho0 + trow;
            if (rho >= rho_end || col >= a.Q) return kOutOfRange;
            const int n = fast_div(rho, inv_P);
            const int oj = rho - n * a.P;
            return (unsigned)((n * a.Kb * a.P + oj) * a.Qpitch + a.q0 + col) * 16u;
        };
        // (channel blocks beyond the tensor are out of range as a whole: zeros)
        auto load_in = [&](int pl, int p0, unsigned off) {
            load_to_lds_16<CONVMI_UPD_POLICY>(rsrc_in, cb0 + pl < a.Cb ? off : kOutOfRange,
                           (unsigned)(cb0 + pl) * (unsigned)HW * 16u, ib + (pl * a.PLS_in + p0) * 16);
        };
        auto load_out = [&](int pl, int p0, unsigned off) {
            load_to_lds_16<CONVMI_UPD_POLICY>(rsrc_out, kb0 + pl < a.Kb ? off : kOutOfRange,
                           (unsigned)(kb0 + pl) * (unsigned)PQ * 16u, ob + (pl * a.PLS_out + p0) * 16);
        };
        // Unit of staging work: one 64-position chunk x 8 planes (8 wave-level
        // loads behind one offset computation).  Input units go to the waves in
        // ascending order, dO units in descending order, so that a band's units
        // spread over all waves instead of piling up on the first ones.
        static_assert(NPI % 8 == 0 && NPO % 8 == 0, "plane groups of 8");
        constexpr int GI = NPI / 8, GO = NPO / 8;
        const int nu_in = (cov_in >> 6) * GI, nu_out = (cov_out >> 6) * GO;
        for (int u = wave_u; u < nu_in; u += NW) {
            const int ch = u / GI, g = u - ch * GI;
            const unsigned off = in_off(ch * 64 + lane);
#pragma unroll
            for (int pl = 0; pl < 8; ++pl) load_in(g * 8 + pl, ch * 64, off);
        }
        for (int u = NW - 1 - wave_u; u < nu_out; u += NW) {
            const int ch = u / GO, g = u - ch * GO;
            const unsigned off = out_off(ch * 64 + lane);
#pragma unroll
            for (int pl = 0; pl < 8; ++pl) load_out(g * 8 + pl, ch * 64, off);
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

    // Byte offset, within a staged band, of what this lane addresses in a
    // transposing read: pixel (i16 / 4) of the 4-pixel group, channels
    // 16*grp + 4*(i16 % 4) .. +3 of the fragment.
    int a_lane[FC], b_lane[FK];
#pragma unroll
    for (int i = 0; i < FC; ++i) {
        const int c = (wave_c * FC + i) * 32 + grp * 16 + (i16 & 3) * 4;
        a_lane[i] = ((c / V) * a.PLS_in + lst * (i16 >> 2)) * 16 + (c % V) * 2;
    }
#pragma unroll
    for (int j = 0; j < FK; ++j) {
        const int k = (wave_k * FK + j) * 32 + grp * 16 + (i16 & 3) * 4;
        b_lane[j] = ((k / V) * a.PLS_out + (i16 >> 2)) * 16 + (k % V) * 2;
    }

    int nsteps = 0;
    for (int rho0 = rho_begin; rho0 < rho_end; rho0 += a.TR) ++nsteps;
    if (nsteps > 0) {
        fetch(rho_begin, 0);
        wait_all_memory();
    }
    __syncthreads();

    int step = 0;
    for (int rho0 = rho_begin; rho0 < rho_end; rho0 += a.TR, ++step) {
        // (the even waves issue the next band's loads at the top of the band, the odd ones halfway
        // through their run pairs)
        bool pending = rho0 + a.TR < rho_end;
        if (pending && (wave & 1) == 0) {
            fetch(rho0 + a.TR, (step + 1) & 1);
            pending = false;
        }
        const unsigned char *ib = lds + (step & 1) * bufbytes;
        const unsigned char *ob = ib + ibytes;

        const int rows = min(a.TR, rho_end - rho0);
        const int nruns = rows * a.runs;
        const int n0 = fast_div(rho0, inv_P);
        const int oj0 = rho0 - n0 * a.P;
        // Run pairs: lane half h takes run 2*t + h; waves along pixels interleave t.
        // (Two waves per SIMD: one wave's LDS latency hides behind the other's MFMAs.)
        // (The transposing reads are issued untracked -- see lds_read_tr16_b64_untracked -- so that
        // the next band's loads, which write into the other buffer, stay in flight behind them.)
        constexpr int PER_ROW = STRIDED ? 2 * S : WIN;  // reads per filter row and fragment
        const unsigned ib_a = lds_address(ib), ob_a = lds_address(ob);
        struct PairAddr {
            int ipix, opix;
        };
        auto pair_addr = [&](int t) -> PairAddr {
            const int q = 2 * t + h;
            const bool live = q < nruns;
            const int trow = fast_div(q, inv_runs);
            const int ri = q - trow * a.runs;
            int lrow = trow;
            if (STRIDED) {
                const int dn = fast_div(oj0 + trow, inv_P);
                lrow = dn * a.Hs + (oj0 + trow - dn * a.P - oj0) * lst;
            } else if (!a.sampled) {
                // staged row of output row (rho0 + trow), tap row 0
                const int dn = fast_div(oj0 + trow, inv_P);
                lrow = trow + dn * gap;
            }
            // (a pair beyond the band's runs reads position 0 and the zero run: valid addresses)
            return PairAddr{live ? (lrow * a.LW + ri * 8 * lst) * 16 : 0,
                            live ? (trow * RP + ri * 8) * 16 : a.TR * RP * 16};
        };
        auto read_out = [&](const PairAddr &pa, u32x2 (&bf)[FK][2]) {
#pragma unroll
            for (int j = 0; j < FK; ++j) {
                const unsigned p = ob_a + b_lane[j] + pa.opix;
                bf[j][0] = lds_read_tr16_b64_untracked<0>(p);
                bf[j][1] = lds_read_tr16_b64_untracked<4 * 16>(p);
            }
        };
        // filter rows [r0, r1) of the input operand
        auto read_in = [&](const PairAddr &pa, int r0, int r1, u32x2 (&w)[R][FC][PER_ROW]) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                if (r < r0 || r >= r1) continue;
#pragma unroll
                for (int i = 0; i < FC; ++i) {
                    const unsigned p = ib_a + a_lane[i] + pa.ipix + r * a.LW * 16;
                    if constexpr (STRIDED) {
                        // the 8 output pixels of the run under tap (r, sx): input pixels
                        // stride*j + sx of the window, four per read
                        const unsigned p2 = p + lst * 4 * 16;
                        static_for<0, S>([&](auto sx) {
                            constexpr int SX = decltype(sx)::value;
                            w[r][i][2 * SX] = lds_read_tr16_b64_untracked<SX * 16>(p);
                            w[r][i][2 * SX + 1] = lds_read_tr16_b64_untracked<SX * 16>(p2);
                        });
                    } else {
                        // window of 4*WIN consecutive pixels of this lane's channel, 2 per dword
                        static_for<0, WIN>([&](auto g) {
                            constexpr int G = decltype(g)::value;
                            w[r][i][G] = lds_read_tr16_b64_untracked<4 * G * 16>(p);
                        });
                    }
                }
            }
        };
        // The MFMAs of one filter row, once its reads (and, with the first row, dO's) have landed.
        auto mma_row = [&](auto rr, u32x2 (&w)[R][FC][PER_ROW], u32x2 (&bf)[FK][2]) {
            constexpr int r = decltype(rr)::value;
            if constexpr (r == 0) {
#pragma unroll
                for (int j = 0; j < FK; ++j) {
                    lds_read_landed(bf[j][0]);
                    lds_read_landed(bf[j][1]);
                }
            }
#pragma unroll
            for (int i = 0; i < FC; ++i)
#pragma unroll
                for (int g = 0; g < PER_ROW; ++g) lds_read_landed(w[r][i][g]);
#pragma unroll
            for (int i = 0; i < FC; ++i)
#pragma unroll
                for (int s = 0; s < S; ++s) {
                    u32x4 af;
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        if constexpr (STRIDED) {
                            af[d] = w[r][i][2 * s + d / 2][d & 1];
                        } else {
                            const int lo = d + s / 2;
                            const unsigned w_lo = w[r][i][lo / 2][lo & 1];
                            af[d] = (s & 1) ? __builtin_amdgcn_alignbit(w[r][i][(lo + 1) / 2][(lo + 1) & 1],
                                                                        w_lo, 16)
                                            : w_lo;
                        }
                    }
#pragma unroll
                    for (int j = 0; j < FK; ++j) {
                        const u32x4 bq = {bf[j][0][0], bf[j][0][1], bf[j][1][0], bf[j][1][1]};
                        acc[r * S + s][i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            __builtin_bit_cast(bf16x8, af), __builtin_bit_cast(bf16x8, bq),
                            acc[r * S + s][i][j], 0, 0, 0);
                    }
                }
        };
        constexpr int ROW_READS = FC * PER_ROW;           // reads of one filter row
        constexpr int HEAD_READS = 2 * FK + ROW_READS;    // dO's and the first filter row's
        constexpr int PAIR_READS = 2 * FK + R * ROW_READS;
        // The reads of the next pair go out while this pair's MFMAs issue, if the wave's counter of
        // pending LDS operations (four bits) can hold a pair's reads.
        constexpr bool AHEAD = !STRIDED && PAIR_READS <= 15;
        if constexpr (AHEAD) {
            // One pair: `w`, `bf` hold (or are about to receive) this pair's operands, all of its
            // reads pending at most; the next pair's reads are issued into `wn`, `bn` in two parts --
            // dO and the first filter row as soon as this pair's have landed, the other rows before
            // the last row's MFMAs -- so that PAIR_READS are pending again when it returns.
            auto pair_step = [&](int tn, u32x2 (&w)[R][FC][PER_ROW], u32x2 (&bf)[FK][2],
                                 u32x2 (&wn)[R][FC][PER_ROW], u32x2 (&bn)[FK][2]) {
                const PairAddr pn = pair_addr(tn);
                static_for<0, R>([&](auto rr) {
                    constexpr int r = decltype(rr)::value;
                    lds_reads_pending<(R - 1 - r) * ROW_READS + (r > 0 ? HEAD_READS : 0)>();
                    if constexpr (r == 0) {
                        mma_row(rr, w, bf);  // (registers pinned first, then the MFMAs)
                        read_out(pn, bn);
                        read_in(pn, 0, 1, wn);
                    } else {
                        if constexpr (r == R - 1) read_in(pn, 1, R, wn);
                        mma_row(rr, w, bf);
                    }
                });
            };
            int t = wave_p;
            if (2 * t < nruns) {
                u32x2 wa[R][FC][PER_ROW], wb[R][FC][PER_ROW];
                u32x2 ba[FK][2], bb[FK][2];
                {
                    const PairAddr p0 = pair_addr(t);
                    read_out(p0, ba);
                    read_in(p0, 0, R, wa);
                }
                for (;;) {
                    if (pending && 4 * t >= nruns) {
                        fetch(rho0 + a.TR, (step + 1) & 1);
                        pending = false;
                    }
                    pair_step(t + WP, wa, ba, wb, bb);
                    t += WP;
                    if (2 * t >= nruns) break;
                    if (pending && 4 * t >= nruns) {
                        fetch(rho0 + a.TR, (step + 1) & 1);
                        pending = false;
                    }
                    pair_step(t + WP, wb, bb, wa, ba);
                    t += WP;
                    if (2 * t >= nruns) break;
                }
            }
        } else {
            u32x2 w0[R][FC][PER_ROW];
            u32x2 b0[FK][2];
            for (int t = wave_p; 2 * t < nruns; t += WP) {
                if (pending && 4 * t >= nruns) {
                    fetch(rho0 + a.TR, (step + 1) & 1);
                    pending = false;
                }
                const PairAddr p0 = pair_addr(t);
                read_out(p0, b0);
                read_in(p0, 0, R, w0);
                static_for<0, R>([&](auto rr) {
                    constexpr int r = decltype(rr)::value;
                    // the reads of the filter rows behind this one may still be on their way
                    lds_reads_pending<(R - 1 - r) * ROW_READS>();
                    mma_row(rr, w0, b0);
                });
            }
        }
        if (pending) fetch(rho0 + a.TR, (step + 1) & 1);
        wait_all_memory();
        __syncthreads();
    }

    // ---- this (split, pixel wave)'s partial dW tile: [copy][cb][tap][k][c%8]
    // (a launch may serve taps [tap0, tap0 + R*S) of a taller filter with ntaps_all taps)
    const size_t copy = (size_t)a.Cb * a.ntaps_all * a.Kp * V;
    float *dst = a.partial + ((size_t)a.copy0 + (size_t)split * WP + wave_p) * copy;
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

typedef void (*upd_rows_fn_t)(const UpdArgs);
struct UpdRowsEntry {
    UpdRowsVariant v;
    upd_rows_fn_t fn;
};
#define UPD_ROWS_ENTRY(R, S, WC, WK, WP, FC, FK)                                         \
    {                                                                                    \
        {R, S, WC, WK, WP, FC, FK}, upd_rows_bf16_kernel<R, S, WC, WK, WP, FC, FK>       \
    }
#define UPD_ROWS_ENTRY_STRIDED(R, S, WC, WK, WP, FC, FK)                                 \
    {                                                                                    \
        {R, S, WC, WK, WP, FC, FK, 1}, upd_rows_bf16_kernel<R, S, WC, WK, WP, FC, FK, true>    \
    }
static UpdRowsEntry g_rows[] = {
    UPD_ROWS_ENTRY(3, 3, 2, 4, 1, 1, 1),  // 64 x 128 channels, eight waves
    UPD_ROWS_ENTRY(3, 3, 2, 2, 2, 1, 1),  // 64 x 64 channels, two wave groups along pixels
    // one-row and one-column filters (factorised 7x7 and 3x3), the same two tiles
    UPD_ROWS_ENTRY(1, 7, 2, 4, 1, 1, 1),
    UPD_ROWS_ENTRY(1, 7, 2, 2, 2, 1, 1),
    UPD_ROWS_ENTRY(7, 1, 2, 4, 1, 1, 1),
    UPD_ROWS_ENTRY(7, 1, 2, 2, 2, 1, 1),
    UPD_ROWS_ENTRY(1, 3, 2, 4, 1, 1, 1),
    UPD_ROWS_ENTRY(1, 3, 2, 2, 2, 1, 1),
    UPD_ROWS_ENTRY(3, 1, 2, 4, 1, 1, 1),
    UPD_ROWS_ENTRY(3, 1, 2, 2, 2, 1, 1),
    // one row of a 5x5 filter per launch
    UPD_ROWS_ENTRY(1, 5, 2, 4, 1, 1, 1),
    UPD_ROWS_ENTRY(1, 5, 2, 2, 2, 1, 1),
    // 3x3 with stride > 1 (per-tap strided operands)
    UPD_ROWS_ENTRY_STRIDED(3, 3, 2, 4, 1, 1, 1),
    UPD_ROWS_ENTRY_STRIDED(3, 3, 2, 2, 2, 1, 1),
    // 1x1 (input staged sampled): channel tiles TC x TK
    UPD_ROWS_ENTRY(1, 1, 2, 2, 2, 1, 1),  //  64 x  64
    UPD_ROWS_ENTRY(1, 1, 2, 4, 1, 1, 1),  //  64 x 128
    UPD_ROWS_ENTRY(1, 1, 4, 2, 1, 1, 1),  // 128 x  64
    UPD_ROWS_ENTRY(1, 1, 2, 4, 1, 1, 2),  //  64 x 256
    UPD_ROWS_ENTRY(1, 1, 4, 2, 1, 2, 1),  // 256 x  64
    UPD_ROWS_ENTRY(1, 1, 2, 4, 1, 2, 2),  // 128 x 256
    UPD_ROWS_ENTRY(1, 1, 4, 2, 1, 2, 2),  // 256 x 128
};

static UpdRowsEntry *find_rows(const UpdRowsVariant &v)
{
    for (auto &e : g_rows)
        if (e.v.r == v.r && e.v.s == v.s && e.v.wc == v.wc && e.v.wk == v.wk && e.v.wp == v.wp &&
            e.v.fc == v.fc && e.v.fk == v.fk && e.v.strided == v.strided)
            return &e;
    return nullptr;
}
bool upd_rows_variant_exists(const UpdRowsVariant &v) { return find_rows(v) != nullptr; }

hipError_t launch_upd_rows(const UpdRowsVariant &v, const UpdArgs &a, size_t lds_bytes, int grid,
                           hipStream_t stream)
{
    UpdRowsEntry *e = find_rows(v);
    if (!e) return hipErrorInvalidDeviceFunction;
    if (hipError_t err = ensure_dynamic_lds(reinterpret_cast<const void *>(e->fn), lds_bytes);
        err != hipSuccess)
        return err;
    hipLaunchKernelGGL(e->fn, dim3(grid), dim3(v.wc * v.wk * v.wp * 64), lds_bytes, stream, a);
    return hipGetLastError();
}

}  // namespace convmi
