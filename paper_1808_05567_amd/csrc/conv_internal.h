// Internal declarations shared by the translation units of libconv_mi355x.
// Not part of the public ABI (that is include/conv_mi355x.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include <type_traits>

#include "conv_mi355x.h"

namespace convmi {

// ---------------------------------------------------------------------------
// Arguments of the implicit-GEMM kernel that serves the forward pass and, via
// the two duality scenarios of Section II-I, the backward-by-data pass.
//
//   out[n][kb][oy][ox][:] = sum_{cb,r,s,c} in[n][cb][oy*stride-pad_h+r][ox*stride-pad_w+s][c]
//                                          * wt[cb][r][s][k][c]
//
// M = output channels (weights are the MFMA A operand), N = output pixels
// (the staged input tile is the B operand), reduction = (channel block, r, s):
// the paper's M^=k, N^=pixels, K^=c small-GEMM chain (Section II-D) at
// workgroup scale.
// ---------------------------------------------------------------------------
struct IgemmArgs {
    const void *in;
    const void *wt;
    void *out;
    int N;
    int Cb;        // input channel blocks (reduction planes)
    int H, W;      // input extent
    int Kp;        // output channels rounded up to vlen (rows of A)
    int P, Q;      // extent of the convolution result
    int stride, pad_h, pad_w;
    int cstride;   // input pixels between consecutive result columns (== stride, except where a
                   // column of the result stands for several cells of a strided backward pass)
    int OH, OW;    // extent of the output tensor (== P,Q unless scattering)
    int ostr;      // result pixel (oj,oi) is written at (oj*ostr+oy0, oi*ostr_x+ox0)
    int ostr_x;    // (== ostr, except as for cstride)
    int oy0, ox0;
    int zero_fill; // ostr>1: also write zeros to the other positions of each ostr x ostr cell
    int shuffle;   // ostr>1: result channel block b is position (b / ostr_x, b % ostr_x) of the
                   // ostr x ostr_x cell of an output tensor with ONE channel block
    int out_kb;    // channel blocks of the output tensor
    int TR, TQ;    // tile = TR linear output rows (n*P+oj) x TQ columns
    int n_qt;      // column tiles
    int n_mt;      // row tiles
    int n_kt;      // output-channel tiles
    int Hs;        // rows per image in the padded row space of the staged tile
    int LW;        // staged tile width  (pixels)
    int LRW;       // staged tile size   (pixels) = rows * LW
    int PLS;       // LDS plane pitch    (16-byte units)
    int sampled;   // R=S=1, pad=0: stage only the pixels that are read
    int live_ch;   // channel slots of an input block that can be non-zero: min(C, slots per block)
                   // with one channel block, else all of them (the rest is zero padding on both sides)
    // 1.0f / P, Hs, LW, TQ for the kernel's exact small divisions (see fast_div)
    float inv_P, inv_Hs, inv_LW, inv_TQ;
    int total;     // workgroups doing work
    int per_xcd;   // workgroups per XCD (the grid is 8 * per_xcd)
    int jstep;     // resident-filter kernel only: workgroups per XCD of its launch; a workgroup
                   // takes pixel tiles j, j + jstep, ... of its XCD (set at launch)
    // Tiles over the 8 XCDs: gk channel groups of kt_per channel tiles x 8/gk pixel groups
    // of mq_per pixel tiles (per_xcd = kt_per * mq_per); unused when the reduction is split
    int gk, kt_per, mq_per;
    // Channel tile kt of pixel tile mq starts its reduction at step
    // (kt * rot_k + mq * rot_m) mod (its number of steps) and wraps round (0, 0: all start at 0)
    int rot_k, rot_m;
    int n_stage;   // ceil(Cb / planes per stage)
    // Reduction split (few tiles, long reduction): workgroup lin covers tile
    // lin % total and reduction steps [sp*st_per, (sp+1)*st_per), sp = lin / total,
    // and writes an fp32 partial result, copy sp, for split_reduce to sum.
    int ksplit;    // number of splits (1: none, the result is written directly)
    int st_per;    // reduction steps per split
    // Operators fused into the store of the result (forward pass only)
    const float *scale; // per output channel row, Kp entries, multiplies the result, or null
    const float *bias;  // per output channel row, Kp entries, or null
    const void *resid;  // tensor of the output's layout and type added to the result, or null
    int relu;           // clamp at zero after the additions
};

// Optional geometry of a plan beyond the plain convolution's (0: as the strides say).
struct IgemmGeo {
    int cstride = 0;  // IgemmArgs::cstride
    int ostr_x = 0;   // IgemmArgs::ostr_x
};

// Key of a kernel instantiation; the host picks one per pass at plan time.
struct IgemmVariant {
    int dtype;   // conv_dtype_t
    int wk, wm;  // waves along channels / pixels
    int fk, fm;  // 32x32 MFMA fragments per wave along channels / pixels
    int npl;     // reduction planes (channel blocks) staged per step
    int r, s;    // filter extent
    int ppt;     // staged input pixels per thread
    int nb = 2;  // LDS buffers of the staging ring
    int nt = 0;  // 1: the input tile is loaded non-temporally (plans with one channel tile)
};

// Raise a kernel's dynamic-LDS limit to at least `bytes` (once per kernel and size; safe to
// call from several host threads, whatever handles they use).
hipError_t ensure_dynamic_lds(const void *kernel, size_t bytes);

hipError_t launch_igemm(const IgemmVariant &v, const IgemmArgs &a, size_t lds_bytes,
                        int grid, hipStream_t stream);
bool igemm_variant_exists(const IgemmVariant &v);
// The resident-filter kernel for first layers (one channel block in, one reduction step, one
// channel tile): LDS it needs for the plan, 0 if it does not serve it; and its launch (plain
// store only: no fused operators).
size_t igemm_stem_lds(const IgemmVariant &v, const IgemmArgs &a);
hipError_t launch_igemm_stem(const IgemmVariant &v, const IgemmArgs &a, size_t lds_bytes, hipStream_t stream);
// out[e] = sum over copies j (ascending) of partial[j][e], converted to the tensor's type
// Fused operators (null / 0: none): scale[channel], bias[channel], residual (output
// layout), ReLU; pq = pixels per image, kb = channel blocks, for the channel of an element.
hipError_t launch_split_reduce(int dtype, const float *partial, void *out, size_t n_elems, int copies,
                               const float *scale, const float *bias, const void *resid, int relu,
                               int pq, int kb, hipStream_t stream);

// Weight transform for backward by data:  dst[kb][r'][s'][c][k%v] (tap-flipped,
// channel roles swapped, optionally a stride-decimated sub-filter).
struct WtXformArgs {
    const void *src;   // Wb[Cb][R][S][Kp][v]
    void *dst;         // [Kb][R2][S2][Cp][v]
    int Cb, Kb, Cp, Kp, R, S, R2, S2;
    int tap_stride;    // source tap r = tap_stride*(Rsub-1-r') + r_off, valid if r' < Rsub
    int r_off, s_off, Rsub, Ssub;
};
hipError_t launch_wt_xform(int dtype, const WtXformArgs &a, hipStream_t stream);

// Weight transform for a strided backward pass whose dI has one channel block:
// the sub-filters of all stride-parity classes side by side as the rows of ONE
// filter over a common window,  dst[kb][u][v][cls*V + c][k%V],  cls = py*st + px.
// Class row index py uses window rows u with r2 = u - rsh[py] in [0, rsub[py]),
// source tap r = st*(rsub[py]-1-r2) + roff[py]; columns likewise.
struct WtMergeArgs {
    const void *src;  // Wb[1][R][S][Kp][v]
    void *dst;        // [Kb][R2][S2][cells*st*st*v][v]
    int Kb, Kp, R, S, R2, S2, st;
    // Cells per column of the result (1 or 2).  With 2, row block (py, e, px) holds class
    // (py, px) of cell e of a pair of cells side by side, its taps e columns to the right in
    // a window S2 = (the classes' common window) + 1 wide.
    int cells;
    int rsub[4], roff[4], rsh[4];
    int ssub[4], soff[4], ssh[4];
};
hipError_t launch_wt_merge(int dtype, const WtMergeArgs &a, hipStream_t stream);

// Weight update (Algorithm 8): partial sums over slices of the pixel range,
// then a fixed-order reduction.
struct UpdArgs {
    const void *in;
    const void *dout;
    float *partial;  // [splits][Cb][R][S][Kp][v] fp32
    int N, Cb, H, W, Kb, Kp, P, Q, R, S, stride;
    int pad;         // rows of zero padding above the image (may be negative: a launch that
                     // serves one filter row r of a taller filter runs with pad_h - r)
    int pad_w;       // columns of zero padding left of the image
    // The launch computes taps [tap0, tap0 + R*S) of a filter with ntaps_all taps: the
    // partial dW copies have the full filter's layout [Cb][ntaps_all][Kp][v].
    int tap0, ntaps_all;
    // General kernels only: the launch serves the strip of Q output columns that starts at
    // column q0 of rows Qpitch wide (image columns from q0*stride on), and writes partial
    // copies copy0 .. copy0+splits-1.  One strip: q0 = 0, Qpitch = Q, copy0 = 0.
    int q0, Qpitch, copy0;
    int TR;          // linear output rows per staged step
    int rows_per_split;
    int splits;
    int n_ct, n_kt;  // tiles over input / output channels
    int Hs, LW, LRW, PLS_in, PLS_out;
    int sampled;
    int total, per_xcd;
    int live_ch;     // few-channel fp32 kernel: input channels that exist (1..4)
    int runs;        // bf16 row kernel: 8-pixel runs per output row
    int Qp;          // fp32 kernel: row pitch of the staged dO band (pixels)
};
struct UpdVariant {
    int dtype;
    int r, s;
    int wc, wk;            // waves along input / output channels
    int fc, fk;            // 32x32 fragments per wave along input / output channels
    int ppt_in, ppt_out;   // bf16: staged 16-byte chunks per thread (input band, dO band);
                           // fp32: plane groups of the staging map (input band, dO band)
};
hipError_t launch_upd(const UpdVariant &v, const UpdArgs &a, size_t lds_bytes, int grid,
                      hipStream_t stream);
bool upd_variant_exists(const UpdVariant &v);
// bf16, stride 1 (or 1x1 sampled): 8-pixel runs along a row, filter-column shifts in registers
struct UpdRowsVariant {
    int r, s;
    int wc, wk, wp;  // waves along input channels / output channels / pixels
    int fc, fk;      // 32x32 fragments per wave along input / output channels
    int strided;     // 1: stride > 1 with a filter larger than 1x1 (an operand read per tap)
};
bool upd_rows_variant_exists(const UpdRowsVariant &v);
hipError_t launch_upd_rows(const UpdRowsVariant &v, const UpdArgs &a, size_t lds_bytes, int grid,
                           hipStream_t stream);
// fp32, filters larger than 1x1: eight waves, double-buffered bands
bool upd_f32_bands_exists(int r, int s);
// layout: 0 = 2 x 2 channel waves x 2 pixel groups, 1 = 1 x 2 x 4, 2 = 1 x 1 x 8
bool upd_f32_bands_layout_exists(int r, int s, int layout, bool odd_rows);
size_t upd_f32_bands_exchange_bytes(int r, int s, int layout);
hipError_t launch_upd_f32_bands(int r, int s, int layout, const UpdArgs &a, size_t lds_bytes, int grid,
                                hipStream_t stream);
// bf16, 1x1 without padding: eight waves on the flat pixel list, bands of 64 pixels
// (UpdArgs::rows_per_split = pixels per split, a multiple of 64)
bool upd_bf16_1x1_variant_exists(const UpdRowsVariant &v);
size_t upd_bf16_1x1_lds_bytes(const UpdRowsVariant &v);
hipError_t launch_upd_bf16_1x1(const UpdRowsVariant &v, const UpdArgs &a, int grid, hipStream_t stream);
// fp32, 1x1 without padding, at least 256 channels on one side: eight waves, 256 x (64*wb)
// channel tile, bands of 32 pixels of the flat pixel list (UpdArgs::rows_per_split = pixels
// per split, a multiple of 32; n_ct / n_kt = tiles over input / output channels)
size_t upd_f32_1x1_lds_bytes(int wb);
hipError_t launch_upd_f32_1x1(int wb, bool a_is_in, const UpdArgs &a, int grid, hipStream_t stream);
// at most 4 input channels: filter-row formulation, 7x7 and 3x3; fp32 tensors, or bf16
// tensors widened on their way into LDS (then UpdArgs::Kb counts blocks of 8 channels)
hipError_t launch_upd_c4(int dtype, int r, int s, const UpdArgs &a, size_t lds_bytes, int grid,
                         hipStream_t stream);
// bf16 tensors, at most 4 input channels: the same formulation on the bf16 MFMA
bool upd_c4_bf16_exists(int r, int s);
hipError_t launch_upd_c4_bf16(int r, int s, const UpdArgs &a, size_t lds_bytes, int grid,
                              hipStream_t stream);
hipError_t launch_upd_reduce(const float *partial, float *dwt, size_t n_elems, int splits,
                             hipStream_t stream);

// Untiled direct kernels for descriptors outside the tiled kernels' reach: any filter,
// stride and per-axis pad.  x / wt / y are (input, weights, output) for the forward pass,
// (dO, weights, dI) for backward by data and (input, dO, fp32 dW) for the update.
struct DirectArgs {
    const void *x;
    const void *wt;
    void *y;
    int N, Cb, Kb, H, W, P, Q, R, S, stride, pad_h, pad_w;
    // forward only: operators applied to the result (null / 0: none)
    const float *scale;
    const float *bias;
    const void *resid;
    int relu;
};
// whether the grids of the three passes fit the launch limits
bool direct_fits(int dtype, int N, int Cb, int Kb, int H, int W, int P, int Q, int R, int S);
hipError_t launch_direct_fwd(int dtype, const DirectArgs &a, hipStream_t stream);
hipError_t launch_direct_bwd(int dtype, const DirectArgs &a, hipStream_t stream);
hipError_t launch_direct_upd(int dtype, const DirectArgs &a, hipStream_t stream);

// Layout conversion (pure permutations).
hipError_t launch_pack_act(int dtype, const void *nchw, void *blk, int N, int C, int H, int W,
                           hipStream_t stream);
hipError_t launch_unpack_act(int dtype, const void *blk, void *nchw, int N, int C, int H, int W,
                             hipStream_t stream);
hipError_t launch_pack_wt(int dtype, const void *kcrs, void *blk, int K, int C, int R, int S,
                          hipStream_t stream);
hipError_t launch_unpack_wt(int dtype, const void *blk, void *kcrs, int K, int C, int R, int S,
                            int vlen, hipStream_t stream);

// Exact floor(x / d) for 0 <= x < 2^22 with inv = 1.0f / d: (x + 0.5) / d is
// never an integer and stays 0.5/d away from one, more than the rounding error.
static __device__ __forceinline__ int fast_div(int x, float inv)
{
    return (int)(((float)x + 0.5f) * inv);
}

// Product of two integers that each fit 24 bits (signed): one full-rate instruction where
// a 32-bit multiply takes four.  The planner bounds every operand it is used on.
// `u` must be wave-uniform (a kernel argument or derived from one): it rides in a scalar register.
static __device__ __forceinline__ int mul24(int a, int u)
{
    int r;  // (spelled out: the compiler turns the library's 24-bit multiply back into a 32-bit one)
    asm("v_mul_i32_i24 %0, %1, %2" : "=v"(r) : "s"(u), "v"(a));
    return r;
}

// Buffer addressing: a tensor is reached through a buffer resource
// (base, byte size) plus a 32-bit per-lane byte offset.  Loads whose offset is
// at or beyond the size return zero and stores there are dropped, so padding
// and ragged tiles need no branches: such lanes carry the offset kOutOfRange.
// A wave-uniform byte offset (channel block, reduction step) rides in the
// scalar offset of the instruction; the range check covers the sum.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
constexpr unsigned kOutOfRange = 0xFFFFFFFFu;
static __device__ __forceinline__ rsrc_t make_rsrc(const void *base, size_t skip, size_t total)
{
    // view of [base + skip, base + total); the range check stays exact
    return __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char *>(static_cast<const char *>(base)) + skip, 0,
        (int)(unsigned)(total - skip), 0x00020000);
}
// 16-byte load from global memory straight into LDS: lane i of the wave writes
// lds_wave_base + 16*i (the LDS base must be wave-uniform), zero if out of range.
// POLICY: cache policy bits of the load (0: default; 2: non-temporal -- the line is the first
// to leave the L2, for data that streams past once and must not push out what is re-read).
template <int POLICY = 0>
static __device__ __forceinline__ void load_to_lds_16(rsrc_t r, unsigned byte_off,
                                                      unsigned uniform_off,
                                                      unsigned char *lds_wave_base)
{
    typedef __attribute__((address_space(3))) void *lds_vptr_t;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_vptr_t)lds_wave_base, 16, byte_off, uniform_off,
                                             0, POLICY);
}
// Transposing 64-bit LDS reads the compiler does not track.  Before a transposing read issued
// through its builtin the compiler waits for EVERY outstanding load of the wave, loads that
// write straight into LDS included (it cannot tell that they fill the other buffer; before
// ordinary LDS reads it places no such wait) -- a band's prefetch would be awaited in the
// instruction after it was issued.  These reads are plain instructions to the compiler
// instead: the caller waits for them with lds_reads_pending<N>() (LDS operations of a wave
// complete in order: "at most N still pending") and then passes every register they wrote
// through lds_read_landed(), which pins each use of the value behind that wait.
// Within a group of 16 lanes, lane i slot j receives 16-bit element (i % 4) of the 8 bytes
// addressed by lane 4*j + i/4.  `addr` is the LDS byte address, OFF a constant added to it.
typedef unsigned int lds_u32x2 __attribute__((ext_vector_type(2)));
static __device__ __forceinline__ unsigned lds_address(const unsigned char *p)
{
    return (unsigned)(size_t)(const __attribute__((address_space(3))) unsigned char *)p;
}
template <int OFF>
static __device__ __forceinline__ lds_u32x2 lds_read_tr16_b64_untracked(unsigned addr)
{
    static_assert(OFF >= 0 && OFF < 65536, "16-bit offset field");
    lds_u32x2 v;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}
template <int N>
static __device__ __forceinline__ void lds_reads_pending()
{
    // (the counter has four bits: a count it cannot hold waits for everything)
    asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N <= 15 ? N : 0));
}
static __device__ __forceinline__ void lds_read_landed(lds_u32x2 &v) { asm volatile("" : "+v"(v)); }
// Compile-time loop: f(std::integral_constant<int, I>) for I in [I0, I1).
template <int I0, int I1, class F>
static __device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I0 < I1) {
        f(std::integral_constant<int, I0>{});
        static_for<I0 + 1, I1>(f);
    }
}
// Cache policy of the loads of the update kernels, which read both tensors exactly once:
// non-temporal (the lines are not kept in the last-level cache and leave the L2 first).
#ifndef CONVMI_UPD_POLICY
#define CONVMI_UPD_POLICY 2
#endif
// Wait until every outstanding memory operation of this wave, staging loads included, is done.
static __device__ __forceinline__ void wait_all_memory() { __builtin_amdgcn_s_waitcnt(0); }

static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
static inline int vlen_of(int dtype) { return dtype == CONV_BF16 ? 8 : 4; }
static inline int esize_of(int dtype) { return dtype == CONV_BF16 ? 2 : 4; }

}  // namespace convmi
