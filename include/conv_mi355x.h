/*
 * conv_mi355x.h -- C ABI of the MI355X (gfx950) direct-convolution library.
 *
 * The three training passes of a 2-D convolution layer, after "Anatomy Of
 * High-Performance Deep Learning Convolutions On SIMD Architectures"
 * (Section II): forward (Algorithm 1), backward by data (Algorithm 6) and
 * weight-gradient update (Algorithm 8), computed directly (no im2col buffer)
 * over channel-blocked tensors (Section II-B, Algorithm 2), with padding added:
 *
 *   input position of output (oj,oi), tap (r,s):  ij = stride*oj - pad + r,
 *                                                 ii = stride*oi - pad + s,
 *   terms whose (ij,ii) lies outside the image are zero;
 *   P = floor((H + 2 pad - R)/stride) + 1,  Q likewise.
 *
 * Conventions common to every entry point
 *   - All tensor pointers are DEVICE pointers, 16-byte aligned, allocated and
 *     owned by the caller.  The library never allocates or frees device
 *     memory and keeps no pointer after a call returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work; they never synchronise.  Errors raised by the
 *     device asynchronously surface at the caller's next synchronisation.
 *   - Outputs are overwritten (the "+=" of the printed loops starts from 0).
 *   - A handle owns only a host-side plan.  One handle may be used from one
 *     host thread at a time.
 *   - Every function returns a conv_status_t; nothing is ever computed by
 *     another library or on the host as a fallback.
 *
 * Blocked layouts (v = 16 bytes / element size: 4 for fp32, 8 for bf16; the
 * role the paper's VLEN plays for a 512-bit SIMD register is played here by
 * the 128-bit per-lane vector that feeds one MFMA operand):
 *   activations   X[N][Cb][H][W][v]        Cb = ceil(C / v), channel c lives in
 *                                          block c / v at slot c % v; slots
 *                                          beyond C hold zeros
 *   weights       Wb[Cb][R][S][Kp][v]      Kp = K rounded up to v; element
 *                                          (k, c, r, s) at [c/v][r][s][k][c%v]
 *   weight grads  same index structure as Wb, element type always fp32
 * Callers should not hard-code these; conv_query reports sizes, and the pack /
 * unpack entry points convert from and to the logical layouts I[N][C][H][W],
 * W[K][C][R][S], O[N][K][P][Q] of Section II.
 */
#ifndef CONV_MI355X_H
#define CONV_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CONV_F32 = 0,  /* fp32 tensors, fp32 MFMA accumulation                      */
    CONV_BF16 = 1  /* bf16 activations/weights/gradients, fp32 accumulation,
                      bf16 outputs for fwd/bwd_data, fp32 weight gradients      */
} conv_dtype_t;

typedef enum {
    CONV_OK = 0,
    CONV_EINVAL = 1,       /* NULL pointer, non-positive extent, negative pad,
                              empty output, unknown dtype, misaligned pointer  */
    CONV_EUNSUPPORTED = 2, /* valid problem beyond the library's size limits   */
    CONV_EWORKSPACE = 3,   /* workspace required but ws == NULL, or (the _ws
                              entry points) smaller than the pass needs        */
    CONV_ELAUNCH = 4,      /* the HIP runtime refused a launch                 */
    CONV_ESCRATCH = 5      /* conv_bwd_data_noalloc: the pass needs more scratch
                              than the library's static device buffer holds    */
} conv_status_t;

/* Problem statement (Section II notation).  One stride and one pad for both
 * spatial axes; no dilation, groups or bias (the paper has none). */
typedef struct {
    int32_t N, C, K, H, W, R, S, stride, pad;
    int32_t dtype; /* conv_dtype_t */
} conv_desc_t;

typedef struct {
    int32_t P, Q;           /* output extent                                  */
    int32_t vlen;           /* v above                                         */
    int32_t Cb, Kb;         /* channel blocks of the input / output tensors    */
    int32_t Cp, Kp;         /* C, K rounded up to vlen                         */
    size_t in_bytes;        /* blocked I / dI                                  */
    size_t out_bytes;       /* blocked O / dO                                  */
    size_t wt_bytes;        /* blocked W                                       */
    size_t dwt_bytes;       /* blocked dW (fp32)                               */
    size_t workspace_bytes; /* max over the three passes; may be 0             */
    int32_t upd_splits;     /* partial dW copies summed by conv_upd            */
    int32_t reserved;
} conv_info_t;

typedef struct conv_plan *conv_handle_t;

/* Host only: validate the descriptor and plan every pass -- kernel variant, tile
 * shape, grid, LDS size, the split of the weight update -- once per layer.  This is
 * the role of the paper's set-up: the dryrun phase of the kernel streams
 * (Section II-H), which walks the loops once to record what each thread will
 * run, and the division of the work items over the threads (Section II-F); the
 * pass entry points below are the replay phase and only launch.
 * Errors: CONV_EINVAL for a NULL pointer, an extent < 1, a negative pad, an
 * unknown dtype, or an empty output (H + 2 pad < R or W + 2 pad < S);
 * CONV_EUNSUPPORTED beyond the size limits: N, C, K, H, W <= 2^24; R, S, stride,
 * pad <= 2^16; at most 2^39 elements per activation tensor and 2^31 - 1 per
 * weight tensor (channels rounded up to the block).  On success *out owns a
 * host-side plan (no device memory) until conv_destroy. */
conv_status_t conv_create(const conv_desc_t *desc, conv_handle_t *out);
/* As conv_create, with one pad per axis (desc->pad is ignored):
 *     ij = stride*oj - pad_h + r,  ii = stride*oi - pad_w + s,
 *     P = floor((H + 2 pad_h - R)/stride) + 1,  Q = floor((W + 2 pad_w - S)/stride) + 1,
 * the same reading of padding applied to each axis on its own.  It serves the 1xS and
 * Rx1 filters of Inception-style layers, which pad along their long side only (the paper
 * reports averages over such a topology next to ResNet-50, Section III).  Everything else
 * is as for conv_create: CONV_EINVAL for a negative pad or an empty output.
 * Every accepted descriptor has all three passes.  Filters the tiled MFMA kernels are
 * instantiated for (1x1, 3x3, 5x5, 1x3, 3x1, 1x7, 7x1, and 7x7 where a staged tile fits
 * the LDS) run on those; any other filter, stride or row width runs the plain loop nests of
 * Algorithms 1, 6 and 8, one result element per thread, at a small fraction of that rate
 * (conv_describe names the kernel: "direct ...").  CONV_EUNSUPPORTED is left for the size
 * limits listed at conv_create. */
conv_status_t conv_create_rect(const conv_desc_t *desc, int32_t pad_h, int32_t pad_w,
                               conv_handle_t *out);
/* As conv_create_rect, with the minibatch run in chunks of at most max_images images
 * (>= 1; CONV_EINVAL otherwise): every pass launches its kernels once per chunk on that
 * chunk's slice of the tensors (images are independent in Algorithms 1 and 6; Algorithm 8
 * sums over them, so conv_upd writes one dW per chunk into the workspace and adds them in
 * chunk order: still one fixed order).  The tensors, their layouts and every entry point
 * stay the same; conv_query reports the workspace the chunked plan needs.  It bounds the
 * workspace of large minibatches.  conv_create and conv_create_rect choose chunks by
 * themselves in one case only: tensors of 4 GB or more, which the tiled kernels' 32-bit
 * byte offsets do not reach in one launch. */
conv_status_t conv_create_chunked(const conv_desc_t *desc, int32_t pad_h, int32_t pad_w,
                                  int32_t max_images, conv_handle_t *out);
/* Free the host-side plan (the end of the set-up's lifetime, Section II-H; no device
 * memory is involved).  CONV_EINVAL for NULL. */
conv_status_t conv_destroy(conv_handle_t h);
/* Output extent (P, Q as defined above), channel blocking (the VLEN blocking of
 * Section II-B) and the byte sizes of the blocked tensors and of the workspace.
 * CONV_EINVAL for a NULL argument. */
conv_status_t conv_query(conv_handle_t h, conv_info_t *info);
/* Static text for a status code; never NULL. */
const char *conv_status_str(conv_status_t s);

/* Workspace.  conv_fwd, conv_bwd_data and conv_upd take `ws`, a device buffer of at least
 * conv_info_t::workspace_bytes (the maximum over the three passes).  They cannot see its
 * size: a buffer smaller than that is written past its end.  Callers that want the size
 * checked use conv_fwd_ws / conv_bwd_data_ws / conv_upd_ws below, which take ws_bytes and
 * return CONV_EWORKSPACE (nothing is launched) when it is smaller than what that pass
 * of this plan needs. */

/* Algorithm 1 with padding:  out[n,k,oj,oi] = sum_{c,r,s} in[n,c,ij,ii] * wt[k,c,r,s].
 * in: blocked I; wt: blocked W; out: blocked O (fully overwritten, padded
 * channel slots written as zero).  ws: workspace_bytes of scratch; read only by
 * plans that split the reduction over workgroups (few output tiles, e.g. N = 1:
 * fp32 partial results summed in a fixed order), CONV_EWORKSPACE if such a plan
 * gets NULL; other plans ignore it. */
conv_status_t conv_fwd(conv_handle_t h, const void *in, const void *wt, void *out,
                       void *ws, void *stream);

/* Forward pass with fused operators (Section II-G, Algorithm 4: APPLY(L(), O
 * sub-tensor) once the sub-tensor's reduction is complete -- here while it is
 * still in registers):
 *     out[n,k,oj,oi] = L( scale[k] * conv[n,k,oj,oi] + bias[k] + residual[n,k,oj,oi] )
 * with L(x) = max(x, 0) if relu != 0, else the identity; the sum and L are
 * evaluated in fp32 before the one rounding to the output type.  scale and bias
 * together are a normalisation layer applied with given statistics (the
 * "Normalization" and "Bias" layers Section II-G names), residual + relu the
 * element-wise tail of a residual block.
 * scale: device, fp32, Kp entries, or NULL (= 1).
 * bias: device, fp32, Kp entries (entries of padded channels must be 0), or NULL.
 * residual: device, blocked O layout and the tensors' dtype, or NULL; it may
 * alias out (each element is read before it is written, by the same lane).
 * Everything else as conv_fwd; with scale == bias == residual == NULL and
 * relu == 0 the two calls give identical results. */
conv_status_t conv_fwd_fused_norm(conv_handle_t h, const void *in, const void *wt, void *out,
                                  const float *scale, const float *bias, const void *residual,
                                  int32_t relu, void *ws, void *stream);

/* The same without the scale (scale[k] = 1). */
conv_status_t conv_fwd_fused(conv_handle_t h, const void *in, const void *wt, void *out,
                             const float *bias, const void *residual, int32_t relu, void *ws,
                             void *stream);

/* Algorithm 6 with padding:  din[n,c,ij,ii] = sum_{k,r,s} dout[n,k,oj,oi] * wt[k,c,r,s]
 * over all (oj,r), (oi,s) that map to (ij,ii); positions no term maps to are 0.
 * dout: blocked dO; wt: blocked W (the same buffer conv_fwd takes); din: blocked
 * dI, fully overwritten.  ws: workspace_bytes of scratch (holds the transposed,
 * tap-flipped weights of the duality of Section II-I). */
conv_status_t conv_bwd_data(conv_handle_t h, const void *dout, const void *wt, void *din,
                            void *ws, void *stream);

/* conv_bwd_data for callers that cannot allocate device memory or carry a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same operation, arguments, kernels and results as conv_bwd_data, without `ws`: the
 * scratch (the transposed, tap-flipped weights) lives in a static device array of
 * conv_noalloc_scratch_bytes() = 16 MiB that the library's code object brings along
 * (every GPU the library runs on holds its own copy until the process ends).  The call
 * allocates nothing and frees nothing.
 *   - A plan whose backward pass needs more scratch returns CONV_ESCRATCH before anything
 *     is launched (all layers of Table I fit: at most 9.4 MB, layer 18 in fp32).
 *   - The array keeps the previous call's contents; nothing has to start at zero, because
 *     the weight transform writes every byte the convolution kernel then reads.
 *   - All calls on one GPU share the one array: calls that may overlap on a GPU (different
 *     streams, different host threads) race on it.  Serialise them, or use conv_bwd_data
 *     with a workspace per stream.
 *   - The array's address is looked up on the first call on each device (the device that
 *     is current at the call); CONV_ELAUNCH if the runtime cannot provide it. */
conv_status_t conv_bwd_data_noalloc(conv_handle_t h, const void *dout, const void *wt, void *din,
                                    void *stream);
/* Size of that static scratch array in bytes. */
size_t conv_noalloc_scratch_bytes(void);

/* Algorithm 8 with padding:  dwt[k,c,r,s] = sum_{n,oj,oi} in[n,c,ij,ii] * dout[n,k,oj,oi].
 * in: blocked I; dout: blocked dO; dwt: blocked dW, fp32, fully overwritten.
 * ws: workspace_bytes of scratch (partial dW copies over slices of the
 * minibatch/pixel range, summed in a fixed order: results are deterministic). */
conv_status_t conv_upd(conv_handle_t h, const void *in, const void *dout, void *dwt,
                       void *ws, void *stream);

/* The three passes with the workspace size checked (see "Workspace" above); otherwise
 * identical to conv_fwd, conv_bwd_data and conv_upd. */
conv_status_t conv_fwd_ws(conv_handle_t h, const void *in, const void *wt, void *out, void *ws,
                          size_t ws_bytes, void *stream);
conv_status_t conv_bwd_data_ws(conv_handle_t h, const void *dout, const void *wt, void *din,
                               void *ws, size_t ws_bytes, void *stream);
conv_status_t conv_upd_ws(conv_handle_t h, const void *in, const void *dout, void *dwt, void *ws,
                          size_t ws_bytes, void *stream);

/* Layout conversion (Algorithm 2's blocked layouts, Section II-B), pure permutations in the tensor's own element type
 * (dW: fp32).  "nchw"/"kcrs" are the logical layouts, "blk" the blocked ones. */
conv_status_t conv_pack_in(conv_handle_t h, const void *nchw, void *blk, void *stream);
conv_status_t conv_pack_out(conv_handle_t h, const void *nkpq, void *blk, void *stream);
conv_status_t conv_pack_wt(conv_handle_t h, const void *kcrs, void *blk, void *stream);
conv_status_t conv_unpack_in(conv_handle_t h, const void *blk, void *nchw, void *stream);
conv_status_t conv_unpack_out(conv_handle_t h, const void *blk, void *nkpq, void *stream);
conv_status_t conv_unpack_wt(conv_handle_t h, const void *blk, void *kcrs, void *stream);
conv_status_t conv_unpack_dwt(conv_handle_t h, const void *blk_f32, void *kcrs_f32, void *stream);

/* Name, launch geometry and dynamic LDS bytes of the kernel a pass would
 * launch (pass: 0 fwd, 1 bwd_data, 2 upd): what the set-up decided (Section II-H's
 * dryrun record, in readable form); for benchmarks and profiles.  buf receives a
 * NUL-terminated string of at most buflen bytes.  CONV_EINVAL for NULL / buflen 0 /
 * an unknown pass, CONV_EUNSUPPORTED if the pass has no kernel. */
conv_status_t conv_describe(conv_handle_t h, int32_t pass, char *buf, size_t buflen);

/* Measured ceilings of the device, for the roofline columns of a benchmark (Section III
 * quotes kernel rates against the machine's peak; these loops measure what part of a
 * published peak this device sustains on a loop that does nothing else).  They only
 * launch: the caller owns every buffer and times the launch with events on `stream`.
 * None of them is part of the convolution path.
 *
 * conv_ceiling_mfma: `blocks` workgroups of 4 waves, each wave issuing `iters` rounds of
 *   eight independent 32x32 MFMAs of the type (fp32: 32x32x2, bf16: 32x32x16) from
 *   registers.  Flops = blocks * 4 * iters * 8 * 2*32*32*k, k = 2 (fp32) or 16 (bf16).
 *   sink: device, blocks * 256 floats, written once (keeps the loop alive).
 * conv_ceiling_copy: dst[0, bytes) = src[0, bytes), 16 bytes per lane, non-temporal loads
 *   and stores (as the convolution kernels issue them for tensors that stream past once);
 *   device pointers, 16-byte aligned, bytes a multiple of 16.  HBM traffic = 2 * bytes.
 * conv_ceiling_read / conv_ceiling_write: the read half and the write half of that copy on
 *   their own (read: sink receives 8192 * 256 words at most, device, at least that large;
 *   write: dst is overwritten with a pattern).  HBM traffic = bytes.
 * conv_ceiling_l2_to_lds: `blocks` workgroups of 4 waves, each streaming its own 96 KiB
 *   window of src (window index = workgroup index modulo src_bytes / 96 KiB) into LDS,
 *   16 KiB per step, `iters` steps, round and round: larger than a CU's vector L1, so after
 *   the first pass the loads are served by the XCD's L2 as long as the windows of the
 *   workgroups sharing an XCD fit it (src_bytes = 24 MiB: 32 windows of 96 KiB per XCD).
 *   through_registers == 0: 16-byte loads that write straight into LDS (the staging pattern of
 *   the forward kernel); != 0: 16-byte loads into registers followed by LDS writes.
 *   Bytes moved = blocks * iters * 16 KiB.  src: device, 16-byte aligned,
 *   96 KiB <= src_bytes < 4 GiB; sink as above.
 * conv_ceiling_lds_read: `blocks` workgroups of 8 waves, each wave keeping eight 16-byte LDS
 *   reads per lane in flight, `iters` times.  row_len == 0: lane i reads chunk i (no two
 *   lanes of a 16-lane pass on the same banks); row_len > 0: lane i reads the chunk of pixel
 *   i of a tile whose rows of row_len pixels lie row_pitch chunks apart (the operand read
 *   over a staged tile with a halo: pitch = row_len + S - 1), at most 2 KiB per wave.
 *   Bytes read = blocks * 512 * iters * 8 * 16.  sink: device, blocks * 512 floats.
 * conv_ceiling_shader_clock: `blocks` (1..256) workgroups of one wave each wait for
 *   duration_us (1..1000000) microseconds of the constant 100 MHz clock, asleep most of the
 *   time, and report the shader-clock cycles that went by: ticks[2*b] = cycles, ticks[2*b+1] =
 *   100 MHz ticks, for workgroup b (consecutive workgroups go to consecutive XCDs).  Launched
 *   on a second stream next to other work, it says at which clock the compute units ran under
 *   that load (the published peaks assume 2.4 GHz).  ticks: device, 2 * blocks int64, written
 *   once; the wave holds no LDS and a handful of registers, and ends after a bounded number of
 *   iterations whatever the clocks do.
 * Errors: CONV_EINVAL for a NULL or misaligned pointer or a count < 1, CONV_EUNSUPPORTED
 * beyond the stated sizes, CONV_ELAUNCH if the runtime refuses the launch. */
conv_status_t conv_ceiling_mfma(int32_t dtype, int32_t blocks, int32_t iters, float *sink,
                                void *stream);
conv_status_t conv_ceiling_copy(void *dst, const void *src, size_t bytes, void *stream);
conv_status_t conv_ceiling_read(const void *src, size_t bytes, float *sink, void *stream);
conv_status_t conv_ceiling_write(void *dst, size_t bytes, void *stream);
conv_status_t conv_ceiling_l2_to_lds(const void *src, size_t src_bytes, int32_t blocks,
                                     int32_t iters, int32_t through_registers, float *sink,
                                     void *stream);
conv_status_t conv_ceiling_lds_read(int32_t blocks, int32_t iters, int32_t row_len,
                                    int32_t row_pitch, float *sink, void *stream);
conv_status_t conv_ceiling_shader_clock(int32_t blocks, int32_t duration_us, int64_t *ticks,
                                        void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CONV_MI355X_H */
