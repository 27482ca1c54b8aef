// Implicit-GEMM direct convolution on MFMA for gfx950: the kernel behind the
// forward pass (Algorithm 1 of the paper, with padding) and, through the two
// duality scenarios of Section II-I, the backward-by-data pass (Algorithm 6).
//
// Mapping of the paper's ingredients:
//   * Section II-B blocked layouts: channels are blocked by v = 16 bytes/element
//     size, the 128-bit vector a lane feeds into one MFMA operand (the role a
//     512-bit register's VLEN plays on AVX-512).
//   * Section II-D microkernel (chain of small GEMMs M^=k, N^=pixels, K^=c into
//     one output tile, stores hoisted out of the r,s loops): a workgroup owns a
//     tile of TK output channels x TM output pixels, each wave keeps FK x FM
//     32x32 accumulator tiles in registers for the whole (c_b, r, s) reduction
//     and writes them once.
//   * Section II-C: the input-channel loop is innermost around a resident
//     output tile for every filter size.
//   * Section II-E prefetching: the next channel step streams from HBM straight
//     into the second LDS buffer while the current one is consumed.
//   * "Direct": the input halo tile is staged once per channel step and reused
//     by all R*S taps out of LDS; no im2col copy exists anywhere.
//   * Section II-F work split (N, then K_b, then P_b/Q_b): the grid enumerates
//     (row tile, column tile, channel tile) with the channel tile fastest and
//     consecutive tiles kept on one XCD so that they share its L2.
#include "igemm_kernel.h"

namespace convmi {

// ---------------------------------------------------------------------------
// Instantiations and dispatch
// ---------------------------------------------------------------------------
static IgemmEntry g_igemm[] = {
    // fp32
    IGEMM_ENTRY(CONV_F32, 4, 1, 1, 7, 2, 3, 3, 2),
    IGEMM_ENTRY(CONV_F32, 2, 2, 1, 7, 2, 3, 3, 3),
    IGEMM_ENTRY(CONV_F32, 4, 1, 1, 7, 4, 1, 1, 1),
    IGEMM_ENTRY(CONV_F32, 2, 2, 1, 7, 4, 1, 1, 2),
    IGEMM_ENTRY(CONV_F32, 2, 2, 1, 7, 1, 1, 1, 2),
    IGEMM_ENTRY(CONV_F32, 2, 2, 1, 7, 1, 3, 3, 3),
    IGEMM_ENTRY(CONV_F32, 2, 2, 1, 7, 1, 7, 7, 12),
    // 4x4: the stride-2 residue classes of a 7x7 backward pass (conv1), one launch each
    // or, where dI has a single channel block, all four as the rows of one filter
    IGEMM_ENTRY(CONV_F32, 2, 2, 1, 7, 2, 4, 4, 4),
    IGEMM_ENTRY(CONV_F32, 1, 4, 1, 7, 2, 4, 4, 6),
    IGEMM_ENTRY(CONV_BF16, 1, 4, 1, 7, 2, 4, 4, 6),
    // (eight pixel waves, 32 x 1792)
    IGEMM_ENTRY(CONV_BF16, 1, 8, 1, 7, 2, 4, 4, 9),
    // (an odd number of channel blocks of dO: one block per step)
    IGEMM_ENTRY(CONV_F32, 1, 4, 1, 7, 1, 4, 4, 6),
    IGEMM_ENTRY(CONV_BF16, 1, 4, 1, 7, 1, 4, 4, 6),
    // (two cells per column: the window is one tap wider)
    IGEMM_ENTRY(CONV_F32, 1, 4, 1, 7, 1, 4, 5, 9),
    IGEMM_ENTRY(CONV_F32, 1, 4, 1, 7, 2, 4, 5, 8),
    // bf16
    IGEMM_ENTRY(CONV_BF16, 4, 1, 1, 7, 2, 3, 3, 2),
    IGEMM_ENTRY(CONV_BF16, 2, 2, 1, 7, 2, 3, 3, 3),
    IGEMM_ENTRY(CONV_BF16, 4, 1, 1, 7, 4, 1, 1, 1),
    IGEMM_ENTRY(CONV_BF16, 2, 2, 1, 7, 4, 1, 1, 2),
    IGEMM_ENTRY(CONV_BF16, 2, 2, 1, 7, 1, 1, 1, 2),
    IGEMM_ENTRY(CONV_BF16, 2, 2, 1, 7, 1, 3, 3, 3),
    IGEMM_ENTRY(CONV_BF16, 2, 2, 1, 7, 1, 7, 7, 12),
    // bf16, two channel fragments per wave: every staged-input fragment read
    // from LDS feeds two MFMAs (LDS bandwidth is what bounds bf16 otherwise)
    IGEMM_ENTRY(CONV_BF16, 2, 2, 2, 7, 2, 3, 3, 3),
    IGEMM_ENTRY(CONV_BF16, 1, 4, 2, 7, 2, 3, 3, 5),
    IGEMM_ENTRY(CONV_BF16, 2, 2, 2, 7, 4, 1, 1, 2),
    IGEMM_ENTRY(CONV_BF16, 1, 4, 2, 7, 4, 1, 1, 4),
    // bf16, 128 accumulator registers per wave: two workgroups share a CU, so one
    // workgroup's prologue and output writes overlap the other's MFMA stream
    IGEMM_ENTRY(CONV_BF16, 1, 4, 2, 4, 2, 3, 3, 3),
    IGEMM_ENTRY(CONV_BF16, 1, 4, 2, 4, 2, 3, 3, 4),
    IGEMM_ENTRY(CONV_BF16, 1, 4, 2, 4, 4, 1, 1, 2),
    // 2x2, 1x2, 2x1: the stride-2 residue classes of a 3x3 backward pass
    IGEMM_ENTRY(CONV_F32, 2, 2, 1, 7, 2, 2, 2, 3),
    IGEMM_ENTRY(CONV_F32, 4, 1, 1, 7, 2, 2, 2, 2),
    IGEMM_ENTRY(CONV_F32, 2, 2, 1, 7, 2, 1, 2, 3),
    IGEMM_ENTRY(CONV_F32, 4, 1, 1, 7, 2, 1, 2, 2),
    IGEMM_ENTRY(CONV_F32, 2, 2, 1, 7, 2, 2, 1, 3),
    IGEMM_ENTRY(CONV_F32, 4, 1, 1, 7, 2, 2, 1, 2),
    IGEMM_ENTRY(CONV_BF16, 1, 4, 2, 4, 2, 2, 2, 3),
    IGEMM_ENTRY(CONV_BF16, 2, 2, 1, 7, 2, 2, 2, 3),
    IGEMM_ENTRY(CONV_BF16, 1, 4, 2, 4, 2, 1, 2, 3),
    IGEMM_ENTRY(CONV_BF16, 2, 2, 1, 7, 2, 1, 2, 3),
    IGEMM_ENTRY(CONV_BF16, 1, 4, 2, 4, 2, 2, 1, 3),
    IGEMM_ENTRY(CONV_BF16, 2, 2, 1, 7, 2, 2, 1, 3),
    // bf16 1x1: a step is only two MFMA rounds, so the loads run two steps ahead
    IGEMM_ENTRY_NB(CONV_BF16, 4, 1, 1, 7, 4, 1, 1, 1, 3),
    IGEMM_ENTRY_NB(CONV_BF16, 2, 2, 1, 7, 4, 1, 1, 2, 3),
    // bf16, eight waves (two per SIMD inside one workgroup, 128 accumulator registers each)
    // 1x1: 256 x 256 tiles, four MFMA rounds per step.  (Measured and dropped: two rounds per
    // step with rings of three to five buffers, 128 x 512 tiles, a 256 x 256 tile on four waves,
    // and eight-wave fp32 tiles: none faster on any Table I layer.)
    IGEMM_ENTRY_NB(CONV_BF16, 4, 2, 2, 4, 8, 1, 1, 1, 2),
    // 1x1, four waves, 128 x 256: two workgroups per CU where the reduction is short
    IGEMM_ENTRY_NB(CONV_BF16, 2, 2, 2, 4, 4, 1, 1, 1, 2),
    // (eight planes per step: for plans of at most one workgroup per CU, see plan_igemm_tile)
    IGEMM_ENTRY_NB(CONV_BF16, 4, 1, 1, 7, 8, 1, 1, 1, 2),
    // 3x3: 128 x 512 tiles
    IGEMM_ENTRY(CONV_BF16, 2, 4, 2, 4, 2, 3, 3, 3),
    IGEMM_ENTRY(CONV_BF16, 2, 4, 2, 4, 2, 3, 3, 4),
    // 1x1 with a single channel tile: the input streams past once, loaded non-temporally
    IGEMM_ENTRY_NB_NT(CONV_F32, 4, 1, 1, 7, 4, 1, 1, 1, 2, 1),
    IGEMM_ENTRY_NB_NT(CONV_F32, 2, 2, 1, 7, 4, 1, 1, 2, 2, 1),
    IGEMM_ENTRY_NB_NT(CONV_BF16, 4, 1, 1, 7, 4, 1, 1, 1, 2, 1),
    IGEMM_ENTRY_NB_NT(CONV_BF16, 4, 1, 1, 7, 4, 1, 1, 1, 3, 1),
    IGEMM_ENTRY_NB_NT(CONV_BF16, 2, 2, 1, 7, 4, 1, 1, 2, 2, 1),
    IGEMM_ENTRY_NB_NT(CONV_BF16, 2, 2, 1, 7, 4, 1, 1, 2, 3, 1),
    IGEMM_ENTRY_NB_NT(CONV_BF16, 4, 2, 2, 4, 8, 1, 1, 1, 2, 1),
};

static IgemmEntry *find_in(IgemmEntry *tab, int n, const IgemmVariant &v)
{
    for (int i = 0; i < n; ++i) {
        const IgemmVariant &w = tab[i].v;
        if (w.dtype == v.dtype && w.wk == v.wk && w.wm == v.wm && w.fk == v.fk && w.fm == v.fm &&
            w.npl == v.npl && w.r == v.r && w.s == v.s && w.ppt == v.ppt && w.nb == v.nb && w.nt == v.nt)
            return &tab[i];
    }
    return nullptr;
}

static IgemmEntry *find_igemm(const IgemmVariant &v)
{
    if (IgemmEntry *e = find_in(g_igemm, (int)(sizeof(g_igemm) / sizeof(g_igemm[0])), v)) return e;
    int n = 0;
    IgemmEntry *rect = igemm_rect_entries(&n);
    return find_in(rect, n, v);
}

bool igemm_variant_exists(const IgemmVariant &v) { return find_igemm(v) != nullptr; }

// Sum of the fp32 partial results of a split reduction, copies ascending (a fixed
// order: reproducible), written in the tensor's type.  One thread per 4 elements.
template <bool BF16>
__global__ __launch_bounds__(256) void split_reduce_kernel(const float *__restrict__ partial,
                                                           void *out, size_t n4, int copies,
                                                           const float *__restrict__ scale,
                                                           const float *__restrict__ bias,
                                                           const void *resid, int relu, int pq, int kb)
{
    constexpr int V = BF16 ? 8 : 4;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n4) return;
    const f32x4 *p = reinterpret_cast<const f32x4 *>(partial);
    f32x4 s = p[idx];
    for (int j = 1; j < copies; ++j) {
        const f32x4 v = p[(size_t)j * n4 + idx];
        s[0] += v[0];
        s[1] += v[1];
        s[2] += v[2];
        s[3] += v[3];
    }
    // element e of [n][kb][pixel][V]: channel = block * V + e % V
    const size_t e0 = idx * 4;
    const int ch0 = (int)((e0 / ((size_t)pq * V)) % (size_t)kb) * V + (int)(e0 % V);
    if (scale) {
        const f32x4 g = *reinterpret_cast<const f32x4 *>(scale + ch0);
        s[0] *= g[0]; s[1] *= g[1]; s[2] *= g[2]; s[3] *= g[3];
    }
    if (resid) {
        if (BF16) {
            const u32x2 r = reinterpret_cast<const u32x2 *>(resid)[idx];
            s[0] += __uint_as_float(r[0] << 16);
            s[1] += __uint_as_float(r[0] & 0xFFFF0000u);
            s[2] += __uint_as_float(r[1] << 16);
            s[3] += __uint_as_float(r[1] & 0xFFFF0000u);
        } else {
            const f32x4 r = reinterpret_cast<const f32x4 *>(resid)[idx];
            s[0] += r[0]; s[1] += r[1]; s[2] += r[2]; s[3] += r[3];
        }
    }
    if (bias) {
        const f32x4 b = *reinterpret_cast<const f32x4 *>(bias + ch0);
        s[0] += b[0]; s[1] += b[1]; s[2] += b[2]; s[3] += b[3];
    }
    if (relu) {
        s[0] = fmaxf(s[0], 0.f); s[1] = fmaxf(s[1], 0.f);
        s[2] = fmaxf(s[2], 0.f); s[3] = fmaxf(s[3], 0.f);
    }
    if (BF16) {
        u32x2 o = {pack_bf16x2(s[0], s[1]), pack_bf16x2(s[2], s[3])};
        reinterpret_cast<u32x2 *>(out)[idx] = o;
    } else {
        reinterpret_cast<f32x4 *>(out)[idx] = s;
    }
}

hipError_t launch_split_reduce(int dtype, const float *partial, void *out, size_t n_elems, int copies,
                               const float *scale, const float *bias, const void *resid, int relu,
                               int pq, int kb, hipStream_t stream)
{
    const size_t n4 = n_elems / 4;
    const unsigned grid = (unsigned)((n4 + 255) / 256);
    if (dtype == CONV_BF16)
        hipLaunchKernelGGL(split_reduce_kernel<true>, dim3(grid), dim3(256), 0, stream, partial, out, n4,
                           copies, scale, bias, resid, relu, pq, kb);
    else
        hipLaunchKernelGGL(split_reduce_kernel<false>, dim3(grid), dim3(256), 0, stream, partial, out, n4,
                           copies, scale, bias, resid, relu, pq, kb);
    return hipGetLastError();
}

hipError_t launch_igemm(const IgemmVariant &v, const IgemmArgs &a, size_t lds_bytes, int grid,
                        hipStream_t stream)
{
    IgemmEntry *e = find_igemm(v);
    if (!e) return hipErrorInvalidDeviceFunction;
    if (hipError_t err = ensure_dynamic_lds(reinterpret_cast<const void *>(e->fn), lds_bytes);
        err != hipSuccess)
        return err;
    hipLaunchKernelGGL(e->fn, dim3(grid), dim3(v.wk * v.wm * 64), lds_bytes, stream, a);
    return hipGetLastError();
}

}  // namespace convmi
