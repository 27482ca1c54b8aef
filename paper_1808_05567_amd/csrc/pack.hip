// Layout conversion between the logical tensors of Section II of the paper
// (I[N][C][H][W], W[K][C][R][S]) and the channel-blocked layouts the kernels
// work on (Section II-B; block = 16 bytes of channels).  Pure permutations:
// no arithmetic, padded channel slots are written as zero.
//
// Also the weight transform of the backward-by-data duality (Section II-I):
// channel roles swapped and taps flipped, optionally decimated by the stride.
#include "conv_internal.h"

namespace convmi {

// X[N][C][H][W] -> Xb[N][Cb][H][W][V]; one thread per 16-byte block.
template <typename T, int V>
__global__ __launch_bounds__(256) void pack_act_kernel(const T *__restrict__ src, T *__restrict__ dst,
                                                       int C, int Cb, size_t HW, size_t total)
{
    // (a grid has at most 2^32 work-items: larger tensors take several blocks per thread)
    for (size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (size_t)gridDim.x * 256) {
    const size_t hw = idx % HW;
    const size_t t = idx / HW;
    const int cb = (int)(t % Cb);
    const size_t n = t / Cb;
    T v[V];
#pragma unroll
    for (int j = 0; j < V; ++j) {
        const int c = cb * V + j;
        v[j] = c < C ? src[(n * C + c) * HW + hw] : T(0);
    }
    T *d = dst + idx * V;
#pragma unroll
    for (int j = 0; j < V; ++j) d[j] = v[j];
    }
}

template <typename T, int V>
__global__ __launch_bounds__(256) void unpack_act_kernel(const T *__restrict__ src, T *__restrict__ dst,
                                                         int C, int Cb, size_t HW, size_t total)
{
    for (size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (size_t)gridDim.x * 256) {
    const size_t hw = idx % HW;
    const size_t t = idx / HW;
    const int cb = (int)(t % Cb);
    const size_t n = t / Cb;
    const T *s = src + idx * V;
#pragma unroll
    for (int j = 0; j < V; ++j) {
        const int c = cb * V + j;
        if (c < C) dst[(n * C + c) * HW + hw] = s[j];
    }
    }
}

// W[K][C][R][S] <-> Wb[Cb][R][S][Kp][V]; one thread per (cb, r, s, k).
template <typename T, int V, bool PACK>
__global__ __launch_bounds__(256) void perm_wt_kernel(const T *__restrict__ src, T *__restrict__ dst,
                                                      int K, int C, int RS, int Kp, int total)
{
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int k = idx % Kp;
    const int t = idx / Kp;
    const int rs = t % RS;
    const int cb = t / RS;
#pragma unroll
    for (int j = 0; j < V; ++j) {
        const int c = cb * V + j;
        const bool in = k < K && c < C;
        const size_t lo = ((size_t)k * C + c) * RS + rs;
        const size_t bo = (size_t)idx * V + j;
        if (PACK)
            dst[bo] = in ? src[lo] : T(0);
        else if (in)
            dst[lo] = src[bo];
    }
}

// dst[kb][r2][s2][c][kk] = Wb[c/V][r][s][kb*V+kk][c%V] with
// r = tap_stride*(Rsub-1-r2) + r_off (zero if r2 >= Rsub), likewise s.
template <typename T, int V>
__global__ __launch_bounds__(256) void wt_xform_kernel(const WtXformArgs a, int total)
{
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const T *src = static_cast<const T *>(a.src);
    T *dst = static_cast<T *>(a.dst);
    const int c = idx % a.Cp;
    int t = idx / a.Cp;
    const int s2 = t % a.S2;
    t /= a.S2;
    const int r2 = t % a.R2;
    const int kb = t / a.R2;
    const bool tap_ok = r2 < a.Rsub && s2 < a.Ssub;
    const int r = a.tap_stride * (a.Rsub - 1 - r2) + a.r_off;
    const int s = a.tap_stride * (a.Ssub - 1 - s2) + a.s_off;
    T v[V];
#pragma unroll
    for (int kk = 0; kk < V; ++kk) {
        const int k = kb * V + kk;
        v[kk] = tap_ok ? src[((((size_t)(c / V) * a.R + r) * a.S + s) * a.Kp + k) * V + (c % V)]
                       : T(0);
    }
#pragma unroll
    for (int kk = 0; kk < V; ++kk) dst[(size_t)idx * V + kk] = v[kk];
}

// One thread per (kb, u, v, row): V consecutive output channels k of channel block kb.
template <typename T, int V>
__global__ __launch_bounds__(256) void wt_merge_kernel(const WtMergeArgs a, int total)
{
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const T *src = static_cast<const T *>(a.src);
    T *dst = static_cast<T *>(a.dst);
    const int rows = a.cells * a.st * a.st * V;
    const int row = idx % rows;
    int t = idx / rows;
    const int v = t % a.S2;
    t /= a.S2;
    const int u = t % a.R2;
    const int kb = t / a.R2;
    // row block (py, e, px): the position (py, e*st + px) of a cell pair's st x (cells*st) pixels
    const int blk = row / V, c = row % V;
    const int py = blk / (a.cells * a.st);
    const int e = (blk / a.st) % a.cells, px = blk % a.st;
    const int r2 = u - a.rsh[py], s2 = v - e - a.ssh[px];
    const bool tap_ok = r2 >= 0 && r2 < a.rsub[py] && s2 >= 0 && s2 < a.ssub[px];
    const int r = a.st * (a.rsub[py] - 1 - r2) + a.roff[py];
    const int s = a.st * (a.ssub[px] - 1 - s2) + a.soff[px];
    T val[V];
#pragma unroll
    for (int kk = 0; kk < V; ++kk) {
        const int k = kb * V + kk;
        val[kk] = tap_ok ? src[(((size_t)r * a.S + s) * a.Kp + k) * V + c] : T(0);
    }
#pragma unroll
    for (int kk = 0; kk < V; ++kk) dst[(size_t)idx * V + kk] = val[kk];
}

// (grid x 256 threads stays below the 2^32 work-items of a dispatch; the activation kernels
// stride over what is left, the weight tensors are bounded at conv_create)
static inline int blocks_for(size_t total)
{
    const size_t b = (total + 255) / 256;
    return (int)(b < (1u << 22) ? b : (1u << 22));
}

hipError_t launch_pack_act(int dtype, const void *nchw, void *blk, int N, int C, int H, int W,
                           hipStream_t stream)
{
    const int V = vlen_of(dtype), Cb = ceil_div(C, V);
    const size_t total = (size_t)N * Cb * H * W;
    if (dtype == CONV_BF16)
        hipLaunchKernelGGL((pack_act_kernel<uint16_t, 8>), dim3(blocks_for(total)), dim3(256), 0, stream,
                           (const uint16_t *)nchw, (uint16_t *)blk, C, Cb, (size_t)H * W, total);
    else
        hipLaunchKernelGGL((pack_act_kernel<uint32_t, 4>), dim3(blocks_for(total)), dim3(256), 0, stream,
                           (const uint32_t *)nchw, (uint32_t *)blk, C, Cb, (size_t)H * W, total);
    return hipGetLastError();
}

hipError_t launch_unpack_act(int dtype, const void *blk, void *nchw, int N, int C, int H, int W,
                             hipStream_t stream)
{
    const int V = vlen_of(dtype), Cb = ceil_div(C, V);
    const size_t total = (size_t)N * Cb * H * W;
    if (dtype == CONV_BF16)
        hipLaunchKernelGGL((unpack_act_kernel<uint16_t, 8>), dim3(blocks_for(total)), dim3(256), 0,
                           stream, (const uint16_t *)blk, (uint16_t *)nchw, C, Cb, (size_t)H * W, total);
    else
        hipLaunchKernelGGL((unpack_act_kernel<uint32_t, 4>), dim3(blocks_for(total)), dim3(256), 0,
                           stream, (const uint32_t *)blk, (uint32_t *)nchw, C, Cb, (size_t)H * W, total);
    return hipGetLastError();
}

hipError_t launch_pack_wt(int dtype, const void *kcrs, void *blk, int K, int C, int R, int S,
                          hipStream_t stream)
{
    const int V = vlen_of(dtype), Cb = ceil_div(C, V), Kp = ceil_div(K, V) * V;
    const int total = Cb * R * S * Kp;
    if (dtype == CONV_BF16)
        hipLaunchKernelGGL((perm_wt_kernel<uint16_t, 8, true>), dim3(blocks_for(total)), dim3(256), 0,
                           stream, (const uint16_t *)kcrs, (uint16_t *)blk, K, C, R * S, Kp, total);
    else
        hipLaunchKernelGGL((perm_wt_kernel<uint32_t, 4, true>), dim3(blocks_for(total)), dim3(256), 0,
                           stream, (const uint32_t *)kcrs, (uint32_t *)blk, K, C, R * S, Kp, total);
    return hipGetLastError();
}

// `dtype` is the element type of the buffers, `vlen` the channel block of the
// layout (a bf16 layer's fp32 weight gradients use vlen 8 with 4-byte elements).
hipError_t launch_unpack_wt(int dtype, const void *blk, void *kcrs, int K, int C, int R, int S,
                            int vlen, hipStream_t stream)
{
    const int Cb = ceil_div(C, vlen), Kp = ceil_div(K, vlen) * vlen;
    const int total = Cb * R * S * Kp;
    if (dtype == CONV_BF16)
        hipLaunchKernelGGL((perm_wt_kernel<uint16_t, 8, false>), dim3(blocks_for(total)), dim3(256), 0,
                           stream, (const uint16_t *)blk, (uint16_t *)kcrs, K, C, R * S, Kp, total);
    else if (vlen == 8)
        hipLaunchKernelGGL((perm_wt_kernel<uint32_t, 8, false>), dim3(blocks_for(total)), dim3(256), 0,
                           stream, (const uint32_t *)blk, (uint32_t *)kcrs, K, C, R * S, Kp, total);
    else
        hipLaunchKernelGGL((perm_wt_kernel<uint32_t, 4, false>), dim3(blocks_for(total)), dim3(256), 0,
                           stream, (const uint32_t *)blk, (uint32_t *)kcrs, K, C, R * S, Kp, total);
    return hipGetLastError();
}

hipError_t launch_wt_xform(int dtype, const WtXformArgs &a, hipStream_t stream)
{
    const int total = a.Kb * a.R2 * a.S2 * a.Cp;
    if (dtype == CONV_BF16)
        hipLaunchKernelGGL((wt_xform_kernel<uint16_t, 8>), dim3(blocks_for(total)), dim3(256), 0, stream,
                           a, total);
    else
        hipLaunchKernelGGL((wt_xform_kernel<uint32_t, 4>), dim3(blocks_for(total)), dim3(256), 0, stream,
                           a, total);
    return hipGetLastError();
}

hipError_t launch_wt_merge(int dtype, const WtMergeArgs &a, hipStream_t stream)
{
    const int V = vlen_of(dtype);
    const int total = a.Kb * a.R2 * a.S2 * a.cells * a.st * a.st * V;
    if (dtype == CONV_BF16)
        hipLaunchKernelGGL((wt_merge_kernel<uint16_t, 8>), dim3(blocks_for(total)), dim3(256), 0, stream,
                           a, total);
    else
        hipLaunchKernelGGL((wt_merge_kernel<uint32_t, 4>), dim3(blocks_for(total)), dim3(256), 0, stream,
                           a, total);
    return hipGetLastError();
}

}  // namespace convmi
