// Direct convolution without tiling: the three passes written as the loop nests
// of Algorithms 1, 6 (its gather form) and 8 over the blocked layouts of Section II-B,
// one thread per result element (forward, backward) or one workgroup per
// vlen x vlen block of dW (update).  These kernels serve the descriptors that no
// tiled MFMA kernel is instantiated for (a filter shape outside the tables, a row
// too wide for the staged tile); they are correct for every descriptor conv_create
// accepts, and run at a small fraction of the tiled kernels' rate.
//
// Arithmetic: products and sums in fp32, bf16 operands widened exactly, each
// result summed in one fixed order (channel block, filter row, filter column,
// channel for the first two; pixel order, then a fixed tree, for the update), so
// every call returns the same bits.
#include <algorithm>

#include "conv_internal.h"

namespace convmi {
namespace {

template <int DT> struct Vec;
template <> struct Vec<CONV_F32> {
    static constexpr int V = 4;
    typedef float elem_t;
    static __device__ __forceinline__ void load(const void *base, size_t vec_index, float (&x)[4])
    {
        const float4 v = static_cast<const float4 *>(base)[vec_index];
        x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
    }
    static __device__ __forceinline__ float load1(const void *base, size_t i)
    {
        return static_cast<const float *>(base)[i];
    }
    static __device__ __forceinline__ void store1(void *base, size_t i, float y)
    {
        static_cast<float *>(base)[i] = y;
    }
};
template <> struct Vec<CONV_BF16> {
    static constexpr int V = 8;
    typedef unsigned short elem_t;
    static __device__ __forceinline__ float widen(unsigned short b)
    {
        return __builtin_bit_cast(float, (unsigned)b << 16);
    }
    static __device__ __forceinline__ void load(const void *base, size_t vec_index, float (&x)[8])
    {
        const uint4 v = static_cast<const uint4 *>(base)[vec_index];
        const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[2 * i] = __builtin_bit_cast(float, w[i] << 16);
            x[2 * i + 1] = __builtin_bit_cast(float, w[i] & 0xFFFF0000u);
        }
    }
    static __device__ __forceinline__ float load1(const void *base, size_t i)
    {
        return widen(static_cast<const unsigned short *>(base)[i]);
    }
    static __device__ __forceinline__ void store1(void *base, size_t i, float y)
    {
        const __bf16 b = (__bf16)y;  // round to nearest even
        static_cast<unsigned short *>(base)[i] = __builtin_bit_cast(unsigned short, b);
    }
};

// Forward, Algorithm 1 with padding: thread e owns out[n][kb][oj][oi][kv].
template <int DT>
__global__ __launch_bounds__(256) void direct_fwd_kernel(const DirectArgs a)
{
    constexpr int V = Vec<DT>::V;
    const size_t total = (size_t)a.N * a.Kb * a.P * a.Q * V;
    // (a grid has at most 2^32 work-items: larger tensors take several elements per thread)
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
    const int kv = (int)(e % V);
    size_t t = e / V;
    const int oi = (int)(t % a.Q); t /= a.Q;
    const int oj = (int)(t % a.P); t /= a.P;
    const int kb = (int)(t % a.Kb);
    const int n = (int)(t / a.Kb);
    const int Kp = a.Kb * V;
    const int k = kb * V + kv;
    float acc = 0.f;
    for (int cb = 0; cb < a.Cb; ++cb)
        for (int r = 0; r < a.R; ++r) {
            const int ij = oj * a.stride - a.pad_h + r;
            if (ij < 0 || ij >= a.H) continue;
            for (int s = 0; s < a.S; ++s) {
                const int ii = oi * a.stride - a.pad_w + s;
                if (ii < 0 || ii >= a.W) continue;
                float x[V], w[V];
                Vec<DT>::load(a.x, (((size_t)n * a.Cb + cb) * a.H + ij) * a.W + ii, x);
                Vec<DT>::load(a.wt, (((size_t)cb * a.R + r) * a.S + s) * Kp + k, w);
#pragma unroll
                for (int c = 0; c < V; ++c) acc = fmaf(x[c], w[c], acc);
            }
        }
    float y = acc;
    if (a.scale) y *= a.scale[k];
    if (a.bias) y += a.bias[k];
    if (a.resid) y += Vec<DT>::load1(a.resid, e);
    if (a.relu) y = fmaxf(y, 0.f);
    Vec<DT>::store1(a.y, e, y);
    }
}

// Backward by data, the gather form of Algorithm 6: thread e owns
// din[n][cb][ij][ii][cv] and visits the output pixels whose window holds (ij, ii).
template <int DT>
__global__ __launch_bounds__(256) void direct_bwd_kernel(const DirectArgs a)
{
    constexpr int V = Vec<DT>::V;
    const size_t total = (size_t)a.N * a.Cb * a.H * a.W * V;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
    const int cv = (int)(e % V);
    size_t t = e / V;
    const int ii = (int)(t % a.W); t /= a.W;
    const int ij = (int)(t % a.H); t /= a.H;
    const int cb = (int)(t % a.Cb);
    const int n = (int)(t / a.Cb);
    const int Kp = a.Kb * V;
    float acc = 0.f;
    for (int kb = 0; kb < a.Kb; ++kb)
        for (int r = 0; r < a.R; ++r) {
            const int tj = ij + a.pad_h - r;
            if (tj < 0 || tj % a.stride != 0) continue;
            const int oj = tj / a.stride;
            if (oj >= a.P) continue;
            for (int s = 0; s < a.S; ++s) {
                const int ti = ii + a.pad_w - s;
                if (ti < 0 || ti % a.stride != 0) continue;
                const int oi = ti / a.stride;
                if (oi >= a.Q) continue;
                float g[V];
                Vec<DT>::load(a.x, (((size_t)n * a.Kb + kb) * a.P + oj) * a.Q + oi, g);
                const size_t w0 = ((((size_t)cb * a.R + r) * a.S + s) * Kp + (size_t)kb * V) * V + cv;
#pragma unroll
                for (int k = 0; k < V; ++k) acc = fmaf(g[k], Vec<DT>::load1(a.wt, w0 + (size_t)k * V), acc);
            }
        }
    Vec<DT>::store1(a.y, e, acc);
    }
}

// Weight update, Algorithm 8 without the minibatch split: workgroup b owns the
// V x V block dW[cb][r][s][kb*V .. +V][0 .. V) (fp32).  Thread t sums the pixels
// t, t + 256, ... of the (n, oj, oi) list; the 256 partial blocks are then added
// lane over lane within each wave and wave after wave, a fixed order.
template <int DT>
__global__ __launch_bounds__(256) void direct_upd_kernel(const DirectArgs a)
{
    constexpr int V = Vec<DT>::V;
    __shared__ float red[4][V * V];
    const size_t nblk = (size_t)a.Cb * a.R * a.S * a.Kb;
    for (size_t blk = blockIdx.x; blk < nblk; blk += gridDim.x) {
    size_t b = blk;
    const int kb = (int)(b % a.Kb); b /= a.Kb;
    const int s = (int)(b % a.S); b /= a.S;
    const int r = (int)(b % a.R);
    const int cb = (int)(b / a.R);
    float acc[V][V];
#pragma unroll
    for (int k = 0; k < V; ++k)
#pragma unroll
        for (int c = 0; c < V; ++c) acc[k][c] = 0.f;
    const size_t npix = (size_t)a.N * a.P * a.Q;
    for (size_t px = threadIdx.x; px < npix; px += 256) {
        const int oi = (int)(px % a.Q);
        const size_t u = px / a.Q;
        const int oj = (int)(u % a.P);
        const int n = (int)(u / a.P);
        const int ij = oj * a.stride - a.pad_h + r;
        const int ii = oi * a.stride - a.pad_w + s;
        if (ij < 0 || ij >= a.H || ii < 0 || ii >= a.W) continue;
        float x[V], g[V];
        Vec<DT>::load(a.x, (((size_t)n * a.Cb + cb) * a.H + ij) * a.W + ii, x);
        Vec<DT>::load(a.wt, (((size_t)n * a.Kb + kb) * a.P + oj) * a.Q + oi, g);
#pragma unroll
        for (int k = 0; k < V; ++k)
#pragma unroll
            for (int c = 0; c < V; ++c) acc[k][c] = fmaf(g[k], x[c], acc[k][c]);
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int k = 0; k < V; ++k)
#pragma unroll
        for (int c = 0; c < V; ++c) {
            float v = acc[k][c];
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) v += __shfl_down(v, d, 64);
            if (lane == 0) red[wave][k * V + c] = v;
        }
    __syncthreads();
    if (threadIdx.x < V * V) {
        const int i = threadIdx.x;
        const float v = ((red[0][i] + red[1][i]) + red[2][i]) + red[3][i];
        const int Kp = a.Kb * V;
        static_cast<float *>(a.y)[((((size_t)cb * a.R + r) * a.S + s) * Kp + (size_t)kb * V) * V + i] = v;
    }
    __syncthreads();  // red[] is reused by the next block of dW
    }
}

template <typename K> hipError_t launch(K kernel, const DirectArgs &a, size_t blocks, hipStream_t stream)
{
    if (blocks == 0) return hipErrorInvalidValue;
    // grid x block stays below the 2^32 work-items of a dispatch; the kernels stride over the rest
    const size_t kMaxBlocks = 1u << 22;
    hipLaunchKernelGGL(kernel, dim3((unsigned)std::min(blocks, kMaxBlocks)), dim3(256), 0, stream, a);
    return hipGetLastError();
}

}  // namespace

bool direct_fits(int dtype, int N, int Cb, int Kb, int H, int W, int P, int Q, int R, int S)
{
    // element indices are 64-bit and the grids are capped: what bounds these kernels is the
    // tensor size conv_create accepts (2^39 elements per activation tensor)
    const double V = (double)vlen_of(dtype), lim = 549755813888.0 * 2;
    return (double)N * Kb * P * Q * V <= lim && (double)N * Cb * H * W * V <= lim &&
           (double)Cb * R * S * Kb <= 2147483647.0;
}

hipError_t launch_direct_fwd(int dtype, const DirectArgs &a, hipStream_t stream)
{
    const size_t total = (size_t)a.N * a.Kb * a.P * a.Q * vlen_of(dtype);
    return dtype == CONV_BF16 ? launch(direct_fwd_kernel<CONV_BF16>, a, (total + 255) / 256, stream)
                              : launch(direct_fwd_kernel<CONV_F32>, a, (total + 255) / 256, stream);
}

hipError_t launch_direct_bwd(int dtype, const DirectArgs &a, hipStream_t stream)
{
    const size_t total = (size_t)a.N * a.Cb * a.H * a.W * vlen_of(dtype);
    return dtype == CONV_BF16 ? launch(direct_bwd_kernel<CONV_BF16>, a, (total + 255) / 256, stream)
                              : launch(direct_bwd_kernel<CONV_F32>, a, (total + 255) / 256, stream);
}

hipError_t launch_direct_upd(int dtype, const DirectArgs &a, hipStream_t stream)
{
    const size_t blocks = (size_t)a.Cb * a.R * a.S * a.Kb;
    return dtype == CONV_BF16 ? launch(direct_upd_kernel<CONV_BF16>, a, blocks, stream)
                              : launch(direct_upd_kernel<CONV_F32>, a, blocks, stream);
}

}  // namespace convmi
