// Measured ceilings of the machine, for the benchmark's roofline columns: what the matrix
// cores, the HBM and the L2 -> LDS path of THIS device sustain on loops that do nothing else.
// The convolution kernels are priced against the published peaks; these loops say how much
// of a published peak a kernel can reach at all (Section III of the paper likewise quotes
// its kernels against what the machine sustains on a plain compute loop).
//
// None of this is on the convolution path: the entry points only launch, take every buffer
// from the caller and are timed by the caller with events on the same stream.
#include <algorithm>

#include "conv_internal.h"

namespace convmi {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// `iters` rounds of eight independent 32x32 MFMAs per wave (eight accumulator tiles, 128
// registers: the register blocking of the convolution kernels), operands held in registers.
template <bool BF16>
__global__ __launch_bounds__(256) void mfma_issue_kernel(float *sink, int iters)
{
    f32x16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int t = 0; t < 16; ++t) acc[i][t] = (float)i;  // (distinct chains: nothing to merge)
    const float seed = (float)(threadIdx.x & 7) * 0.125f;
    for (int it = 0; it < iters; ++it) {
        if constexpr (BF16) {
            bf16x8 a, b;
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                a[t] = (__bf16)(seed + (float)t);
                b[t] = (__bf16)(seed - (float)t);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i)
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(seed, seed + 1.0f, acc[i], 0, 0, 0);
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int t = 0; t < 16; ++t) s += acc[i][t];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// dst[i] = src[i], 16 bytes per lane and step, grid-stride; loads and stores non-temporal, as
// the convolution kernels issue them for tensors that stream past once.
typedef unsigned int copy_u32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void copy_kernel(copy_u32x4 *__restrict__ dst,
                                                   const copy_u32x4 *__restrict__ src, size_t n16)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256)
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// Read-only and write-only streams of the same form (what a pass that mostly reads, or mostly
// writes, can reach; a copy pays for the turn-arounds between the two).
__global__ __launch_bounds__(256) void read_kernel(const copy_u32x4 *__restrict__ src, size_t n16,
                                                   unsigned *sink)
{
    copy_u32x4 x = {0u, 0u, 0u, 0u};
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) {
        const copy_u32x4 v = __builtin_nontemporal_load(src + i);
        x[0] ^= v[0]; x[1] ^= v[1]; x[2] ^= v[2]; x[3] ^= v[3];
    }
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = x[0] ^ x[1] ^ x[2] ^ x[3];
}
__global__ __launch_bounds__(256) void write_kernel(copy_u32x4 *__restrict__ dst, size_t n16)
{
    const copy_u32x4 v = {1u, 2u, 3u, (unsigned)threadIdx.x};
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256)
        __builtin_nontemporal_store(v, dst + i);
}

// The staging pattern of the implicit-GEMM kernel with nothing behind it: every workgroup
// streams its own 96 KiB window of `src` into a ring of two 16 KiB LDS buffers, 16 KiB per
// step, `iters` steps, going round the window.  A window is larger than a CU's 32 KiB vector
// L1, and the windows that the workgroups of one XCD touch (at most 32 distinct ones) fit its
// 4 MiB L2: after the first pass every load is an L2 hit that misses the L1.
//   DIRECT: 16-byte loads that write straight into LDS (what the convolution kernels use);
//   else: 16-byte loads into registers, then 16-byte LDS writes.
constexpr int kStep = 16 * 1024;
constexpr int kWindow = 6 * kStep;
template <bool DIRECT>
__global__ __launch_bounds__(256) void l2_to_lds_kernel(const void *src, size_t src_bytes, float *sink,
                                                        int iters)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const size_t windows = src_bytes / kWindow;
    const size_t base = ((size_t)blockIdx.x % windows) * kWindow;
    const rsrc_t r = make_rsrc(src, base, base + kWindow);
    // 1024 chunks of 16 bytes per step: 4 wave-level loads per wave
    int sub = 0;
    for (int it = 0; it < iters; ++it) {
        unsigned char *buf = lds + (it & 1) * kStep;
        const unsigned soff = (unsigned)sub * (unsigned)kStep;
        if constexpr (DIRECT) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int chunk = (i * 4 + wave) * 64;
                load_to_lds_16(r, (unsigned)(chunk + lane) * 16u, soff, buf + chunk * 16);
            }
            // (the previous step's loads have landed; this step's four stay in flight)
            __builtin_amdgcn_s_waitcnt(0x0F70 | 4);
        } else {
            typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
            // (the window does not change, but every step must fetch it again: nothing moves
            // across this point)
            asm volatile("" ::: "memory");
            u32x4 v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int chunk = (i * 4 + wave) * 64;
                v[i] = __builtin_amdgcn_raw_buffer_load_b128(r, (unsigned)(chunk + lane) * 16u, soff, 0);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int chunk = (i * 4 + wave) * 64;
                *reinterpret_cast<u32x4 *>(buf + (chunk + lane) * 16) = v[i];
            }
        }
        sub = sub == 5 ? 0 : sub + 1;
    }
    wait_all_memory();
    __syncthreads();
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] =
        reinterpret_cast<const float *>(lds)[(threadIdx.x * 4 + blockIdx.x) % (2 * kStep / 4)];
}

// 16-byte LDS reads, eight independent ones in flight per wave, `iters` times.  Lane i reads
// chunk i of its wave's 4 KiB (row_len = 0), or the chunk of pixel i of a tile of rows of
// `row_len` pixels that lie `row_pitch` chunks apart: the operand read of the implicit-GEMM
// kernel over a staged tile whose rows are wider than the result's (a 3x3 filter: pitch =
// row_len + 2).  The LDS serves 16 lanes per pass from 64 banks of 4 bytes: lanes of one pass
// whose chunks are equal modulo 16 take turns.
__global__ __launch_bounds__(512) void lds_read_kernel(float *sink, int iters, int row_len, int row_pitch)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    for (int i = threadIdx.x; i < 16384; i += blockDim.x) reinterpret_cast<unsigned *>(lds)[i] = (unsigned)i;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int chunk = row_len > 0 ? (lane / row_len) * row_pitch + lane % row_len : lane;
    const unsigned base = (unsigned)((wave & 7) * 4096 + chunk * 16);
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    unsigned acc = 0;
    for (int it = 0; it < iters; ++it) {
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v[u]) : "v"(base), "n"((u & 1) * 2048));
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u][0] ^ v[u][3];
    }
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = (float)(acc & 0xFFFF);
}

// One wave per workgroup sits out `ticks_100mhz` ticks of the constant 100 MHz clock, asleep
// most of the time, and reports how many shader-clock cycles went by meanwhile: the clock the
// compute units really ran at while other work (on another stream) kept the device busy.  The
// published peaks assume 2.4 GHz; power management lowers the clock under load.  The loop is
// bounded by an iteration count as well, so the wave ends whatever the clocks do.
__global__ __launch_bounds__(64) void shader_clock_kernel(long long *out, long long ticks_100mhz, int max_iters)
{
    const long long w0 = wall_clock64();
    const long long c0 = clock64();
    long long w = w0;
    for (int it = 0; it < max_iters && w - w0 < ticks_100mhz; ++it) {
        __builtin_amdgcn_s_sleep(32);
        w = wall_clock64();
    }
    const long long c1 = clock64();
    if (threadIdx.x == 0) {
        out[2 * blockIdx.x] = c1 - c0;
        out[2 * blockIdx.x + 1] = w - w0;
    }
}

}  // namespace
}  // namespace convmi

using namespace convmi;

extern "C" {

conv_status_t conv_ceiling_mfma(int32_t dtype, int32_t blocks, int32_t iters, float *sink, void *stream)
{
    if ((dtype != CONV_F32 && dtype != CONV_BF16) || blocks < 1 || iters < 1 || !sink) return CONV_EINVAL;
    if (dtype == CONV_BF16)
        hipLaunchKernelGGL(mfma_issue_kernel<true>, dim3(blocks), dim3(256), 0, (hipStream_t)stream, sink,
                           iters);
    else
        hipLaunchKernelGGL(mfma_issue_kernel<false>, dim3(blocks), dim3(256), 0, (hipStream_t)stream, sink,
                           iters);
    return hipGetLastError() == hipSuccess ? CONV_OK : CONV_ELAUNCH;
}

conv_status_t conv_ceiling_copy(void *dst, const void *src, size_t bytes, void *stream)
{
    if (!dst || !src || bytes < 16 || (bytes & 15) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15))
        return CONV_EINVAL;
    const size_t n16 = bytes / 16;
    const unsigned grid = (unsigned)std::min<size_t>((n16 + 255) / 256, 256 * 32);
    hipLaunchKernelGGL(copy_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream,
                       static_cast<copy_u32x4 *>(dst), static_cast<const copy_u32x4 *>(src), n16);
    return hipGetLastError() == hipSuccess ? CONV_OK : CONV_ELAUNCH;
}

conv_status_t conv_ceiling_read(const void *src, size_t bytes, float *sink, void *stream)
{
    if (!src || !sink || bytes < 16 || (bytes & 15) || ((uintptr_t)src & 15)) return CONV_EINVAL;
    const size_t n16 = bytes / 16;
    const unsigned grid = (unsigned)std::min<size_t>((n16 + 255) / 256, 256 * 32);
    hipLaunchKernelGGL(read_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream,
                       static_cast<const copy_u32x4 *>(src), n16, reinterpret_cast<unsigned *>(sink));
    return hipGetLastError() == hipSuccess ? CONV_OK : CONV_ELAUNCH;
}

conv_status_t conv_ceiling_write(void *dst, size_t bytes, void *stream)
{
    if (!dst || bytes < 16 || (bytes & 15) || ((uintptr_t)dst & 15)) return CONV_EINVAL;
    const size_t n16 = bytes / 16;
    const unsigned grid = (unsigned)std::min<size_t>((n16 + 255) / 256, 256 * 32);
    hipLaunchKernelGGL(write_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream,
                       static_cast<copy_u32x4 *>(dst), n16);
    return hipGetLastError() == hipSuccess ? CONV_OK : CONV_ELAUNCH;
}

conv_status_t conv_ceiling_l2_to_lds(const void *src, size_t src_bytes, int32_t blocks, int32_t iters,
                                     int32_t through_registers, float *sink, void *stream)
{
    if (!src || !sink || src_bytes < (size_t)kWindow || blocks < 1 || iters < 1 || ((uintptr_t)src & 15))
        return CONV_EINVAL;
    if (src_bytes >= ((size_t)1 << 32)) return CONV_EUNSUPPORTED;
    const size_t lds_bytes = 2 * kStep;
    if (through_registers)
        hipLaunchKernelGGL(l2_to_lds_kernel<false>, dim3(blocks), dim3(256), lds_bytes, (hipStream_t)stream,
                           src, src_bytes, sink, iters);
    else
        hipLaunchKernelGGL(l2_to_lds_kernel<true>, dim3(blocks), dim3(256), lds_bytes, (hipStream_t)stream,
                           src, src_bytes, sink, iters);
    return hipGetLastError() == hipSuccess ? CONV_OK : CONV_ELAUNCH;
}

conv_status_t conv_ceiling_lds_read(int32_t blocks, int32_t iters, int32_t row_len, int32_t row_pitch,
                                    float *sink, void *stream)
{
    if (!sink || blocks < 1 || iters < 1 || row_len < 0) return CONV_EINVAL;
    // (a wave's 64 lanes stay inside its 4 KiB, the second read of a pair 2 KiB further on)
    if (row_len > 0 && (row_pitch < row_len || ((63 / row_len) * row_pitch + row_len) * 16 > 2048))
        return CONV_EINVAL;
    hipLaunchKernelGGL(lds_read_kernel, dim3(blocks), dim3(512), 65536, (hipStream_t)stream, sink, iters,
                       row_len, row_pitch);
    return hipGetLastError() == hipSuccess ? CONV_OK : CONV_ELAUNCH;
}

conv_status_t conv_ceiling_shader_clock(int32_t blocks, int32_t duration_us, int64_t *ticks, void *stream)
{
    if (!ticks || blocks < 1 || blocks > 256 || duration_us < 1 || duration_us > 1000000) return CONV_EINVAL;
    // (a sleep of 32 x 64 cycles is about 1 us at any clock the device runs at: four times the
    // duration in iterations is never the binding limit, and ends the loop if the clock stood still)
    const int max_iters = 4 * duration_us + 1024;
    hipLaunchKernelGGL(shader_clock_kernel, dim3(blocks), dim3(64), 0, (hipStream_t)stream,
                       reinterpret_cast<long long *>(ticks), (long long)duration_us * 100, max_iters);
    return hipGetLastError() == hipSuccess ? CONV_OK : CONV_ELAUNCH;
}

}  // extern "C"
