// Harness-side kernels for bench.py (libdmi_bench.so); not part of the library.
#include "dmi_bench.h"

#include <hip/hip_runtime.h>

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ void sleep_kernel(uint64_t ticks)
{
    // wall_clock64 runs at a constant 100 MHz; the loop ends after `ticks` or 2^22 naps
    const uint64_t t0 = wall_clock64();
    for (uint32_t i = 0; i < (1u << 22); i++) {
        if (wall_clock64() - t0 >= ticks) break;
        __builtin_amdgcn_s_sleep(64);
    }
}

__device__ __forceinline__ float bf16lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// Each lane streams 16-byte vectors of W with 4 loads in flight; x (8 KB) stays in L1/L2.
__global__ void __launch_bounds__(256) stream_gemv_kernel(const u32x4 *__restrict__ w, uint64_t n_vec,
                                                          const u32x4 *__restrict__ x, float *__restrict__ out)
{
    const uint64_t stride = (uint64_t)gridDim.x * 256u;
    uint64_t i = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    float acc = 0.f;
    for (; i + 3 * stride < n_vec; i += 4 * stride) {
        u32x4 a[4];
#pragma unroll
        for (int k = 0; k < 4; k++) a[k] = __builtin_nontemporal_load(&w[i + k * stride]);
#pragma unroll
        for (int k = 0; k < 4; k++) {
            const u32x4 b = x[(i + k * stride) & 511u];
            acc += bf16lo(a[k].x) * bf16lo(b.x) + bf16hi(a[k].x) * bf16hi(b.x);
            acc += bf16lo(a[k].y) * bf16lo(b.y) + bf16hi(a[k].y) * bf16hi(b.y);
            acc += bf16lo(a[k].z) * bf16lo(b.z) + bf16hi(a[k].z) * bf16hi(b.z);
            acc += bf16lo(a[k].w) * bf16lo(b.w) + bf16hi(a[k].w) * bf16hi(b.w);
        }
    }
    for (; i < n_vec; i += stride) {
        const u32x4 a = __builtin_nontemporal_load(&w[i]);
        const u32x4 b = x[i & 511u];
        acc += bf16lo(a.x) * bf16lo(b.x) + bf16hi(a.x) * bf16hi(b.x);
        acc += bf16lo(a.y) * bf16lo(b.y) + bf16hi(a.y) * bf16hi(b.y);
        acc += bf16lo(a.z) * bf16lo(b.z) + bf16hi(a.z) * bf16hi(b.z);
        acc += bf16lo(a.w) * bf16lo(b.w) + bf16hi(a.w) * bf16hi(b.w);
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) acc += __shfl_xor(acc, d, 64);
    if ((threadIdx.x & 63u) == 0) atomicAdd(&out[(blockIdx.x * 4u + (threadIdx.x >> 6)) & 4095u], acc);
}

__global__ void __launch_bounds__(256) plain_copy_kernel(u32x4 *__restrict__ dst, const u32x4 *__restrict__ src,
                                                         uint64_t n_vec)
{
    const uint64_t stride = (uint64_t)gridDim.x * 256u;
    for (uint64_t i = (uint64_t)blockIdx.x * 256u + threadIdx.x; i < n_vec; i += stride) dst[i] = src[i];
}

extern "C" int dmi_bench_copy(void *dst, const void *src, uint64_t n_bytes, void *hip_stream)
{
    if (!dst || !src || n_bytes % 16u || (uintptr_t)dst % 16u || (uintptr_t)src % 16u) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(plain_copy_kernel, dim3(2048), dim3(256), 0, (hipStream_t)hip_stream, (u32x4 *)dst,
                       (const u32x4 *)src, n_bytes / 16u);
    return (int)hipGetLastError();
}

extern "C" int dmi_bench_sleep(void *hip_stream, uint32_t microseconds)
{
    hipLaunchKernelGGL(sleep_kernel, dim3(1), dim3(64), 0, (hipStream_t)hip_stream, (uint64_t)microseconds * 100u);
    return (int)hipGetLastError();
}

extern "C" int dmi_bench_stream_gemv(const void *w, uint64_t n_elems, const void *x, float *out, void *hip_stream)
{
    if (!w || !x || !out || n_elems % 8u || (uintptr_t)w % 16u) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(stream_gemv_kernel, dim3(4096), dim3(256), 0, (hipStream_t)hip_stream,
                       (const u32x4 *)w, n_elems / 8u, (const u32x4 *)x, out);
    return (int)hipGetLastError();
}
