// Measurement kernels (lrd_measure.h): a register-only loop of matrix instructions and a plain
// streaming kernel.  They compute nothing of the layers; a benchmark times them in the same run as
// the layer passes to see what the machine delivers with no memory, and with nothing but memory.
#include "lrd_measure.h"
#include "lrd_internal.hpp"

namespace lrd {
namespace {

__global__ __launch_bounds__(256) void mfma_loop_kernel(float* __restrict__ sink, int iters)
{
    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    bf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = (bf16_t)(float)(threadIdx.x % 3);
        b[e] = (bf16_t)(float)(threadIdx.x % 5);
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) s += acc[i][0];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// Every lane reads 16 bytes of LDS per access in the pattern of a k-contiguous operand fragment of the
// matrix instruction (32 rows at the product kernel's row pitch of 144 bytes, two k halves), eight
// ds_read_b128 in flight before one wait; nothing else runs, so the launch time is the LDS read time.
// (Written with the instruction itself: a read through a generic pointer is a flat load, which takes
// the vector-memory path and measures that instead.)
__global__ __launch_bounds__(256) void lds_read_kernel(unsigned* __restrict__ sink, int iters)
{
    typedef __attribute__((address_space(3))) unsigned char lds_byte;
    __shared__ __align__(16) unsigned char lds_bytes[32768];
    const int tid = threadIdx.x, lane = tid & 63;
    for (int i = tid; i < 8192; i += 256) reinterpret_cast<unsigned*>(lds_bytes)[i] = (unsigned)i;
    __syncthreads();
    // largest byte touched: 16384 + 31 * 144 + 16 + 4704 + 15 < 32768
    const unsigned base = (unsigned)(uintptr_t)(lds_byte*)lds_bytes + (unsigned)((lane & 31) * 144 + (lane >> 5) * 16);
    unsigned acc = 0;
    for (int it = 0; it < iters; ++it) {
        const unsigned a = base + ((unsigned)(it & 1) << 14);
        u32x4 v0, v1, v2, v3, v4, v5, v6, v7;
        asm volatile("ds_read_b128 %0, %8\n ds_read_b128 %1, %8 offset:32\n ds_read_b128 %2, %8 offset:64\n ds_read_b128 %3, %8 offset:96\n"
                     "ds_read_b128 %4, %8 offset:4608\n ds_read_b128 %5, %8 offset:4640\n ds_read_b128 %6, %8 offset:4672\n"
                     "ds_read_b128 %7, %8 offset:4704\n s_waitcnt lgkmcnt(0)"
                     : "=v"(v0), "=v"(v1), "=v"(v2), "=v"(v3), "=v"(v4), "=v"(v5), "=v"(v6), "=v"(v7)
                     : "v"(a));
        acc += v0.x + v1.y + v2.z + v3.w + v4.x + v5.y + v6.z + v7.w;
    }
    sink[(size_t)blockIdx.x * 256 + tid] = acc;
}

constexpr int STREAM_THREADS = 256;
constexpr int STREAM_PER_THREAD = 8;   // 16-byte accesses per thread: 32 KiB per workgroup

template <int MODE>
__global__ __launch_bounds__(STREAM_THREADS) void stream_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n16)
{
    const size_t base = (size_t)blockIdx.x * (STREAM_THREADS * STREAM_PER_THREAD) + threadIdx.x;
    u32x4 v[STREAM_PER_THREAD];
    if (MODE != LRD_STREAM_WRITE) {
#pragma unroll
        for (int i = 0; i < STREAM_PER_THREAD; ++i) {
            const size_t idx = base + (size_t)i * STREAM_THREADS;
            const u32x4 z = {0u, 0u, 0u, 0u};
            v[i] = idx < n16 ? __builtin_nontemporal_load(src + idx) : z;
        }
    } else {
#pragma unroll
        for (int i = 0; i < STREAM_PER_THREAD; ++i) v[i] = u32x4{(uint32_t)base, 1u, 2u, 3u};
    }
    if (MODE == LRD_STREAM_READ) {
        u32x4 s = v[0];
#pragma unroll
        for (int i = 1; i < STREAM_PER_THREAD; ++i) s ^= v[i];
        // a store that (almost) never happens keeps the loads alive without adding traffic
        if ((s.x ^ s.y ^ s.z ^ s.w) == 0x9E3779B9u) dst[threadIdx.x] = s;
    } else {
#pragma unroll
        for (int i = 0; i < STREAM_PER_THREAD; ++i) {
            const size_t idx = base + (size_t)i * STREAM_THREADS;
            if (idx < n16) __builtin_nontemporal_store(v[i], dst + idx);
        }
    }
}

}  // namespace
}  // namespace lrd

using namespace lrd;

extern "C" {

lrd_status lrd_measure_mfma_loop(float* sink, int32_t workgroups, int32_t iters, double* flops_host, void* hip_stream)
{
    if (!sink || workgroups < 1 || workgroups > (1 << 20) || iters < 1) return LRD_ERR_INVALID_ARG;
    hipLaunchKernelGGL(mfma_loop_kernel, dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)hip_stream, sink, (int)iters);
    if (hipGetLastError() != hipSuccess) return LRD_ERR_RUNTIME;
    // 4 waves x iters x 4 instructions x (32 x 32 x 16 multiply-adds)
    if (flops_host) *flops_host = (double)workgroups * 4.0 * (double)iters * 4.0 * 2.0 * 32.0 * 32.0 * 16.0;
    return LRD_OK;
}

lrd_status lrd_measure_lds_read(uint32_t* sink, int32_t workgroups, int32_t iters, double* bytes_host, void* hip_stream)
{
    if (!sink || workgroups < 1 || workgroups > (1 << 20) || iters < 1) return LRD_ERR_INVALID_ARG;
    hipLaunchKernelGGL(lds_read_kernel, dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)hip_stream, sink, (int)iters);
    if (hipGetLastError() != hipSuccess) return LRD_ERR_RUNTIME;
    if (bytes_host) *bytes_host = (double)workgroups * 256.0 * (double)iters * 8.0 * 16.0;
    return LRD_OK;
}

lrd_status lrd_measure_stream(const void* src, void* dst, size_t bytes, int32_t mode, void* hip_stream)
{
    if (!dst || bytes < 16 || bytes % 16 != 0) return LRD_ERR_INVALID_ARG;
    if (mode != LRD_STREAM_READ && mode != LRD_STREAM_WRITE && mode != LRD_STREAM_COPY) return LRD_ERR_INVALID_ARG;
    if (mode != LRD_STREAM_WRITE && !src) return LRD_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u) return LRD_ERR_ALIGNMENT;
    const size_t n16 = bytes / 16;
    const size_t per_wg = (size_t)STREAM_THREADS * STREAM_PER_THREAD;
    const size_t wgs = (n16 + per_wg - 1) / per_wg;
    if (wgs > 0x7FFFFFFFu) return LRD_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)hip_stream;
    const u32x4* s = (const u32x4*)src;
    u32x4* d = (u32x4*)dst;
    if (mode == LRD_STREAM_READ) hipLaunchKernelGGL(stream_kernel<LRD_STREAM_READ>, dim3((unsigned)wgs), dim3(STREAM_THREADS), 0, st, s, d, n16);
    else if (mode == LRD_STREAM_WRITE) hipLaunchKernelGGL(stream_kernel<LRD_STREAM_WRITE>, dim3((unsigned)wgs), dim3(STREAM_THREADS), 0, st, s, d, n16);
    else hipLaunchKernelGGL(stream_kernel<LRD_STREAM_COPY>, dim3((unsigned)wgs), dim3(STREAM_THREADS), 0, st, s, d, n16);
    return hipGetLastError() == hipSuccess ? LRD_OK : LRD_ERR_RUNTIME;
}

}  // extern "C"
