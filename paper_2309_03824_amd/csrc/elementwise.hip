// Elementwise glue and small reductions: GELU (erf form) forward/backward, column sums for the
// bias gradient, and the fixed-order sum of split-K partial products.
#include "lrd_internal.hpp"

namespace lrd {
namespace {

// 8 bf16 (16 bytes) per thread per step; n8 = number of whole groups of 8.
__global__ __launch_bounds__(256) void gelu_fwd_bf16(const bf16_t* __restrict__ Z, bf16_t* __restrict__ A, int64_t n)
{
    int64_t n8 = n / 8;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < n8; g += stride) {
        bf16x8 z = *reinterpret_cast<const bf16x8*>(Z + g * 8);
        bf16x8 a;
#pragma unroll
        for (int e = 0; e < 8; ++e) a[e] = (bf16_t)gelu_bf16_f((float)z[e]);
        *reinterpret_cast<bf16x8*>(A + g * 8) = a;
    }
    if (blockIdx.x == 0 && threadIdx.x < n - n8 * 8) {
        int64_t i = n8 * 8 + threadIdx.x;
        A[i] = (bf16_t)gelu_bf16_f((float)Z[i]);
    }
}

__global__ __launch_bounds__(256) void gelu_bwd_bf16(const bf16_t* dA, const bf16_t* __restrict__ Z,
                                                     bf16_t* dZ, int64_t n)   // dZ may alias dA
{
    int64_t n8 = n / 8;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < n8; g += stride) {
        bf16x8 z = *reinterpret_cast<const bf16x8*>(Z + g * 8);
        bf16x8 d = *reinterpret_cast<const bf16x8*>(dA + g * 8);
        bf16x8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = (bf16_t)((float)d[e] * gelu_grad_bf16_f((float)z[e]));
        *reinterpret_cast<bf16x8*>(dZ + g * 8) = o;
    }
    if (blockIdx.x == 0 && threadIdx.x < n - n8 * 8) {
        int64_t i = n8 * 8 + threadIdx.x;
        dZ[i] = (bf16_t)((float)dA[i] * gelu_grad_bf16_f((float)Z[i]));
    }
}

__global__ __launch_bounds__(256) void gelu_fwd_f32(const float* __restrict__ Z, float* __restrict__ A, int64_t n)
{
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) A[i] = gelu_f(Z[i]);
}

__global__ __launch_bounds__(256) void gelu_bwd_f32(const float* dA, const float* __restrict__ Z,
                                                    float* dZ, int64_t n)   // dZ may alias dA
{
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
        dZ[i] = dA[i] * gelu_grad_f(Z[i]);
}

// out[c] = sum_t dY[t][c]; one block per 64 columns, 4 row-lanes per column, fixed order.
template <class T>
__global__ __launch_bounds__(256) void column_sums_kernel(const T* __restrict__ dY, float* __restrict__ out,
                                                          int64_t Tn, int64_t n)
{
    __shared__ float part[4][64];
    int c = threadIdx.x % 64, lane = threadIdx.x / 64;
    int64_t col = (int64_t)blockIdx.x * 64 + c;
    float s = 0.f;
    if (col < n)
        for (int64_t t = lane; t < Tn; t += 4) s += to_f32(dY[t * n + col]);
    part[lane][c] = s;
    __syncthreads();
    if (lane == 0 && col < n) out[col] = (part[0][c] + part[1][c]) + (part[2][c] + part[3][c]);
}

// The optimizer step of sgd_step_kernel on four consecutive weights whose gradient g has just been
// summed (same arithmetic, so that a step does not depend on where it ran).
struct SgdArgs { float* w; float* m; void* copy; int copy_bf16; float lr, mu, wd; };
__device__ __forceinline__ void sgd_apply4(const SgdArgs& a, int64_t i, f32x4 g)
{
    f32x4 w = *reinterpret_cast<const f32x4*>(a.w + i), m = *reinterpret_cast<const f32x4*>(a.m + i);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        m[e] = fmaf(a.mu, m[e], fmaf(a.wd, w[e], g[e]));
        w[e] = fmaf(-a.lr, m[e], w[e]);
    }
    *reinterpret_cast<f32x4*>(a.m + i) = m;
    *reinterpret_cast<f32x4*>(a.w + i) = w;
    if (a.copy) {
        if (a.copy_bf16) {
            u32x2 pk = {pack_bf16(w[0], w[1]), pack_bf16(w[2], w[3])};
            *reinterpret_cast<u32x2*>(reinterpret_cast<bf16_t*>(a.copy) + i) = pk;
        } else {
            *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(a.copy) + i) = w;
        }
    }
}

// C[m][n] = sum_z partial[z][m][n], slices added in ascending z so the result does not depend on
// scheduling.  VEC consecutive columns per thread (N and ldc are multiples of VEC); OutT is the
// result type (fp32 weight gradients, or bf16 activations rounded once from the fp32 sum).
// With SGD (VEC == 4, fp32, ldc == N) the sum feeds the optimizer step and is not stored.
template <int VEC, class OutT, bool SGD = false>
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float* __restrict__ partial, OutT* __restrict__ C,
                                                              int64_t ldc, int64_t M, int64_t N, int splits, SgdArgs sgd = SgdArgs{})
{
    const int64_t total = M * N;
    const int64_t groups = total / VEC;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < groups; g += stride) {
        const int64_t i = g * VEC;
        float s[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) s[e] = 0.f;
        for (int z = 0; z < splits; ++z) {
            const float* p = partial + (int64_t)z * total + i;
            if constexpr (VEC % 4 == 0) {
#pragma unroll
                for (int q = 0; q < VEC / 4; ++q) {
                    f32x4 v = *reinterpret_cast<const f32x4*>(p + 4 * q);
                    s[4 * q] += v.x; s[4 * q + 1] += v.y; s[4 * q + 2] += v.z; s[4 * q + 3] += v.w;
                }
            } else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) s[e] += p[e];
            }
        }
        OutT* out = C + (i / N) * ldc + (i % N);
        if constexpr (VEC == 8 && sizeof(OutT) == 2) {
            u32x4 pk = {pack_bf16(s[0], s[1]), pack_bf16(s[2], s[3]), pack_bf16(s[4], s[5]), pack_bf16(s[6], s[7])};
            *reinterpret_cast<u32x4*>(out) = pk;
        } else if constexpr (VEC == 4 && sizeof(OutT) == 4) {
            f32x4 v = {s[0], s[1], s[2], s[3]};
            if constexpr (SGD) sgd_apply4(sgd, i, v);
            else *reinterpret_cast<f32x4*>(out) = v;
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) out[e] = from_f32<OutT>(s[e]);
        }
    }
}

// The same sum for small fp32 results cut into many slices (weight gradients of narrow layers, whose
// reduction runs over all pixels): one thread per output would leave most of the chip idle and walk
// the slices one after the other, so LANES threads share a group of 4 outputs, thread l adds slices
// l, l + LANES, ... in ascending order and the LANES sums are combined by a pairwise tree.  Still a
// fixed order.
template <int LANES, bool SGD = false>
__global__ __launch_bounds__(256) void reduce_partials_wide_kernel(const float* __restrict__ partial, float* __restrict__ C,
                                                                   int64_t ldc, int64_t M, int64_t N, int splits,
                                                                   SgdArgs sgd = SgdArgs{})
{
    constexpr int GROUPS = 256 / LANES;       // groups of 4 outputs per block
    __shared__ f32x4 part[LANES][GROUPS + 1];
    const int64_t total = M * N, groups = total / 4;
    const int gl = threadIdx.x % GROUPS, l = threadIdx.x / GROUPS;
    const int64_t g = (int64_t)blockIdx.x * GROUPS + gl;
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    if (g < groups)
        for (int z = l; z < splits; z += LANES) s += *reinterpret_cast<const f32x4*>(partial + (int64_t)z * total + g * 4);
    part[l][gl] = s;
    __syncthreads();
    // pairwise tree over the LANES sums (lane l takes in lane l + half): one fixed order again
#pragma unroll
    for (int half = LANES / 2; half >= 1; half /= 2) {
        if (l < half) part[l][gl] += part[l + half][gl];
        __syncthreads();
    }
    if (l == 0 && g < groups) {
        const f32x4 t = part[0][gl];
        const int64_t i = g * 4;
        if constexpr (SGD) sgd_apply4(sgd, i, t);
        else *reinterpret_cast<f32x4*>(C + (i / N) * ldc + (i % N)) = t;
    }
}

// dst[i][j] (rows_d x cols_d, leading dimension ldd) = src[i][j] where it exists (i < rows_s, j < cols_s), else 0.
template <class T>
__global__ __launch_bounds__(256) void copy2d_kernel(const T* __restrict__ src, int64_t lds_, int64_t rows_s, int64_t cols_s,
                                                     T* __restrict__ dst, int64_t ldd, int64_t rows_d, int64_t cols_d)
{
    const int64_t total = rows_d * cols_d;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += stride) {
        int64_t i = e / cols_d, j = e - i * cols_d;
        T v = (T)0.f;
        if (i < rows_s && j < cols_s) v = src[i * lds_ + j];
        dst[i * ldd + j] = v;
    }
}

// w <- w - lr * (m <- mu * m + (g + wd * w)) on fp32 master weights; the compute copy (bf16 or fp32,
// optional) is refreshed from the new master value.
__global__ __launch_bounds__(256) void sgd_step_kernel(float* __restrict__ w, float* __restrict__ m, const float* __restrict__ g,
                                                       void* copy, bool copy_bf16, int64_t n, float lr, float mu, float wd)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const float wi = w[i];
        const float mi = fmaf(mu, m[i], fmaf(wd, wi, g[i]));
        const float wn = fmaf(-lr, mi, wi);
        m[i] = mi;
        w[i] = wn;
        if (copy) {
            if (copy_bf16) reinterpret_cast<bf16_t*>(copy)[i] = (bf16_t)wn;
            else reinterpret_cast<float*>(copy)[i] = wn;
        }
    }
}

// wt[i][k*k - 1 - t][o] = w[o][t][i]: the weights with which the data gradient of a stride-1
// convolution is itself a forward convolution (of dY, with padding k - 1 - pad).
__global__ __launch_bounds__(256) void flip_conv_weights_kernel(const bf16_t* __restrict__ w, bf16_t* __restrict__ wt, int O, int I,
                                                                int kk)
{
    const int total = O * kk * I;
    for (int e = blockIdx.x * 256 + threadIdx.x; e < total; e += gridDim.x * 256) {
        const int i = e / (kk * O), rem = e - i * kk * O;
        const int tf = rem / O, o = rem - tf * O;
        wt[e] = w[((int64_t)o * kk + (kk - 1 - tf)) * I + i];
    }
}

inline unsigned blocks_for(int64_t items)
{
    int64_t b = ceil_div(items, 256);
    if (b < 1) b = 1;
    if (b > 256 * 16) b = 256 * 16;
    return (unsigned)b;
}

}  // namespace

hipError_t gelu_fwd(const void* Z, void* A, int64_t n, bool bf16, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    if (bf16) hipLaunchKernelGGL(gelu_fwd_bf16, dim3(blocks_for(n / 8 + 1)), dim3(256), 0, st, (const bf16_t*)Z, (bf16_t*)A, n);
    else hipLaunchKernelGGL(gelu_fwd_f32, dim3(blocks_for(n)), dim3(256), 0, st, (const float*)Z, (float*)A, n);
    return hipGetLastError();
}

hipError_t gelu_bwd(const void* dA, const void* Z, void* dZ, int64_t n, bool bf16, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    if (bf16) hipLaunchKernelGGL(gelu_bwd_bf16, dim3(blocks_for(n / 8 + 1)), dim3(256), 0, st, (const bf16_t*)dA, (const bf16_t*)Z, (bf16_t*)dZ, n);
    else hipLaunchKernelGGL(gelu_bwd_f32, dim3(blocks_for(n)), dim3(256), 0, st, (const float*)dA, (const float*)Z, (float*)dZ, n);
    return hipGetLastError();
}

hipError_t column_sums(const void* dY, float* out, int64_t T, int64_t n, bool bf16, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    dim3 grid((unsigned)ceil_div(n, 64));
    if (bf16) hipLaunchKernelGGL(column_sums_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)dY, out, T, n);
    else hipLaunchKernelGGL(column_sums_kernel<float>, grid, dim3(256), 0, st, (const float*)dY, out, T, n);
    return hipGetLastError();
}

hipError_t copy2d(const void* src, int64_t ld_src, int64_t rows_src, int64_t cols_src, void* dst, int64_t ld_dst,
                  int64_t rows_dst, int64_t cols_dst, int elem_bytes, hipStream_t st)
{
    if (rows_dst <= 0 || cols_dst <= 0) return hipSuccess;
    dim3 grid(blocks_for(rows_dst * cols_dst));
    if (elem_bytes == 2)
        hipLaunchKernelGGL(copy2d_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)src, ld_src, rows_src, cols_src,
                           (bf16_t*)dst, ld_dst, rows_dst, cols_dst);
    else
        hipLaunchKernelGGL(copy2d_kernel<float>, grid, dim3(256), 0, st, (const float*)src, ld_src, rows_src, cols_src,
                           (float*)dst, ld_dst, rows_dst, cols_dst);
    return hipGetLastError();
}

hipError_t flip_conv_weights(const void* w, void* wt, int O, int I, int k, hipStream_t st)
{
    const int64_t total = (int64_t)O * k * k * I;
    if (total <= 0) return hipSuccess;
    hipLaunchKernelGGL(flip_conv_weights_kernel, dim3(blocks_for(total)), dim3(256), 0, st, (const bf16_t*)w, (bf16_t*)wt, O, I, k * k);
    return hipGetLastError();
}

hipError_t sgd_step(float* w, float* m, const float* g, void* copy, bool copy_bf16, int64_t n, float lr, float mu, float wd,
                    hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(sgd_step_kernel, dim3(blocks_for(n)), dim3(256), 0, st, w, m, g, copy, copy_bf16, n, lr, mu, wd);
    return hipGetLastError();
}

hipError_t reduce_partials(const float* partial, void* C, bool c_bf16, int64_t ldc, int64_t M, int64_t N, int splits,
                           hipStream_t st, const SgdFuse* sgd)
{
    if (M <= 0 || N <= 0) return hipSuccess;
    auto al16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
    const bool al = al16(C) && al16(partial);
    if (c_bf16) {
        if (al && N % 8 == 0 && ldc % 8 == 0)
            hipLaunchKernelGGL((reduce_partials_kernel<8, bf16_t>), dim3(blocks_for(M * N / 8)), dim3(256), 0, st, partial,
                               (bf16_t*)C, ldc, M, N, splits, SgdArgs{});
        else
            hipLaunchKernelGGL((reduce_partials_kernel<1, bf16_t>), dim3(blocks_for(M * N)), dim3(256), 0, st, partial,
                               (bf16_t*)C, ldc, M, N, splits, SgdArgs{});
        return hipGetLastError();
    }
    const bool vec4 = al && N % 4 == 0 && ldc % 4 == 0;
    const bool wide64 = vec4 && splits >= 64 && M * N / 4 <= 4096;
    const bool wide16 = vec4 && splits >= 16 && M * N / 4 < 256 * 256;
    if (sgd && !sgd->done && vec4 && ldc == N && al16(sgd->w) && al16(sgd->m) && (reinterpret_cast<uintptr_t>(sgd->copy) & 15u) == 0) {
        const SgdArgs a{sgd->w, sgd->m, sgd->copy, sgd->copy_bf16 ? 1 : 0, sgd->lr, sgd->mu, sgd->wd};
        if (wide64)
            hipLaunchKernelGGL((reduce_partials_wide_kernel<64, true>), dim3((unsigned)ceil_div(M * N / 4, 4)), dim3(256), 0, st,
                               partial, (float*)C, ldc, M, N, splits, a);
        else if (wide16)
            hipLaunchKernelGGL((reduce_partials_wide_kernel<16, true>), dim3((unsigned)ceil_div(M * N / 4, 16)), dim3(256), 0, st,
                               partial, (float*)C, ldc, M, N, splits, a);
        else
            hipLaunchKernelGGL((reduce_partials_kernel<4, float, true>), dim3(blocks_for(M * N / 4)), dim3(256), 0, st, partial,
                               (float*)C, ldc, M, N, splits, a);
        sgd->done = true;
        return hipGetLastError();
    }
    if (wide64)
        hipLaunchKernelGGL((reduce_partials_wide_kernel<64>), dim3((unsigned)ceil_div(M * N / 4, 4)), dim3(256), 0, st, partial,
                           (float*)C, ldc, M, N, splits, SgdArgs{});
    else if (wide16)
        hipLaunchKernelGGL((reduce_partials_wide_kernel<16>), dim3((unsigned)ceil_div(M * N / 4, 16)), dim3(256), 0, st, partial,
                           (float*)C, ldc, M, N, splits, SgdArgs{});
    else if (vec4)
        hipLaunchKernelGGL((reduce_partials_kernel<4, float>), dim3(blocks_for(M * N / 4)), dim3(256), 0, st, partial,
                           (float*)C, ldc, M, N, splits, SgdArgs{});
    else
        hipLaunchKernelGGL((reduce_partials_kernel<1, float>), dim3(blocks_for(M * N)), dim3(256), 0, st, partial,
                           (float*)C, ldc, M, N, splits, SgdArgs{});
    return hipGetLastError();
}

}  // namespace lrd
