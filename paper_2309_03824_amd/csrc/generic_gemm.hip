// General tile kernel: any operand strides, any alignment, optional convolution gather, fp32 FMA
// accumulation.  It backs the fp32 path and every bf16 shape the MFMA engine does not take.
#include "lrd_internal.hpp"

namespace lrd {
namespace {

constexpr int GT = 64;   // output tile edge
constexpr int GK = 16;   // K step

template <class T, int G>
struct Loader {
    const T* A;
    const T* B;
    int64_t a_sm, a_sk, b_sn, b_sk;
    int64_t M, N, K;
    ConvShape cs;

    __device__ __forceinline__ float a(int64_t m, int64_t k) const
    {
        if (m >= M || k >= K) return 0.f;
        if constexpr (G == GATHER_CONV_FWD) {
            // m = (n, y, x) over the output grid; k = (u, v, i)
            int i = (int)(k % cs.I);
            int tap = (int)(k / cs.I);
            int v = tap % cs.k, u = tap / cs.k;
            int x = (int)(m % cs.Wo);
            int64_t q = m / cs.Wo;
            int y = (int)(q % cs.Ho);
            int64_t n = q / cs.Ho;
            int yy = y * cs.stride + u - cs.pad, xx = x * cs.stride + v - cs.pad;
            if (yy < 0 || yy >= cs.H || xx < 0 || xx >= cs.W) return 0.f;
            return to_f32(A[((n * cs.H + yy) * cs.W + xx) * cs.I + i]);
        } else if constexpr (G == GATHER_CONV_DGRAD) {
            // m = (n, a, b) over the input grid; k = (u, v, o); A is the output-side gradient
            int o = (int)(k % cs.O);
            int tap = (int)(k / cs.O);
            int v = tap % cs.k, u = tap / cs.k;
            int b = (int)(m % cs.W);
            int64_t q = m / cs.W;
            int a_ = (int)(q % cs.H);
            int64_t n = q / cs.H;
            int ys = a_ + cs.pad - u, xs = b + cs.pad - v;
            if (ys < 0 || xs < 0 || ys % cs.stride != 0 || xs % cs.stride != 0) return 0.f;
            int y = ys / cs.stride, x = xs / cs.stride;
            if (y >= cs.Ho || x >= cs.Wo) return 0.f;
            return to_f32(A[((n * cs.Ho + y) * cs.Wo + x) * cs.O + o]);
        } else {
            return to_f32(A[m * a_sm + k * a_sk]);
        }
    }

    __device__ __forceinline__ float b(int64_t n, int64_t k) const
    {
        if (n >= N || k >= K) return 0.f;
        if constexpr (G == GATHER_CONV_DGRAD) {
            // n = i; k = (u, v, o); weight stored [o][u][v][i]
            int o = (int)(k % cs.O);
            int tap = (int)(k / cs.O);
            return to_f32(B[((int64_t)o * cs.k * cs.k + tap) * cs.I + n]);
        } else if constexpr (G == GATHER_CONV_WGRAD) {
            // n = (u, v, i); k = (img, y, x) over the output grid; B is the layer input
            int i = (int)(n % cs.I);
            int tap = (int)(n / cs.I);
            int v = tap % cs.k, u = tap / cs.k;
            int x = (int)(k % cs.Wo);
            int64_t q = k / cs.Wo;
            int y = (int)(q % cs.Ho);
            int64_t img = q / cs.Ho;
            int yy = y * cs.stride + u - cs.pad, xx = x * cs.stride + v - cs.pad;
            if (yy < 0 || yy >= cs.H || xx < 0 || xx >= cs.W) return 0.f;
            return to_f32(B[((img * cs.H + yy) * cs.W + xx) * cs.I + i]);
        } else {
            return to_f32(B[n * b_sn + k * b_sk]);
        }
    }
};

template <class T, class TOut, int G>
__global__ __launch_bounds__(256) void generic_gemm_kernel(Loader<T, G> ld, TOut* C, int64_t ldc,
                                                           const float* bias, float* partial,
                                                           int64_t k_per_split)
{
    __shared__ float As[GK][GT + 4];
    __shared__ float Bs[GK][GT + 4];
    const int tid = threadIdx.x;
    const int tx = tid % 16, ty = tid / 16;
    const int64_t m0 = (int64_t)blockIdx.x * GT, n0 = (int64_t)blockIdx.y * GT;
    const int64_t kbeg = (int64_t)blockIdx.z * k_per_split;
    int64_t kend = kbeg + k_per_split;
    if (kend > ld.K) kend = ld.K;

    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

    for (int64_t k0 = kbeg; k0 < kend; k0 += GK) {
        // 64 x 16 elements per operand, 4 per thread; consecutive threads walk k first when the
        // operand is k-contiguous, rows first otherwise (chosen by stride at run time).
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            int idx = tid + e * 256;
            int kk, rr;
            if (ld.a_sk == 1 || G == GATHER_CONV_FWD || G == GATHER_CONV_DGRAD) { kk = idx % GK; rr = idx / GK; }
            else { rr = idx % GT; kk = idx / GT; }
            int64_t k = k0 + kk;
            As[kk][rr] = (k < kend) ? ld.a(m0 + rr, k) : 0.f;
            if (ld.b_sk == 1 && G != GATHER_CONV_WGRAD) { kk = idx % GK; rr = idx / GK; }
            else { rr = idx % GT; kk = idx / GT; }
            k = k0 + kk;
            Bs[kk][rr] = (k < kend) ? ld.b(n0 + rr, k) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < GK; ++kk) {
            float av[4], bv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) av[i] = As[kk][ty + 16 * i];
#pragma unroll
            for (int j = 0; j < 4; ++j) bv[j] = Bs[kk][tx + 16 * j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
        }
        __syncthreads();
    }

#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int64_t m = m0 + ty + 16 * i;
        if (m >= ld.M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int64_t n = n0 + tx + 16 * j;
            if (n >= ld.N) continue;
            if (partial) {
                partial[((int64_t)blockIdx.z * ld.M + m) * ld.N + n] = acc[i][j];
            } else {
                float v = acc[i][j] + (bias ? bias[n] : 0.f);
                C[m * ldc + n] = from_f32<TOut>(v);
            }
        }
    }
}

template <class T, class TOut, int G>
hipError_t launch(const MatOp& op, hipStream_t st)
{
    Loader<T, G> ld;
    ld.A = (const T*)op.A;
    ld.B = (const T*)op.B;
    ld.a_sm = op.a_sm; ld.a_sk = op.a_sk; ld.b_sn = op.b_sn; ld.b_sk = op.b_sk;
    ld.M = op.M; ld.N = op.N; ld.K = op.K;
    ld.cs = op.cs;
    int splits = (op.splits > 1 && op.partial) ? op.splits : 1;
    int64_t kps = ceil_div(ceil_div(op.K, splits), GK) * GK;
    splits = (int)ceil_div(op.K, kps);
    dim3 grid((unsigned)ceil_div(op.M, GT), (unsigned)ceil_div(op.N, GT), (unsigned)splits);
    float* partial = splits > 1 ? op.partial : nullptr;
    hipLaunchKernelGGL((generic_gemm_kernel<T, TOut, G>), grid, dim3(256), 0, st, ld, (TOut*)op.C,
                       op.ldc, op.bias, partial, kps);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (splits > 1) return reduce_partials(op.partial, op.C, false, op.ldc, op.M, op.N, splits, st, op.sgd);
    return hipSuccess;
}

template <class T, class TOut>
hipError_t by_gather(const MatOp& op, hipStream_t st)
{
    switch (op.gather) {
        case GATHER_NONE: return launch<T, TOut, GATHER_NONE>(op, st);
        case GATHER_CONV_FWD: return launch<T, TOut, GATHER_CONV_FWD>(op, st);
        case GATHER_CONV_DGRAD: return launch<T, TOut, GATHER_CONV_DGRAD>(op, st);
        case GATHER_CONV_WGRAD: return launch<T, TOut, GATHER_CONV_WGRAD>(op, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t generic_matop(const MatOp& op, hipStream_t st)
{
    note_kernel("generic_gemm_kernel (FMA tiles)");
    if (op.M <= 0 || op.N <= 0) return hipSuccess;
    // Split-K output goes through fp32 partials, so it is only offered for fp32 results.
    if (op.splits > 1 && !op.out_f32) return hipErrorInvalidValue;
    if (op.in_bf16) {
        if (op.out_f32) return by_gather<bf16_t, float>(op, st);
        return by_gather<bf16_t, bf16_t>(op, st);
    }
    return by_gather<float, float>(op, st);
}

}  // namespace lrd
