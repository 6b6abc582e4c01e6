// One-time factorization on the device (eq. 1, 2: truncated SVD of a layer weight; eq. 4: Tucker-2
// of a convolution weight by higher-order SVD on its two channel modes).
//
// The SVD is one-sided (Hestenes) Jacobi in fp64 on the ROWS of a row-major matrix M [p x q],
// p <= q (the weight or its transpose): plane rotations make the rows mutually orthogonal, the
// same rotations applied to Q (initially the identity) collect the left vectors.  At convergence
// row i of M is sigma_i times a right singular vector and row i of Q the matching left vector.
// Rows are contiguous, so every access is coalesced; the p/2 disjoint pairs of a round-robin
// tournament step are independent and run as one launch, one workgroup per pair.  A sweep is
// p - 1 (p even) or p (p odd) such steps; after each sweep the host reads the number of rotations
// applied and stops at zero.  These calls therefore synchronise the stream.
//
// A matrix at least twice as wide as it is tall is preconditioned first: the same iteration runs on
// its small Gram matrix G = M.M^T [p x p] (rows of length p instead of q, a fraction of the traffic
// per sweep), collecting the rotations in Q; then M is replaced by Q.M, whose rows are already
// orthogonal up to the tolerance of that first phase, and the iteration proper needs only the sweep
// that finds nothing left to rotate (or one or two more) instead of a dozen.  The convergence test and its
// tolerance on the rows of M are the same either way, so the result has the accuracy of the plain
// iteration; the Gram matrix only supplies the starting basis.
#include <algorithm>
#include <cmath>
#include <numeric>
#include <vector>

#include "lrd.h"
#include "lrd_internal.hpp"

namespace lrd {
namespace {

constexpr int FT = 256;                 // threads per workgroup in this file
constexpr double JACOBI_TOL = 1e-14;    // rows count as orthogonal when |a.b| <= tol * |a| |b|
// The same test on the rows of the Gram matrix.  Taken as tight as the main one: 13 sweeps there and a single
// (empty) sweep on M for a 768 x 3072 weight, against 12 + 3 at 1e-11 and 11 + 5 at 1e-7; a sweep on the
// Gram matrix costs a fraction of one on M.
constexpr double GRAM_TOL = 1e-14;
constexpr int MAX_SWEEPS = 60;

inline bool preconditioned(int64_t p, int64_t q) { return p >= 32 && q >= 2 * p; }

inline size_t round256(size_t b) { return (b + 255) & ~size_t(255); }

// M[i][j] = transpose ? W[j][i] : W[i][j]  (W row-major with leading dimension ldw), Q = identity.
// Every kernel of the Jacobi iteration takes a batch of problems of one shape: blockIdx.y selects the
// matrix, consecutive matrices lie bw / bm / bq elements apart (W, M, Q).
struct BatchStride { int64_t bw = 0, bm = 0, bq = 0; };

__global__ __launch_bounds__(FT) void load_matrix_kernel(const float* __restrict__ W, int64_t ldw, bool transpose,
                                                         double* __restrict__ M, double* __restrict__ Q, int p, int q, BatchStride bs)
{
    W += blockIdx.y * bs.bw; M += blockIdx.y * bs.bm; Q += blockIdx.y * bs.bq;
    const int64_t total = (int64_t)p * q, stride = (int64_t)gridDim.x * FT;
    for (int64_t e = (int64_t)blockIdx.x * FT + threadIdx.x; e < total; e += stride) {
        int i = (int)(e / q), j = (int)(e - (int64_t)i * q);
        M[e] = (double)(transpose ? W[(int64_t)j * ldw + i] : W[(int64_t)i * ldw + j]);
    }
    const int64_t tq = (int64_t)p * p;
    for (int64_t e = (int64_t)blockIdx.x * FT + threadIdx.x; e < tq; e += stride) {
        int i = (int)(e / p), j = (int)(e - (int64_t)i * p);
        Q[e] = i == j ? 1.0 : 0.0;
    }
}

__device__ __forceinline__ double block_sum(double v, double* scratch)
{
    const int tid = threadIdx.x;
    scratch[tid] = v;
    __syncthreads();
#pragma unroll
    for (int s = FT / 2; s > 0; s >>= 1) {
        if (tid < s) scratch[tid] += scratch[tid + s];
        __syncthreads();
    }
    double r = scratch[0];
    __syncthreads();
    return r;
}

// One step of the round-robin ordering on n players (n even; player n - 1 stays, the others
// rotate): workgroup k pairs (n - 1, step) for k = 0 and ((step + k) mod (n - 1), (step - k) mod (n - 1))
// otherwise.  Players >= p are byes.
__global__ __launch_bounds__(FT) void jacobi_step_kernel(double* __restrict__ M, double* __restrict__ Q, int p, int q, int n,
                                                         int step, double tol, unsigned int* __restrict__ rotations, BatchStride bs)
{
    M += blockIdx.y * bs.bm; Q += blockIdx.y * bs.bq;
    static_assert(FT == 256, "four waves per workgroup");
    __shared__ double scratch[12];
    __shared__ double cs[2];
    const int k = blockIdx.x, m = n - 1;
    int a, b;
    if (k == 0) {
        a = n - 1;
        b = step;
    } else {
        a = (step + k) % m;
        b = (step - k + m) % m;
    }
    if (a >= p || b >= p) return;
    if (a > b) { int t = a; a = b; b = t; }
    double* ra = M + (int64_t)a * q;
    double* rb = M + (int64_t)b * q;
    double saa = 0.0, sbb = 0.0, sab = 0.0;
    for (int j = threadIdx.x; j < q; j += FT) {
        double x = ra[j], y = rb[j];
        saa += x * x;
        sbb += y * y;
        sab += x * y;
    }
    // the three sums in one pass: within each wave by lane shuffles, across the four waves through LDS
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        saa += __shfl_down(saa, off);
        sbb += __shfl_down(sbb, off);
        sab += __shfl_down(sab, off);
    }
    if ((threadIdx.x & 63) == 0) {
        const int w = threadIdx.x >> 6;
        scratch[3 * w] = saa;
        scratch[3 * w + 1] = sbb;
        scratch[3 * w + 2] = sab;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        const double alpha = (scratch[0] + scratch[3]) + (scratch[6] + scratch[9]);
        const double beta = (scratch[1] + scratch[4]) + (scratch[7] + scratch[10]);
        const double gamma = (scratch[2] + scratch[5]) + (scratch[8] + scratch[11]);
        double c = 1.0, s = 0.0;
        if (gamma != 0.0 && fabs(gamma) > tol * sqrt(alpha * beta)) {
            const double zeta = (beta - alpha) / (2.0 * gamma);
            const double t = (zeta >= 0.0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
            c = 1.0 / sqrt(1.0 + t * t);
            s = c * t;
            atomicAdd(rotations, 1u);
        }
        cs[0] = c;
        cs[1] = s;
    }
    __syncthreads();
    const double c = cs[0], s = cs[1];
    if (s == 0.0) return;
    for (int j = threadIdx.x; j < q; j += FT) {
        double x = ra[j], y = rb[j];
        ra[j] = c * x - s * y;
        rb[j] = s * x + c * y;
    }
    double* qa = Q + (int64_t)a * p;
    double* qb = Q + (int64_t)b * p;
    for (int j = threadIdx.x; j < p; j += FT) {
        double x = qa[j], y = qb[j];
        qa[j] = c * x - s * y;
        qb[j] = s * x + c * y;
    }
}

// sigma[i] = |row i of M|
__global__ __launch_bounds__(FT) void row_norms_kernel(const double* __restrict__ M, int q, double* __restrict__ sigma, BatchStride bs)
{
    __shared__ double scratch[FT];
    M += blockIdx.y * bs.bm; sigma += (int64_t)blockIdx.y * gridDim.x;
    const double* r = M + (int64_t)blockIdx.x * q;
    double s = 0.0;
    for (int j = threadIdx.x; j < q; j += FT) s += r[j] * r[j];
    s = block_sum(s, scratch);
    if (threadIdx.x == 0) sigma[blockIdx.x] = sqrt(s);
}

// Rank-r pair with the singular values shared evenly (eq. 2).  order[j] = row holding the j-th
// largest singular value.  wide (M = W): V[j][:] = M[row] / sqrt(sigma), U[:, j] = Q[row] * sqrt(sigma).
// Otherwise (M = W^T) the roles of the two row spaces swap.
__global__ __launch_bounds__(FT) void emit_pair_kernel(const double* __restrict__ M, const double* __restrict__ Q,
                                                       const double* __restrict__ sigma, const int* __restrict__ order, int p,
                                                       int q, int r, bool wide, float* __restrict__ U, float* __restrict__ V,
                                                       BatchStride bs, int64_t ustride, int64_t vstride)
{
    M += blockIdx.y * bs.bm; Q += blockIdx.y * bs.bq; sigma += (int64_t)blockIdx.y * p; order += (int64_t)blockIdx.y * p;
    U += blockIdx.y * ustride; V += blockIdx.y * vstride;
    const int j = blockIdx.x, row = order[j];
    const double sg = sigma[row];
    const double down = sg > 0.0 ? 1.0 / sqrt(sg) : 0.0, up = sqrt(sg);
    const double* mr = M + (int64_t)row * q;   // sigma * vector in q-space
    const double* qr = Q + (int64_t)row * p;   // unit vector in p-space
    if (wide) {      // out = p, in = q
        for (int i = threadIdx.x; i < q; i += FT) V[(int64_t)j * q + i] = (float)(mr[i] * down);
        for (int o = threadIdx.x; o < p; o += FT) U[(int64_t)o * r + j] = (float)(qr[o] * up);
    } else {         // in = p, out = q
        for (int i = threadIdx.x; i < p; i += FT) V[(int64_t)j * p + i] = (float)(qr[i] * up);
        for (int o = threadIdx.x; o < q; o += FT) U[(int64_t)o * r + j] = (float)(mr[o] * down);
    }
}

// Leading left singular vectors as rows: B[j][:] (length p) = Q[order[j]] (M = unfolding, p <= q) or
// (length q) = M[order[j]] / sigma (M = unfolding^T).
__global__ __launch_bounds__(FT) void emit_basis_kernel(const double* __restrict__ M, const double* __restrict__ Q,
                                                        const double* __restrict__ sigma, const int* __restrict__ order, int p,
                                                        int q, bool from_q, double* __restrict__ B)
{
    const int j = blockIdx.x, row = order[j];
    if (from_q) {
        for (int i = threadIdx.x; i < p; i += FT) B[(int64_t)j * p + i] = Q[(int64_t)row * p + i];
    } else {
        const double sg = sigma[row], inv = sg > 0.0 ? 1.0 / sg : 0.0;
        for (int i = threadIdx.x; i < q; i += FT) B[(int64_t)j * q + i] = M[(int64_t)row * q + i] * inv;
    }
}

// Mode-C unfolding of W [S][kk][C]: Mc[c][(o, t)] = W[o][t][c]  (transpose = false), or its transpose.
__global__ __launch_bounds__(FT) void unfold_c_kernel(const float* __restrict__ W, int S, int kk, int C, bool transpose,
                                                      double* __restrict__ M, double* __restrict__ Q, int p)
{
    const int64_t cols = (int64_t)S * kk, total = cols * C, stride = (int64_t)gridDim.x * FT;
    for (int64_t e = (int64_t)blockIdx.x * FT + threadIdx.x; e < total; e += stride) {
        int64_t ot = e / C;
        int c = (int)(e - ot * C);
        M[transpose ? ot * C + c : (int64_t)c * cols + ot] = (double)W[e];
    }
    const int64_t tq = (int64_t)p * p;
    for (int64_t e = (int64_t)blockIdx.x * FT + threadIdx.x; e < tq; e += stride) {
        int i = (int)(e / p), j = (int)(e - (int64_t)i * p);
        Q[e] = i == j ? 1.0 : 0.0;
    }
}

// tmp[o][t][a] = sum_c W[o][t][c] B1[a][c]
__global__ __launch_bounds__(FT) void core_step1_kernel(const float* __restrict__ W, const double* __restrict__ B1, int64_t rows,
                                                        int C, int r1, double* __restrict__ tmp)
{
    const int64_t total = rows * r1, stride = (int64_t)gridDim.x * FT;
    for (int64_t e = (int64_t)blockIdx.x * FT + threadIdx.x; e < total; e += stride) {
        int64_t ot = e / r1;
        int a = (int)(e - ot * r1);
        double s = 0.0;
        for (int c = 0; c < C; ++c) s += (double)W[ot * C + c] * B1[(int64_t)a * C + c];
        tmp[e] = s;
    }
}

// G[b][t][a] = sum_o B2[b][o] tmp[o][t][a];  also the factor outputs P1 = B1, P2[o][b] = B2[b][o].
__global__ __launch_bounds__(FT) void core_step2_kernel(const double* __restrict__ tmp, const double* __restrict__ B1,
                                                        const double* __restrict__ B2, int S, int kk, int C, int r1, int r2,
                                                        float* __restrict__ G, float* __restrict__ P1, float* __restrict__ P2)
{
    const int64_t inner = (int64_t)kk * r1, total = (int64_t)r2 * inner, stride = (int64_t)gridDim.x * FT;
    for (int64_t e = (int64_t)blockIdx.x * FT + threadIdx.x; e < total; e += stride) {
        int b = (int)(e / inner);
        int64_t ta = e - (int64_t)b * inner;
        double s = 0.0;
        for (int o = 0; o < S; ++o) s += B2[(int64_t)b * S + o] * tmp[(int64_t)o * inner + ta];
        G[e] = (float)s;
    }
    for (int64_t e = (int64_t)blockIdx.x * FT + threadIdx.x; e < (int64_t)r1 * C; e += stride) P1[e] = (float)B1[e];
    for (int64_t e = (int64_t)blockIdx.x * FT + threadIdx.x; e < (int64_t)S * r2; e += stride) {
        int o = (int)(e / r2), b = (int)(e - (int64_t)o * r2);
        P2[e] = (float)B2[(int64_t)b * S + o];
    }
}

// C[m x n] = A[m x k] . B^T (BT: B is [n x k]) or A . B (B is [k x n]), row-major fp64, 64 x 64 tiles of C per
// workgroup, 4 x 4 results per thread, 16-deep steps through LDS.  Used twice per preconditioned problem.
template <bool BT>
__global__ __launch_bounds__(FT) void product_f64_kernel(const double* __restrict__ A, const double* __restrict__ B, double* __restrict__ C,
                                                         int m, int n, int k, int64_t a_bs, int64_t b_bs, int64_t c_bs)
{
    A += blockIdx.z * a_bs; B += blockIdx.z * b_bs; C += blockIdx.z * c_bs;
    __shared__ double As[16][65], Bs[16][65];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int i0 = blockIdx.y * 64, j0 = blockIdx.x * 64;
    double acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = 0.0;
    for (int k0 = 0; k0 < k; k0 += 16) {
        // A tile: 64 rows x 16 k, element e -> row e / 16, k e % 16 (k contiguous in memory)
#pragma unroll
        for (int e = tid; e < 64 * 16; e += FT) {
            const int r = e >> 4, kk = e & 15;
            As[kk][r] = (i0 + r < m && k0 + kk < k) ? A[(int64_t)(i0 + r) * k + k0 + kk] : 0.0;
        }
        if (BT) {
#pragma unroll
            for (int e = tid; e < 64 * 16; e += FT) {
                const int r = e >> 4, kk = e & 15;
                Bs[kk][r] = (j0 + r < n && k0 + kk < k) ? B[(int64_t)(j0 + r) * k + k0 + kk] : 0.0;
            }
        } else {
#pragma unroll
            for (int e = tid; e < 64 * 16; e += FT) {
                const int kk = e >> 6, c = e & 63;
                Bs[kk][c] = (j0 + c < n && k0 + kk < k) ? B[(int64_t)(k0 + kk) * n + j0 + c] : 0.0;
            }
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            double a[4], b[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) { a[u] = As[kk][ty + 16 * u]; b[u] = Bs[kk][tx + 16 * u]; }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[u][v] = fma(a[u], b[v], acc[u][v]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int i = i0 + ty + 16 * u, j = j0 + tx + 16 * v;
            if (i < m && j < n) C[(int64_t)i * n + j] = acc[u][v];
        }
}

inline unsigned blocks_for(int64_t items)
{
    int64_t b = (items + FT - 1) / FT;
    return (unsigned)std::min<int64_t>(std::max<int64_t>(b, 1), 256 * 32);
}

struct JacobiBuffers {
    double* M;       // [p x q]
    double* Q;       // [p x p]
    double* sigma;   // [p]
    int* order;      // [p]
    unsigned int* rotations;
    double* G = nullptr;    // [p x p] Gram matrix and [p x q] rotated copy of M, preconditioned problems only
    double* M2 = nullptr;
};

size_t jacobi_bytes(int64_t p, int64_t q, int64_t batch = 1)
{
    size_t b = round256((size_t)batch * p * q * 8) + round256((size_t)batch * p * p * 8) + round256((size_t)batch * p * 8) +
               round256((size_t)batch * p * 4) + 256;
    if (preconditioned(p, q)) b += round256((size_t)batch * p * p * 8) + round256((size_t)batch * p * q * 8);
    return b;
}

JacobiBuffers carve_jacobi(char*& at, int64_t p, int64_t q, int64_t batch = 1)
{
    JacobiBuffers jb;
    jb.M = (double*)at;            at += round256((size_t)batch * p * q * 8);
    jb.Q = (double*)at;            at += round256((size_t)batch * p * p * 8);
    jb.sigma = (double*)at;        at += round256((size_t)batch * p * 8);
    jb.order = (int*)at;           at += round256((size_t)batch * p * 4);
    jb.rotations = (unsigned int*)at; at += 256;
    if (preconditioned(p, q)) {
        jb.G = (double*)at;        at += round256((size_t)batch * p * p * 8);
        jb.M2 = (double*)at;       at += round256((size_t)batch * p * q * 8);
    }
    return jb;
}

// Matrices of a batch factorized together: as many as keep the iteration's working set (M and Q of
// every matrix, read and written once per tournament step) inside the last-level cache.
int64_t jacobi_chunk(int64_t p, int64_t q, int64_t batch)
{
    const int64_t per = (p * q + p * p) * 8;
    return std::max<int64_t>(1, std::min<int64_t>(batch, (int64_t(96) << 20) / std::max<int64_t>(per, 1)));
}

// Sweeps until no pair rotates (in any matrix of the batch: one counter, one host read per sweep); then
// singular values to the host, descending order to the device (both [batch][p]).
// Returns the sweeps used, or -1 on a runtime error, -2 if MAX_SWEEPS did not suffice.
// Sweeps on the rows of Mx [p x len] (rotations collected in Q) until a sweep rotates nothing; returns the
// sweeps used, -1 on a runtime error, -2 when MAX_SWEEPS did not suffice.
int sweep_until_orthogonal(double* Mx, double* Q, unsigned int* rotations, int p, int len, double tol, hipStream_t st, int batch,
                           BatchStride bs)
{
    const int n = (p + 1) & ~1;       // players of the tournament (one bye when p is odd)
    int sweeps = 0;
    bool converged = p < 2;
    while (!converged && sweeps < MAX_SWEEPS) {
        // the counter is cleared by a kernel-free path the stream orders with the launches
        if (hipMemsetAsync(rotations, 0, sizeof(unsigned int), st) != hipSuccess) return -1;
        for (int step = 0; step < n - 1; ++step)
            hipLaunchKernelGGL(jacobi_step_kernel, dim3(n / 2, batch), dim3(FT), 0, st, Mx, Q, p, len, n, step, tol, rotations, bs);
        if (hipGetLastError() != hipSuccess) return -1;
        unsigned int count = 0;
        if (hipMemcpyAsync(&count, rotations, sizeof count, hipMemcpyDeviceToHost, st) != hipSuccess) return -1;
        if (hipStreamSynchronize(st) != hipSuccess) return -1;
        ++sweeps;
        converged = count == 0;
    }
    return converged ? sweeps : -2;
}

int run_jacobi(JacobiBuffers& jb, int p, int q, std::vector<double>& sigma_host, std::vector<int>& order_host, hipStream_t st,
               int batch = 1, BatchStride bs = BatchStride{})
{
    int sweeps = 0;
    if (jb.G && jb.M2) {
        // starting basis from the Gram matrix: G = M.M^T, rows of G made orthogonal (rotations into Q), M <- Q.M
        const int64_t sm = (int64_t)p * q, sq = (int64_t)p * p;
        BatchStride gs = bs;
        gs.bm = sq;                      // the "matrix" of this phase is G: stride p*p, row length p
        gs.bq = sq;
        const unsigned tp = (unsigned)((p + 63) / 64), tq = (unsigned)((q + 63) / 64);
        hipLaunchKernelGGL((product_f64_kernel<true>), dim3(tp, tp, batch), dim3(FT), 0, st, jb.M, jb.M, jb.G, p, p, q, sm, sm, sq);
        if (hipGetLastError() != hipSuccess) return -1;
        const int pre = sweep_until_orthogonal(jb.G, jb.Q, jb.rotations, p, p, GRAM_TOL, st, batch, gs);
        if (pre == -1) return -1;        // (not converged within the limit is no error here: the main phase finishes the job)
        sweeps += pre > 0 ? pre : MAX_SWEEPS;
        hipLaunchKernelGGL((product_f64_kernel<false>), dim3(tq, tp, batch), dim3(FT), 0, st, jb.Q, jb.M, jb.M2, p, q, p, sq, sm, sm);
        if (hipGetLastError() != hipSuccess) return -1;
        std::swap(jb.M, jb.M2);
    }
    BatchStride ms = bs;
    ms.bm = (int64_t)p * q;
    ms.bq = (int64_t)p * p;
    const int main_sweeps = sweep_until_orthogonal(jb.M, jb.Q, jb.rotations, p, q, JACOBI_TOL, st, batch, ms);
    if (main_sweeps < 0) return main_sweeps;
    sweeps += main_sweeps;
    hipLaunchKernelGGL(row_norms_kernel, dim3(p, batch), dim3(FT), 0, st, jb.M, q, jb.sigma, bs);
    sigma_host.resize((size_t)p * batch);
    if (hipMemcpyAsync(sigma_host.data(), jb.sigma, (size_t)p * batch * 8, hipMemcpyDeviceToHost, st) != hipSuccess) return -1;
    if (hipStreamSynchronize(st) != hipSuccess) return -1;
    order_host.resize((size_t)p * batch);
    for (int b = 0; b < batch; ++b) {
        int* ord = order_host.data() + (size_t)b * p;
        const double* sg = sigma_host.data() + (size_t)b * p;
        std::iota(ord, ord + p, 0);
        std::stable_sort(ord, ord + p, [&](int x, int y) { return sg[x] > sg[y]; });
    }
    if (hipMemcpyAsync(jb.order, order_host.data(), (size_t)p * batch * 4, hipMemcpyHostToDevice, st) != hipSuccess) return -1;
    if (hipStreamSynchronize(st) != hipSuccess) return -1;     // order_host may be reused by the caller
    return sweeps;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace
}  // namespace lrd

using namespace lrd;

extern "C" {

size_t lrd_svd_factors_workspace_bytes(int64_t out, int64_t in)
{
    if (out < 1 || in < 1 || out >= (int64_t(1) << 20) || in >= (int64_t(1) << 20)) return 0;
    return jacobi_bytes(std::min(out, in), std::max(out, in));
}

lrd_status lrd_svd_factors(const float* W, int64_t out, int64_t in, int64_t r, float* U, float* V, double* sigma_host,
                           int32_t* sweeps_host, void* ws, size_t ws_bytes, void* hip_stream)
{
    if (!W || !U || !V || out < 1 || in < 1 || r < 1 || r > std::min(out, in)) return LRD_ERR_INVALID_ARG;
    if (out >= (int64_t(1) << 20) || in >= (int64_t(1) << 20)) return LRD_ERR_INVALID_ARG;
    if (!aligned16(W) || !aligned16(U) || !aligned16(V) || !aligned16(ws)) return LRD_ERR_ALIGNMENT;
    if (!ws || ws_bytes < lrd_svd_factors_workspace_bytes(out, in)) return LRD_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    const bool wide = out <= in;                 // M = W when its rows are the short side, else M = W^T
    const int p = (int)std::min(out, in), q = (int)std::max(out, in);
    char* at = (char*)ws;
    JacobiBuffers jb = carve_jacobi(at, p, q);
    hipLaunchKernelGGL(load_matrix_kernel, dim3(blocks_for((int64_t)p * q)), dim3(FT), 0, st, W, in, !wide, jb.M, jb.Q, p, q, BatchStride{});
    if (hipGetLastError() != hipSuccess) return LRD_ERR_RUNTIME;
    std::vector<double> sg;
    std::vector<int> order;
    const int sweeps = run_jacobi(jb, p, q, sg, order, st);
    if (sweeps < 0) return LRD_ERR_RUNTIME;
    hipLaunchKernelGGL(emit_pair_kernel, dim3((unsigned)r), dim3(FT), 0, st, jb.M, jb.Q, jb.sigma, jb.order, p, q, (int)r, wide, U, V,
                       BatchStride{}, (int64_t)0, (int64_t)0);
    if (hipGetLastError() != hipSuccess || hipStreamSynchronize(st) != hipSuccess) return LRD_ERR_RUNTIME;
    if (sigma_host)
        for (int j = 0; j < p; ++j) sigma_host[j] = sg[order[j]];
    if (sweeps_host) *sweeps_host = sweeps;
    return LRD_OK;
}

size_t lrd_svd_factors_batched_workspace_bytes(int64_t batch, int64_t out, int64_t in)
{
    if (batch < 1 || out < 1 || in < 1 || out >= (int64_t(1) << 20) || in >= (int64_t(1) << 20)) return 0;
    const int64_t p = std::min(out, in), q = std::max(out, in);
    return jacobi_bytes(p, q, jacobi_chunk(p, q, batch));
}

lrd_status lrd_svd_factors_batched(const float* W, int64_t batch, int64_t out, int64_t in, int64_t r, float* U, float* V,
                                   double* sigma_host, int32_t* sweeps_host, void* ws, size_t ws_bytes, void* hip_stream)
{
    if (!W || !U || !V || batch < 1 || batch > 65535 || out < 1 || in < 1 || r < 1 || r > std::min(out, in)) return LRD_ERR_INVALID_ARG;
    if (out >= (int64_t(1) << 20) || in >= (int64_t(1) << 20)) return LRD_ERR_INVALID_ARG;
    if (!aligned16(W) || !aligned16(U) || !aligned16(V) || !aligned16(ws)) return LRD_ERR_ALIGNMENT;
    if (!ws || ws_bytes < lrd_svd_factors_batched_workspace_bytes(batch, out, in)) return LRD_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    const bool wide = out <= in;
    const int p = (int)std::min(out, in), q = (int)std::max(out, in);
    const int64_t chunk = jacobi_chunk(p, q, batch);
    std::vector<double> sg;
    std::vector<int> order;
    int max_sweeps = 0;
    for (int64_t b0 = 0; b0 < batch; b0 += chunk) {
        const int nb = (int)std::min(chunk, batch - b0);
        char* at = (char*)ws;
        JacobiBuffers jb = carve_jacobi(at, p, q, chunk);
        BatchStride bs;
        bs.bw = out * in; bs.bm = (int64_t)p * q; bs.bq = (int64_t)p * p;
        hipLaunchKernelGGL(load_matrix_kernel, dim3(blocks_for((int64_t)p * q), nb), dim3(FT), 0, st, W + b0 * out * in, in, !wide, jb.M,
                           jb.Q, p, q, bs);
        if (hipGetLastError() != hipSuccess) return LRD_ERR_RUNTIME;
        const int sweeps = run_jacobi(jb, p, q, sg, order, st, nb, bs);
        if (sweeps < 0) return LRD_ERR_RUNTIME;
        max_sweeps = std::max(max_sweeps, sweeps);
        hipLaunchKernelGGL(emit_pair_kernel, dim3((unsigned)r, nb), dim3(FT), 0, st, jb.M, jb.Q, jb.sigma, jb.order, p, q, (int)r, wide,
                           U + b0 * out * r, V + b0 * r * in, bs, out * r, r * in);
        if (hipGetLastError() != hipSuccess || hipStreamSynchronize(st) != hipSuccess) return LRD_ERR_RUNTIME;
        if (sigma_host)
            for (int b = 0; b < nb; ++b)
                for (int j = 0; j < p; ++j) sigma_host[(b0 + b) * p + j] = sg[(size_t)b * p + order[(size_t)b * p + j]];
    }
    if (sweeps_host) *sweeps_host = max_sweeps;
    return LRD_OK;
}

size_t lrd_tucker2_factors_workspace_bytes(int64_t S, int64_t C, int32_t k)
{
    if (S < 1 || C < 1 || k < 1 || k > 31 || S >= (int64_t(1) << 16) || C >= (int64_t(1) << 16)) return 0;
    const int64_t kk = (int64_t)k * k;
    const int64_t pc = std::min(C, S * kk), qc = std::max(C, S * kk);
    const int64_t ps = std::min(S, C * kk), qs = std::max(S, C * kk);
    // one Jacobi problem at a time, the two bases, and the half-contracted weight
    return std::max(jacobi_bytes(pc, qc), jacobi_bytes(ps, qs)) + round256((size_t)C * C * 8) + round256((size_t)S * S * 8) +
           round256((size_t)S * kk * C * 8);
}

lrd_status lrd_tucker2_factors(const float* W, int64_t S, int64_t C, int32_t k, int64_t r1, int64_t r2, float* P1, float* G,
                               float* P2, int32_t* sweeps_host, void* ws, size_t ws_bytes, void* hip_stream)
{
    if (!W || !P1 || !G || !P2 || S < 1 || C < 1 || k < 1 || k > 31) return LRD_ERR_INVALID_ARG;
    if (S >= (int64_t(1) << 16) || C >= (int64_t(1) << 16)) return LRD_ERR_INVALID_ARG;
    const int64_t kk = (int64_t)k * k;
    if (r1 < 1 || r2 < 1 || r1 > std::min(C, S * kk) || r2 > std::min(S, C * kk)) return LRD_ERR_INVALID_ARG;
    if (!aligned16(W) || !aligned16(P1) || !aligned16(G) || !aligned16(P2) || !aligned16(ws)) return LRD_ERR_ALIGNMENT;
    if (!ws || ws_bytes < lrd_tucker2_factors_workspace_bytes(S, C, k)) return LRD_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    char* base = (char*)ws;
    const int64_t pc = std::min(C, S * kk), qc = std::max(C, S * kk);
    const int64_t ps = std::min(S, C * kk), qs = std::max(S, C * kk);
    char* at = base + std::max(jacobi_bytes(pc, qc), jacobi_bytes(ps, qs));
    double* B1 = (double*)at;  at += round256((size_t)C * C * 8);     // [r1 x C] rows = basis vectors of the C mode
    double* B2 = (double*)at;  at += round256((size_t)S * S * 8);     // [r2 x S]
    double* tmp = (double*)at;
    std::vector<double> sg;
    std::vector<int> order;
    int total_sweeps = 0;

    {   // C mode: unfolding [C x S*kk]
        char* j0 = base;
        JacobiBuffers jb = carve_jacobi(j0, pc, qc);
        const bool tall = C > S * kk;             // then M is the transposed unfolding
        hipLaunchKernelGGL(unfold_c_kernel, dim3(blocks_for(S * kk * C)), dim3(FT), 0, st, W, (int)S, (int)kk, (int)C, tall, jb.M,
                           jb.Q, (int)pc);
        if (hipGetLastError() != hipSuccess) return LRD_ERR_RUNTIME;
        int sw = run_jacobi(jb, (int)pc, (int)qc, sg, order, st);
        if (sw < 0) return LRD_ERR_RUNTIME;
        total_sweeps += sw;
        hipLaunchKernelGGL(emit_basis_kernel, dim3((unsigned)r1), dim3(FT), 0, st, jb.M, jb.Q, jb.sigma, jb.order, (int)pc, (int)qc,
                           !tall, B1);
        if (hipGetLastError() != hipSuccess || hipStreamSynchronize(st) != hipSuccess) return LRD_ERR_RUNTIME;
    }
    {   // S mode: unfolding [S x kk*C] is W itself
        char* j0 = base;
        JacobiBuffers jb = carve_jacobi(j0, ps, qs);
        const bool tall = S > C * kk;
        hipLaunchKernelGGL(load_matrix_kernel, dim3(blocks_for(S * kk * C)), dim3(FT), 0, st, W, kk * C, tall, jb.M, jb.Q, (int)ps,
                           (int)qs, BatchStride{});
        if (hipGetLastError() != hipSuccess) return LRD_ERR_RUNTIME;
        int sw = run_jacobi(jb, (int)ps, (int)qs, sg, order, st);
        if (sw < 0) return LRD_ERR_RUNTIME;
        total_sweeps += sw;
        hipLaunchKernelGGL(emit_basis_kernel, dim3((unsigned)r2), dim3(FT), 0, st, jb.M, jb.Q, jb.sigma, jb.order, (int)ps, (int)qs,
                           !tall, B2);
        if (hipGetLastError() != hipSuccess || hipStreamSynchronize(st) != hipSuccess) return LRD_ERR_RUNTIME;
    }
    hipLaunchKernelGGL(core_step1_kernel, dim3(blocks_for(S * kk * r1)), dim3(FT), 0, st, W, B1, S * kk, (int)C, (int)r1, tmp);
    hipLaunchKernelGGL(core_step2_kernel, dim3(blocks_for(r2 * kk * r1)), dim3(FT), 0, st, tmp, B1, B2, (int)S, (int)kk, (int)C, (int)r1,
                       (int)r2, G, P1, P2);
    if (hipGetLastError() != hipSuccess || hipStreamSynchronize(st) != hipSuccess) return LRD_ERR_RUNTIME;
    if (sweeps_host) *sweeps_host = total_sweeps;
    return LRD_OK;
}

}  // extern "C"
