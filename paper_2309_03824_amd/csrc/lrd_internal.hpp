// Internal (C++) interface between the C-ABI entry points and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "lrd_device.hpp"

namespace lrd {

enum Gather : int {
    GATHER_NONE = 0,
    GATHER_CONV_FWD = 1,    // A rows are output pixels, K runs over (u,v,i) taps of an NHWC input
    GATHER_CONV_DGRAD = 2,  // A rows are input pixels, K runs over (u,v,o); B is W[o,u,v,i] read as (i | u,v,o)
    GATHER_CONV_WGRAD = 3   // B rows are taps (u,v,i), K runs over output pixels
};

// An SGD step (see sgd_step) to be applied to a weight where its gradient is finished.  An engine
// that sums split-K partials applies it in that sum and never stores the gradient; otherwise
// run_matop runs it as a kernel of its own on the stored gradient.  Either way `done` is set.
struct SgdFuse {
    float* w = nullptr;        // fp32 master weights, same shape as the gradient (dense)
    float* m = nullptr;        // momentum buffer
    void* copy = nullptr;      // compute copy of the weights to refresh (optional)
    bool copy_bf16 = false;
    float lr = 0.f, mu = 0.f, wd = 0.f;
    mutable bool done = false;
};

// One product  C[M x N] = A[M x K] . B[N x K]^T (+ bias[n]),  fp32 accumulation.
// A(m,k) = A[m*a_sm + k*a_sk], B(n,k) = B[n*b_sn + k*b_sk] (element strides) unless a gather mode
// replaces the addressing of one operand by a convolution's tap geometry.
struct MatOp {
    const void* A = nullptr;
    int64_t a_sm = 0, a_sk = 0;
    const void* B = nullptr;
    int64_t b_sn = 0, b_sk = 0;
    void* C = nullptr;
    int64_t ldc = 0;
    const float* bias = nullptr;
    int64_t M = 0, N = 0, K = 0;
    bool in_bf16 = false;   // operands are bf16 (else fp32)
    bool out_f32 = true;    // C is fp32 (else the operand dtype)
    int gather = GATHER_NONE;
    ConvShape cs{};
    // Split-K: when splits > 1, slice z of K writes partial[z][M][N] (fp32) and a second kernel
    // sums the slices in a fixed order into C, so results do not depend on scheduling.
    int splits = 1;
    float* partial = nullptr;
    int role = 0;           // which product of a layer pass this is (for the event probe)
    // Optional GELU epilogue (bf16 results on the aligned MFMA path only; see epilogue_fusable):
    //   EPI_ACT_STORE: aux[m][n] = gelu(C[m][n]) is written next to C (C keeps the pre-activation);
    //   EPI_ACT_GRAD : C[m][n] is multiplied by gelu'(aux[m][n]) (aux = pre-activation, read).
    int epilogue = 0;
    void* aux = nullptr;
    int64_t ldaux = 0;
    // Optional device scratch an engine may use (the direct convolution's weight gradient keeps
    // its per-workgroup partial sums there, a stride-1 data gradient its flipped weights).
    void* scratch = nullptr;
    size_t scratch_bytes = 0;
    // Optional optimizer step on the finished fp32 result (a dense weight gradient, ldc == N).
    const SgdFuse* sgd = nullptr;
    // A batch of products of one shape (the layers of a group): product z reads A + z * a_bs,
    // B + z * b_bs, bias + z * bias_bs and writes C + z * c_bs, aux + z * aux_bs (element strides).
    int batch = 1;
    int64_t a_bs = 0, b_bs = 0, c_bs = 0, aux_bs = 0, bias_bs = 0;
};
enum { EPI_NONE = 0, EPI_ACT_STORE = 1, EPI_ACT_GRAD = 2 };

// Engines.  Each returns hipSuccess or the launch error.
hipError_t generic_matop(const MatOp& op, hipStream_t st);          // any MatOp, plain FMA tiles
bool mfma_matop_supported(const MatOp& op);                         // bf16 MFMA engine covers it?
hipError_t mfma_matop(const MatOp& op, hipStream_t st);
bool mfma_gemm2_supported(const MatOp& op);                        // aligned fast path covers it?
hipError_t mfma_gemm2(const MatOp& op, hipStream_t st);
bool conv_direct_supported(const MatOp& op);                       // 3 x 3 stride-1 convolution with 32 / 64 channels?
hipError_t conv_direct(const MatOp& op, hipStream_t st);
size_t conv_direct_wgrad_bytes(const ConvShape& cs, bool bf16);    // scratch its weight gradient wants (0: not covered)
hipError_t run_matop(const MatOp& op, hipStream_t st);              // picks an engine
hipError_t apply_epilogue(const MatOp& op, hipStream_t st);        // unfused form of MatOp::epilogue

// Workspace floats a MatOp of this shape needs for split-K (0 if it will not be split).
int choose_splits(int64_t M, int64_t N, int64_t K, bool in_bf16);
// Split-K count for a product whose result is a narrow bf16 activation (1 = not split).
int choose_splits_act(int64_t M, int64_t N, int64_t K, bool in_bf16);
int choose_splits_batched(int64_t M, int64_t N, int64_t K, int64_t batch);

// Fused pair  C2[M x N2] = (A[M x K1] . B1[R x K1]^T) . B2[N2 x R]^T : the rank-R intermediate
// stays on chip; optionally it is also stored (mid_save, [M x R], operand dtype).
struct ChainOp {
    const void* A = nullptr;  int64_t lda = 0;            // [M x K1], K-contiguous
    const void* B1 = nullptr; int64_t b1_sn = 0, b1_sk = 0;  // B1(j,k)
    const void* B2 = nullptr; int64_t b2_sn = 0, b2_sk = 0;  // B2(n,j)
    void* C = nullptr; int64_t ldc = 0;
    void* mid_save = nullptr; int64_t ldmid = 0;
    const float* bias = nullptr;
    int64_t M = 0, K1 = 0, R = 0, N2 = 0;
    int role = 0;
};
bool mfma_chain_supported(const ChainOp& op);
hipError_t mfma_chain(const ChainOp& op, hipStream_t st);

// Event log of the products (lrd_profile_log_start / _stop).  log_begin hands out the events of the
// next record, or returns a negative index when logging is off or the events have run out; log_end
// fills the record.  note_kernel is called by a launcher with the name of the kernel it launched.
int log_begin(hipEvent_t* start, hipEvent_t* stop);
void log_end(int index, int role, int gather, int epilogue, int splits, int64_t M, int64_t N, int64_t K, int64_t batch = 1);
void note_kernel(const char* name);

// Elementwise / reductions.
hipError_t gelu_fwd(const void* Z, void* A, int64_t n, bool bf16, hipStream_t st);
hipError_t gelu_bwd(const void* dA, const void* Z, void* dZ, int64_t n, bool bf16, hipStream_t st);
hipError_t column_sums(const void* dY, float* out, int64_t T, int64_t n, bool bf16, hipStream_t st);
// Zero-padding / cropping copy of a row-major matrix (elem_bytes 2 or 4).
hipError_t copy2d(const void* src, int64_t ld_src, int64_t rows_src, int64_t cols_src, void* dst, int64_t ld_dst,
                  int64_t rows_dst, int64_t cols_dst, int elem_bytes, hipStream_t st);
hipError_t sgd_step(float* w, float* m, const float* g, void* copy, bool copy_bf16, int64_t n, float lr, float mu, float wd,
                    hipStream_t st);
// wt [I][k][k][O] (bf16) = w [O][k][k][I] with the taps reversed: see conv_dgrad_as_fwd.
hipError_t flip_conv_weights(const void* w, void* wt, int O, int I, int k, hipStream_t st);
// Scratch bytes with which run_matop evaluates a stride-1 bf16 data gradient as a forward convolution
// of dY with flipped weights (k-contiguous weights instead of transposing reads); 0 when it would not.
size_t conv_dgrad_flip_bytes(const ConvShape& cs, bool bf16);
// C = sum over split-K slices of partial[z][M][N], ascending z; C is fp32 or (c_bf16) bf16.
// With `sgd` (fp32 results only) the sum is used for that step instead of being stored, when the
// layout allows (then sgd->done is set).
hipError_t reduce_partials(const float* partial, void* C, bool c_bf16, int64_t ldc, int64_t M, int64_t N,
                           int splits, hipStream_t st, const SgdFuse* sgd = nullptr);

}  // namespace lrd
