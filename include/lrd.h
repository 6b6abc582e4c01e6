/*
 * lrd.h -- C ABI of the MI355X (gfx950) library for low-rank-decomposed layers.
 *
 * Method: Hajimolahoseini, Ahmed, Liu, "Training Acceleration of Low-Rank Decomposed Networks
 * using Sequential Freezing and Rank Quantization".  The library evaluates the forward and
 * backward pass of
 *   - an SVD-decomposed fully connected / 1x1 layer: one layer becomes two consecutive layers
 *     through a rank-r bottleneck (Section 2, eq. 1-2, Fig. 1), and
 *   - a Tucker-2-decomposed k x k convolution: 1x1 -> k x k core -> 1x1 (Section 2, eq. 4),
 * with the paper's two accelerations built in: rank quantization (Section 2.1) and sequential
 * freezing (Section 2.2, Algorithm 2), where a frozen factor's weight-gradient product is skipped.
 *
 * Orientation.  The paper writes W in R^{C x S} (C inputs, S outputs) and W' = U' Sigma' V'^T
 * (eq. 2), so its U' is the input-side factor.  This ABI uses the framework orientation
 * W[out x in] = (paper W)^T ~= U.V:
 *     V [r x in]   applied first  = the paper's decomposed layer L_r(0)
 *     U [out x r]  applied second = the paper's decomposed layer L_r(1)
 *     H = X.V^T [T x r],  Y = H.U^T [T x out].
 * Tucker-2: P1 [r1 x C] = L_r(0), G [r2 x k x k x r1] = L_r(1) (core), P2 [S x r2] = L_r(2).
 * The one-time factorization that produces the factors (eq. 1, 2, 4) is lrd_svd_factors /
 * lrd_tucker2_factors below.
 *
 * Conventions common to every device entry point
 *   - All matrix arguments are DEVICE pointers to dense row-major arrays whose leading dimension
 *     equals their logical width; convolution activations are NHWC, conv weights [O][k][k][I].
 *   - dtype LRD_BF16: activations and factors are bfloat16, products accumulate in fp32,
 *     activation outputs (Y, dX, H_save, ...) are bfloat16, weight gradients are fp32.
 *     dtype LRD_F32: everything is fp32.
 *   - The caller owns every buffer, including the workspace `ws` (size from the matching
 *     *_workspace_bytes query; may be NULL when that query returns 0).  The library keeps no
 *     device memory and the calls declared here keep no mutable state between calls (the
 *     measurement aids of lrd_measure.h, a separate header, are the exception and say so).
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = default stream).
 *     No call synchronises or allocates.
 *   - Arguments are validated on the host before anything is launched; on a non-OK status
 *     nothing has been written.  LRD_ERR_INVALID_ARG: non-positive sizes, rank larger than the
 *     layer allows, NULL for a required pointer, unknown dtype or mask bits.  LRD_ERR_ALIGNMENT:
 *     a base pointer that is not 16-byte aligned.  LRD_ERR_WORKSPACE: ws_bytes too small.
 *     LRD_ERR_RUNTIME: the HIP runtime refused a launch.
 *   - Any rank 1 <= r <= min(in,out) is legal.  Ranks that are multiples of 8/16/32 select
 *     faster code (vector loads, whole MFMA tiles); results never depend on the code path
 *     beyond fp32 summation order.
 *   - Freeze mask: bit i set <=> L_r(i) is frozen.  A frozen factor's gradient buffer is neither
 *     read nor written (it may be NULL); the gradient with respect to the layer input still
 *     flows through the frozen factor.  Gradients of trainable factors are overwritten.
 */
#ifndef LRD_H
#define LRD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LRD_OK = 0,
    LRD_ERR_INVALID_ARG = 1,
    LRD_ERR_UNSUPPORTED = 2,
    LRD_ERR_ALIGNMENT = 3,
    LRD_ERR_WORKSPACE = 4,
    LRD_ERR_RUNTIME = 5
} lrd_status;

typedef enum { LRD_F32 = 0, LRD_BF16 = 1 } lrd_dtype;

enum { LRD_KIND_SVD = 0, LRD_KIND_TUCKER = 1 };
enum { LRD_FREEZE_L0 = 1u, LRD_FREEZE_L1 = 2u, LRD_FREEZE_L2 = 4u };
enum { LRD_ROUND_NEAREST = 0, LRD_ROUND_DOWN = 1, LRD_ROUND_UP = 2 };

/* Human-readable name of a status code (static string, never NULL). */
const char* lrd_status_string(lrd_status s);

/* ------------------------------------------------------------------------------------------
 * Host-only integer rules (pure functions, no device involved)
 * ---------------------------------------------------------------------------------------- */

/*
 * Rank quantization, Section 2.1: a rank computed from a compression ratio (e.g. 257 or 309) is
 * moved to a nearby multiple of `multiple` on which the matrix units run whole tiles (the
 * paper's example: 257 -> 256).  mode LRD_ROUND_NEAREST picks the closest multiple, the larger
 * one on a tie; LRD_ROUND_DOWN the next multiple <= r (the direction Algorithm 1 searches in);
 * LRD_ROUND_UP the next multiple >= r.  The result is confined to the multiples that lie in
 * [max(r_min,1), r_max]; if there is none, r is returned unchanged.
 * Returns the quantized rank, or -LRD_ERR_INVALID_ARG if r < 1, multiple < 1, r_min > r_max or
 * mode is unknown.
 */
int32_t lrd_quantize_rank(int32_t r, int32_t multiple, int32_t mode, int32_t r_min, int32_t r_max);

/*
 * Sequential freezing, Algorithm 2: the freeze mask of a decomposed layer at epoch `epoch`
 * (0-based).  Even epoch: L_r(0) (and L_r(2) for Tucker) frozen, L_r(1) trains; odd epoch: the
 * complement.  kind is LRD_KIND_SVD or LRD_KIND_TUCKER (any other value is read as SVD).
 * Regular (non-sequential) freezing is the mask of epoch 0 kept for the whole run.
 */
uint32_t lrd_freeze_mask(int32_t kind, int64_t epoch);

/*
 * Tucker-2 ranks for compression ratio alpha, eq. 6 (r2 = beta * r1); called with alpha + 1 it
 * is the lower bound R_min of eq. 7.  Both ranks are rounded down (the paper's worked example,
 * [512,512,3,3] at 2x -> 309) and confined to [1,C] and [1,S].
 */
lrd_status lrd_tucker_rank(int64_t C, int64_t S, int32_t k, double alpha, double beta,
                           int32_t* r1, int32_t* r2);

/*
 * Rank of an SVD pair for compression ratio alpha: floor(in*out / (alpha*(in+out))), confined
 * to [1, min(in,out)] (same parameter-count argument as eq. 6).  Negative on bad arguments.
 */
int32_t lrd_svd_rank(int64_t in, int64_t out, double alpha);

/*
 * Rank search of Algorithm 1 (Section 2.1, Rank Optimization) from measured step times.
 *   times[i]  host array, step time of the layer decomposed at rank r_min + i, i = 0 .. r_max - r_min
 *             (any unit; the caller measures them, e.g. forward + backward through this library);
 *   t_dense   step time of the original layer in the same unit;
 *   noise     differences t(r) - t(r-1) at or below this value are not drops (>= 0).
 * The printed listing cannot run as it stands (it needs t(r-1) before measuring it and indexes the
 * 257 -> 256 drop at 257), so the search follows the surrounding text: with d(r) = t(r) - t(r-1),
 *   LRD_SELECT_FIRST_PEAK  going down from r_max, the first r with d(r) > noise that is not below
 *                          its neighbours d(r+1), d(r-1)  (the text's "first peak");
 *   LRD_SELECT_ARGMAX      the r with the largest d(r) > noise in the range, ties to the largest r
 *                          (the listing's arg max);
 * *r_opt = r - 1, the rank just below that drop, or r_max when there is none;
 * *keep_decomposed = 1 iff t(*r_opt) < t_dense (otherwise the original layer is the faster one).
 * mode is one of the two selections, optionally OR-ed with LRD_SELECT_REQUIRE_FASTER.  That flag is
 * an extension the paper does not contain (a reading of the caption's "more efficient
 * computations"): a pick whose time is not below t(r_max) is dropped and *r_opt = r_max, so that an
 * estimated rank that is already aligned stays.  Without the flag the result is the literal one.
 * Pure host function.  LRD_ERR_INVALID_ARG for NULL pointers, an empty range, r_min < 1, negative
 * noise, non-finite times or unknown mode bits.
 */
enum { LRD_SELECT_FIRST_PEAK = 0, LRD_SELECT_ARGMAX = 1, LRD_SELECT_REQUIRE_FASTER = 4 };
lrd_status lrd_select_rank(const double* times, int32_t r_min, int32_t r_max, double t_dense, double noise,
                           int32_t mode, int32_t* r_opt, int32_t* keep_decomposed);

/* ------------------------------------------------------------------------------------------
 * SVD-decomposed linear layer (Section 2, Fig. 1; freezing: Section 2.2)
 * ---------------------------------------------------------------------------------------- */

/* Bytes of workspace lrd_linear_fwd / lrd_linear_bwd need for these sizes (upper bound over
 * every nullable-argument combination).  0 on bad arguments. */
size_t lrd_linear_workspace_bytes(int64_t T, int64_t in, int64_t out, int64_t r, lrd_dtype dt,
                                  uint32_t freeze_mask);

/*
 * Forward: H = X.V^T, Y = H.U^T (+ bias).
 *   X [T x in], V [r x in], U [out x r], bias [out] fp32 or NULL, Y [T x out] (written),
 *   H_save [T x r] in the activation dtype or NULL: when given it receives H for the backward
 *   pass (needed there only if U is trainable).
 */
lrd_status lrd_linear_fwd(const void* X, const void* V, const void* U, const float* bias, void* Y,
                          void* H_save, int64_t T, int64_t in, int64_t out, int64_t r,
                          lrd_dtype dt, void* ws, size_t ws_bytes, void* hip_stream);

/*
 * Backward: dH = dY.U, dX = dH.V, dU = dY^T.H unless bit1 of freeze_mask, dV = dH^T.X unless
 * bit0.
 *   dY [T x out]; X [T x in] (required if V is trainable or H is NULL); H [T x r] as saved by
 *   the forward (NULL: recomputed from X into the workspace when U is trainable);
 *   dX [T x in] or NULL (a first layer needs none); dV [r x in] fp32, dU [out x r] fp32,
 *   dbias [out] fp32 or NULL.
 */
lrd_status lrd_linear_bwd(const void* dY, const void* X, const void* H, const void* V,
                          const void* U, void* dX, float* dV, float* dU, float* dbias,
                          uint32_t freeze_mask, int64_t T, int64_t in, int64_t out, int64_t r,
                          lrd_dtype dt, void* ws, size_t ws_bytes, void* hip_stream);

/*
 * lrd_linear_bwd for callers that cannot allocate or hand over device memory: code running under
 * HIP graph capture, tight serving / training loops, harnesses that forbid hipMalloc.  Same
 * arguments and results as lrd_linear_bwd (bit-identical: the same kernels run), but the scratch
 * the pass needs (dH, a recomputed H, split-K partial sums) lives in a fixed device array inside
 * the library instead of a caller workspace.
 *   - The array holds LRD_STATIC_SCRATCH_BYTES (64 MiB) on every GPU the library is used on, from
 *     the first call on that GPU until the process ends.
 *   - A shape whose lrd_linear_workspace_bytes exceeds that size is rejected with
 *     LRD_ERR_WORKSPACE before anything is launched (lrd_linear_bwd_static_fits tells in advance).
 *   - The call allocates nothing and frees nothing; the first call on a device looks up the
 *     array's address (no allocation either).
 *   - All calls on one GPU share the array and it keeps the previous call's contents; every region
 *     a pass reads is written by that pass first, so nothing needs clearing.  Two such calls that
 *     overlap in time on the same GPU (different streams or threads) race; order them.
 */
#define LRD_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
int32_t lrd_linear_bwd_static_fits(int64_t T, int64_t in, int64_t out, int64_t r, lrd_dtype dt, uint32_t freeze_mask);
lrd_status lrd_linear_bwd_static(const void* dY, const void* X, const void* H, const void* V,
                                 const void* U, void* dX, float* dV, float* dU, float* dbias,
                                 uint32_t freeze_mask, int64_t T, int64_t in, int64_t out, int64_t r,
                                 lrd_dtype dt, void* hip_stream);

/*
 * Optimizer of the paper's experiments (Section 3: SGD, momentum 0.9, weight decay 1e-4), in the
 * usual form g' = g + weight_decay * w;  m <- momentum * m + g';  w <- w - lr * m  (a momentum buffer
 * that starts at zero gives the customary first step m = g').
 *   w_master, momentum_buf  device fp32 [n], updated in place;  grad device fp32 [n];
 *   w_copy  device, nullable: the layer's compute copy of the weights in copy_dt (bf16 or fp32),
 *           rewritten from the new master value (may be w_master itself when copy_dt is fp32).
 */
typedef struct lrd_sgd { float lr, momentum, weight_decay; } lrd_sgd;
lrd_status lrd_sgd_step(float* w_master, float* momentum_buf, const float* grad, void* w_copy, lrd_dtype copy_dt,
                        int64_t n, const lrd_sgd* opt, void* hip_stream);

/*
 * lrd_linear_bwd_act followed by that step for every factor freeze_mask leaves trainable, in one
 * call: a frozen factor costs neither a gradient nor an update (Section 2.2 carried through the
 * optimizer), and a trainable factor's step is applied where its gradient is finished: inside the
 * fixed-order sum over the K-slices of the weight-gradient product when that product is sliced (the
 * gradient is then never stored), else on the gradient in the workspace right after the product.  V and U are the compute copies the layer
 * multiplies with (dtype dt) and are rewritten; V_master / U_master and V_momentum / U_momentum are
 * fp32 [r x in] / [out x r], required for the trainable factors, ignored for frozen ones.  The data
 * gradient dX uses the factors as they were before the update.  Other arguments as lrd_linear_bwd_act;
 * workspace from lrd_linear_sgd_workspace_bytes.
 */
size_t lrd_linear_sgd_workspace_bytes(int64_t T, int64_t in, int64_t out, int64_t r, lrd_dtype dt,
                                      uint32_t freeze_mask);
lrd_status lrd_linear_bwd_sgd(const void* dY, const void* X, const void* H, void* V, void* U, void* dX,
                              float* V_master, float* U_master, float* V_momentum, float* U_momentum,
                              float* dbias, uint32_t freeze_mask, const void* Z_in, int32_t act,
                              const lrd_sgd* opt, int64_t T, int64_t in, int64_t out, int64_t r, lrd_dtype dt,
                              void* ws, size_t ws_bytes, void* hip_stream);

/*
 * Several decomposed layers of one shape on the same input (the query, key and value projections of
 * an attention block, each decomposed as in Section 2).  Their first factors are stacked,
 * V_cat [groups*r x in] (group g in rows g*r .. g*r + r - 1), so that the products with X are one
 * product of width groups*r and the data gradients through them one product of depth groups*r; the
 * rest is per group: U [groups][out x r], bias [groups][out] fp32 or NULL, Y and dY [groups][T x out],
 * dU [groups][out x r] fp32, dV_cat [groups*r x in] fp32, dbias [groups][out] fp32 or NULL;
 * H_save / H [T x groups*r] holds the groups' intermediates side by side; dX [T x in] is the sum over
 * the groups.  freeze_mask applies to every group.  Results equal `groups` calls of lrd_linear_fwd /
 * lrd_linear_bwd with the gradients dX added, up to summation order.  Arguments otherwise as there.
 */
size_t lrd_linear_group_workspace_bytes(int64_t T, int64_t in, int64_t out, int64_t r, int32_t groups,
                                        lrd_dtype dt, uint32_t freeze_mask);
lrd_status lrd_linear_group_fwd(const void* X, const void* V_cat, const void* U, const float* bias, void* Y,
                                void* H_save, int64_t T, int64_t in, int64_t out, int64_t r, int32_t groups,
                                lrd_dtype dt, void* ws, size_t ws_bytes, void* hip_stream);
lrd_status lrd_linear_group_bwd(const void* dY, const void* X, const void* H, const void* V_cat, const void* U,
                                void* dX, float* dV_cat, float* dU, float* dbias, uint32_t freeze_mask,
                                int64_t T, int64_t in, int64_t out, int64_t r, int32_t groups, lrd_dtype dt,
                                void* ws, size_t ws_bytes, void* hip_stream);

/*
 * The backward pass of a stack of equal layers in two parts, for callers that keep every layer's
 * gradient input and saved activations until the stack's backward has finished (sizes here make that
 * cheap).  The weight gradients of Section 2 (dU = dY^T.H, dV = dH^T.X) are small products with a
 * long reduction over the tokens: one layer's does not fill the device, the same product for all the
 * layers of one shape, as one launch, does, and needs no sliced reduction.
 *   lrd_linear_bwd_data / lrd_linear_group_bwd_data: only the data gradient, dX = (dY.U).V (times
 *     act'(Z_in) as in lrd_linear_bwd_act).  dH_save [T x r] ([T x groups*r] for a group), dtype dt,
 *     caller's, required, receives dH = dY.U, which the first factor's gradient needs later; dX may
 *     be NULL (first layer of a network: only dH is formed).  Workspace from lrd_linear_workspace_bytes /
 *     lrd_linear_group_workspace_bytes.  Results are bit-identical to lrd_linear_bwd(_act) /
 *     lrd_linear_group_bwd with both factors frozen (bf16 ranks that are not multiples of 8 aside:
 *     only the one-call form pads them).
 *   lrd_linear_wgrad_batched: for l = 0 .. layers-1, dU[l] = dY[l]^T.H[l] (unless LRD_FREEZE_L1) and
 *     dV[l] = dH[l]^T.X[l] (unless LRD_FREEZE_L0).  Layer l's operand starts l * stride elements
 *     after the base pointer (strides multiples of 8 elements): dY [T x out] rows dense; H [T x r]
 *     with row pitch ldh; dH [T x r] with row pitch lddh; X [T x in] rows dense.  The row pitches
 *     let a group's side-by-side intermediates be addressed in place: one call per group member for
 *     dU (base pointer g*r elements in, ldh = groups*r), and one call with r := groups*r for the
 *     stacked first factors.  dU [layers][out x r] and dV [layers][r x in] are fp32, dense,
 *     overwritten.  Operands of a frozen factor may be NULL.  Results equal `layers` calls of
 *     lrd_linear_bwd up to the order of the sum over tokens (both are fixed, so each is
 *     reproducible).
 */
lrd_status lrd_linear_bwd_data(const void* dY, const void* V, const void* U, void* dX, void* dH_save,
                               const void* Z_in, int32_t act, int64_t T, int64_t in, int64_t out, int64_t r,
                               lrd_dtype dt, void* ws, size_t ws_bytes, void* hip_stream);
lrd_status lrd_linear_group_bwd_data(const void* dY, const void* V_cat, const void* U, void* dX, void* dH_save,
                                     int64_t T, int64_t in, int64_t out, int64_t r, int32_t groups, lrd_dtype dt,
                                     void* ws, size_t ws_bytes, void* hip_stream);
size_t lrd_linear_wgrad_batched_workspace_bytes(int64_t layers, int64_t T, int64_t in, int64_t out, int64_t r,
                                                lrd_dtype dt, uint32_t freeze_mask);
lrd_status lrd_linear_wgrad_batched(const void* dY, int64_t dy_stride, const void* H, int64_t ldh, int64_t h_stride,
                                    const void* dH, int64_t lddh, int64_t dh_stride, const void* X, int64_t x_stride,
                                    float* dV, float* dU, uint32_t freeze_mask, int64_t layers, int64_t T, int64_t in,
                                    int64_t out, int64_t r, lrd_dtype dt, void* ws, size_t ws_bytes, void* hip_stream);

/*
 * The same two calls with the activation between stacked layers folded into them (GELU, erf
 * form; not part of the paper's method, it removes two elementwise passes of a layer stack).
 *   lrd_linear_fwd_act: Y receives the pre-activation Z = H.U^T (+ bias), which the backward
 *     needs, and Y_act [T x out] receives act(Z) as rounded to the activation dtype.
 *   lrd_linear_bwd_act: for a layer whose input X is act(Z_in), Z_in [T x in] being the
 *     pre-activation saved by the previous layer's forward: dX receives (dH.V) * act'(Z_in),
 *     i.e. the gradient with respect to Z_in.  Z_in is required iff dX is given.
 * act = LRD_ACT_NONE makes them identical to the plain calls (Y_act / Z_in ignored).  Results are
 * bit-identical to the plain call followed by lrd_gelu_fwd / lrd_gelu_bwd.
 */
enum { LRD_ACT_NONE = 0, LRD_ACT_GELU = 1 };
lrd_status lrd_linear_fwd_act(const void* X, const void* V, const void* U, const float* bias,
                              void* Y, void* Y_act, void* H_save, int32_t act, int64_t T,
                              int64_t in, int64_t out, int64_t r, lrd_dtype dt, void* ws,
                              size_t ws_bytes, void* hip_stream);
lrd_status lrd_linear_bwd_act(const void* dY, const void* X, const void* H, const void* V,
                              const void* U, void* dX, float* dV, float* dU, float* dbias,
                              uint32_t freeze_mask, const void* Z_in, int32_t act, int64_t T,
                              int64_t in, int64_t out, int64_t r, lrd_dtype dt, void* ws,
                              size_t ws_bytes, void* hip_stream);

/*
 * The undecomposed layer Y = X.W^T (+ bias), dX = dY.W, dW = dY^T.X: the "original layer" whose
 * time Algorithm 1 compares a decomposed layer against.  W [out x in]; dX, dW nullable.
 */
size_t lrd_dense_linear_workspace_bytes(int64_t T, int64_t in, int64_t out, lrd_dtype dt);
lrd_status lrd_dense_linear_fwd(const void* X, const void* W, const float* bias, void* Y,
                                int64_t T, int64_t in, int64_t out, lrd_dtype dt, void* ws,
                                size_t ws_bytes, void* hip_stream);
lrd_status lrd_dense_linear_bwd(const void* dY, const void* X, const void* W, void* dX, float* dW,
                                int64_t T, int64_t in, int64_t out, lrd_dtype dt, void* ws,
                                size_t ws_bytes, void* hip_stream);

/* ------------------------------------------------------------------------------------------
 * Tucker-2-decomposed convolution (Section 2, eq. 4: 1x1 -> k x k core -> 1x1)
 * ---------------------------------------------------------------------------------------- */

/* Geometry of one decomposed convolution.  Stride and padding act on the k x k core; the two
 * 1x1 layers have stride 1 and no padding.  Ho = (H + 2*pad - k)/stride + 1, same for Wo. */
typedef struct {
    int64_t N, H, W;   /* batch, input height, input width */
    int64_t C, S;      /* input channels, output channels   */
    int64_t r1, r2;    /* Tucker ranks: C -> r1 -> r2 -> S  */
    int32_t k, stride, pad;
} lrd_conv_geom;

size_t lrd_tucker_conv_workspace_bytes(const lrd_conv_geom* g, lrd_dtype dt, uint32_t freeze_mask);

/*
 * Forward: A = X.P1^T (per pixel), B = conv_kxk(A, G), Y = B.P2^T (per pixel).
 *   X [N,H,W,C], P1 [r1 x C], G [r2,k,k,r1], P2 [S x r2], Y [N,Ho,Wo,S] (written);
 *   A_save [N,H,W,r1] and B_save [N,Ho,Wo,r2] or NULL: the intermediates, kept for the backward.
 */
lrd_status lrd_tucker_conv_fwd(const void* X, const void* P1, const void* G, const void* P2,
                               void* Y, void* A_save, void* B_save, const lrd_conv_geom* g,
                               lrd_dtype dt, void* ws, size_t ws_bytes, void* hip_stream);

/*
 * Backward: dB = dY.P2, dA = conv^T(dB, G), dX = dA.P1; dP1 = dA^T.X unless bit0,
 * dG[o,u,v,i] = sum_pixels dB[..,o] A[shifted ..,i] unless bit1, dP2 = dY^T.B unless bit2.
 *   A, B as saved by the forward (NULL: recomputed into the workspace when needed);
 *   dX nullable; dP1 [r1 x C], dG [r2,k,k,r1], dP2 [S x r2] fp32.
 */
lrd_status lrd_tucker_conv_bwd(const void* dY, const void* X, const void* A, const void* B,
                               const void* P1, const void* G, const void* P2, void* dX,
                               float* dP1, float* dG, float* dP2, uint32_t freeze_mask,
                               const lrd_conv_geom* g, lrd_dtype dt, void* ws, size_t ws_bytes,
                               void* hip_stream);

/*
 * The undecomposed k x k convolution (geometry fields r1, r2 ignored): Y = conv(X, W),
 * dX = conv^T(dY, W), dW = wgrad(dY, X); W [S,k,k,C].  dX, dW nullable.
 */
size_t lrd_dense_conv_workspace_bytes(const lrd_conv_geom* g, lrd_dtype dt);
lrd_status lrd_dense_conv_fwd(const void* X, const void* W, void* Y, const lrd_conv_geom* g,
                              lrd_dtype dt, void* ws, size_t ws_bytes, void* hip_stream);
lrd_status lrd_dense_conv_bwd(const void* dY, const void* X, const void* W, void* dX, float* dW,
                              const lrd_conv_geom* g, lrd_dtype dt, void* ws, size_t ws_bytes,
                              void* hip_stream);

/* ------------------------------------------------------------------------------------------
 * One-time factorization on the device (Section 2: eq. 1, 2 truncated SVD; eq. 4 Tucker-2)
 *
 * Unlike the layer passes these calls SYNCHRONISE the stream (the Jacobi sweeps stop when the host
 * reads that no pair rotated) and compute in fp64; they still allocate nothing.
 * ---------------------------------------------------------------------------------------- */

/* Workspace bytes of lrd_svd_factors for a weight [out x in] (0 on bad sizes). */
size_t lrd_svd_factors_workspace_bytes(int64_t out, int64_t in);

/*
 * Rank-r factor pair of a layer weight (eq. 2) by one-sided Jacobi SVD (eq. 1).
 *   W  device, fp32 [out x in] row-major (read only);
 *   U  device, fp32 [out x r] = (left singular vectors) * sqrt(sigma);
 *   V  device, fp32 [r x in]  = sqrt(sigma) * (right singular vectors)^T, so that U.V is the best
 *      rank-r approximation of W and the singular values are shared evenly between the factors
 *      (the paper leaves the split of Sigma open); components are ordered by descending sigma,
 *      each determined up to a common sign of its U column and V row;
 *   sigma_host   host, nullable: all min(out,in) singular values, descending (eq. 3's error is
 *                the sum of the squares past r);
 *   sweeps_host  host, nullable: Jacobi sweeps used (those on the Gram matrix of a wide weight included).
 * LRD_ERR_INVALID_ARG (NULL, sizes, r > min(out,in)), LRD_ERR_ALIGNMENT (16 bytes),
 * LRD_ERR_WORKSPACE, LRD_ERR_RUNTIME (launch failure or no convergence in 60 sweeps).
 */
lrd_status lrd_svd_factors(const float* W, int64_t out, int64_t in, int64_t r, float* U, float* V,
                           double* sigma_host, int32_t* sweeps_host, void* ws, size_t ws_bytes, void* hip_stream);

/*
 * The same factorization for a batch of weights of one shape (the layers of a stack), W [batch][out x in],
 * U [batch][out x r], V [batch][r x in], all dense and consecutive; sigma_host [batch][min(out,in)] or NULL;
 * *sweeps_host = the largest number of sweeps any part of the batch took.  Every tournament step of the
 * Jacobi iteration (eq. 1) is one launch over all matrices of a group and the convergence test is read
 * once per sweep for the group; groups are sized so that their working set stays in the last-level cache.
 * Each matrix gets the factors lrd_svd_factors would give it (same rotations, same order).
 */
size_t lrd_svd_factors_batched_workspace_bytes(int64_t batch, int64_t out, int64_t in);
lrd_status lrd_svd_factors_batched(const float* W, int64_t batch, int64_t out, int64_t in, int64_t r, float* U, float* V,
                                   double* sigma_host, int32_t* sweeps_host, void* ws, size_t ws_bytes, void* hip_stream);

/* Workspace bytes of lrd_tucker2_factors for a weight [S][k][k][C] (0 on bad sizes). */
size_t lrd_tucker2_factors_workspace_bytes(int64_t S, int64_t C, int32_t k);

/*
 * Tucker-2 factors of a convolution weight (eq. 4) by truncated higher-order SVD on the two channel
 * modes; the spatial modes stay whole.
 *   W   device, fp32 [S][k][k][C] (output channel, kernel row, kernel column, input channel);
 *   P1  device, fp32 [r1 x C]: leading left singular vectors of the C-mode unfolding, as rows;
 *   P2  device, fp32 [S x r2]: those of the S-mode unfolding, as columns;
 *   G   device, fp32 [r2][k][k][r1]: W contracted with P1 over C and with P2 over S,
 * in the layouts lrd_tucker_conv_fwd takes.  Basis vectors are determined up to sign (the core
 * carries the matching signs).  r1 <= min(C, S k^2), r2 <= min(S, C k^2).
 *   sweeps_host  host, nullable: Jacobi sweeps used by the two decompositions together.
 * Status codes as lrd_svd_factors.
 */
lrd_status lrd_tucker2_factors(const float* W, int64_t S, int64_t C, int32_t k, int64_t r1, int64_t r2,
                               float* P1, float* G, float* P2, int32_t* sweeps_host, void* ws, size_t ws_bytes,
                               void* hip_stream);

/* ------------------------------------------------------------------------------------------
 * Glue between stacked layers (not part of the method; used by the layer-stack workloads)
 * ---------------------------------------------------------------------------------------- */

/* GELU in its erf form, A = Z * Phi(Z), and its backward dZ = dA * (Phi(Z) + Z * phi(Z));
 * n elements of the activation dtype. */
lrd_status lrd_gelu_fwd(const void* Z, void* A, int64_t n, lrd_dtype dt, void* hip_stream);
lrd_status lrd_gelu_bwd(const void* dA, const void* Z, void* dZ, int64_t n, lrd_dtype dt,
                        void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* LRD_H */
