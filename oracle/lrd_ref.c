/*
 * lrd_ref.c -- CPU oracle for low-rank-decomposed layers.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 implementation of what the decomposed-layer path computes, written from
 * the paper (Hajimolahoseini, Ahmed, Liu: "Training Acceleration of Low-Rank Decomposed Networks
 * using Sequential Freezing and Rank Quantization").  It exists so that the GPU library can be
 * checked against something that shares no code with it.  Nothing in the product may call it;
 * only tests, the smoke check and the CPU-baseline leg of the benchmark do.
 *
 * Everything is row-major, double precision, straight loops: no blocking, no BLAS, no fusion.
 * OpenMP, when enabled at compile time, only distributes independent output rows over threads.
 *
 * Naming.  The paper writes a layer weight as W in R^{C x S} (C inputs, S outputs; Section 2)
 * and its truncated SVD as U' Sigma' V'^T (eq. 2), so the paper's U' sits on the input side.
 * This file uses the framework-style orientation W[out x in] = (paper W)^T and W ~= U.V with
 *     V [r x in]   applied first   = the paper's decomposed layer L_r(0),
 *     U [out x r]  applied second  = the paper's decomposed layer L_r(1),
 * so V = Sigma'^{1/2} U'^T(paper) and U = V'(paper) Sigma'^{1/2}.
 * For a k x k convolution (eq. 4, Tucker-2): P1 [r1 x C] = L_r(0) (1x1), G [r2,k,k,r1] = L_r(1)
 * (k x k core), P2 [S x r2] = L_r(2) (1x1).  Activations are NHWC, conv weights [O][kh][kw][I].
 *
 * Freeze mask: bit i set <=> L_r(i) frozen (Section 2.2, Algorithm 2).  A frozen factor gets no
 * weight gradient; the gradient with respect to its input still flows through it.
 *
 * Pins (tests/test_oracle_*.py): every function here is pinned against values the paper prints,
 * closed forms, LAPACK, finite differences or brute force.  No function is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define LRD_REF_FREEZE_L0 1u
#define LRD_REF_FREEZE_L1 2u
#define LRD_REF_FREEZE_L2 4u

/* ------------------------------------------------------------------------------------------ */
/* Integer rules                                                                               */
/* ------------------------------------------------------------------------------------------ */

/*
 * Rank quantization (Section 2.1: a rank such as 257 is moved to a nearby hardware-friendly value
 * such as 256).  mode 0: nearest multiple of m, the larger one on a tie; 1: next multiple below
 * or equal; 2: next multiple above or equal.  The result is then confined to the multiples of m
 * that lie in [max(r_min,1), r_max]; when that set is empty r comes back unchanged.
 * Returns -1 on arguments that make no sense.
 */
int32_t lrd_ref_quantize_rank(int32_t r, int32_t m, int32_t mode, int32_t r_min, int32_t r_max)
{
    if (r < 1 || m < 1 || r_min > r_max || mode < 0 || mode > 2) return -1;
    int64_t lo = r_min < 1 ? 1 : r_min;
    int64_t hi = r_max;
    int64_t q;
    if (mode == 0) {
        int64_t below = ((int64_t)r / m) * m;
        int64_t above = below + m;
        q = ((int64_t)r - below < above - (int64_t)r) ? below : above;
        if ((int64_t)r == below) q = below;
    } else if (mode == 1) {
        q = ((int64_t)r / m) * m;
    } else {
        q = (((int64_t)r + m - 1) / m) * m;
    }
    int64_t first = ((lo + m - 1) / m) * m; /* smallest multiple >= lo */
    int64_t last = (hi / m) * m;            /* largest multiple <= hi  */
    if (first > last || last < 1) return r;
    if (q < first) q = first;
    if (q > last) q = last;
    return (int32_t)q;
}

/*
 * Sequential freezing (Algorithm 2).  kind 0 = SVD pair, 1 = Tucker triple.  Even epoch: the
 * outer factor(s) L_r(0) (and L_r(2)) are frozen and L_r(1) trains; odd epoch: the complement.
 */
uint32_t lrd_ref_freeze_mask(int32_t kind, int64_t epoch)
{
    int even = (epoch % 2) == 0;
    if (kind == 1) return even ? (LRD_REF_FREEZE_L0 | LRD_REF_FREEZE_L2) : LRD_REF_FREEZE_L1;
    return even ? LRD_REF_FREEZE_L0 : LRD_REF_FREEZE_L1;
}

/*
 * Tucker-2 ranks for compression ratio alpha (eq. 6; with alpha+1 it is eq. 7).  r2 = beta*r1.
 * The paper's worked example ([512,512,3,3], alpha=2 -> 309) fixes the rounding as floor.
 */
int lrd_ref_tucker_rank(int64_t C, int64_t S, int32_t k, double alpha, double beta, int32_t* r1,
                        int32_t* r2)
{
    if (C < 1 || S < 1 || k < 1 || !(alpha > 0.0) || !(beta > 0.0)) return 1;
    double k2 = (double)k * (double)k;
    double b = ((double)C + beta * (double)S) / (beta * k2);
    double disc = b * b + 4.0 * (double)C * (double)S / (beta * alpha);
    double x = (-b + sqrt(disc)) / 2.0;
    int64_t a = (int64_t)floor(x);
    /* eq. 6 is the positive root of f(r1) = beta k^2 r1^2 + (C + beta S) r1 - C S k^2 / alpha
     * (parameter count of the three layers minus the budget).  When the root is an integer the
     * rounding of sqrt() could land on either side of it, so settle floor() with the sign of f. */
    double budget = (double)C * (double)S * k2 / alpha;
    double lin = (double)C + beta * (double)S;
    double up = (double)(a + 1);
    if (beta * k2 * up * up + lin * up <= budget) a += 1;
    else if (a >= 1 && beta * k2 * (double)a * (double)a + lin * (double)a > budget) a -= 1;
    int64_t c = (int64_t)floor(beta * (double)a);
    if (a < 1) a = 1;
    if (a > C) a = C;
    if (c < 1) c = 1;
    if (c > S) c = S;
    *r1 = (int32_t)a;
    *r2 = (int32_t)c;
    return 0;
}

/*
 * Rank of an SVD pair for compression ratio alpha.  The paper gives no formula for this case;
 * it follows from the same parameter count as eq. 6: r*(in+out) = in*out/alpha, rounded down.
 */
int32_t lrd_ref_svd_rank(int64_t in, int64_t out, double alpha)
{
    if (in < 1 || out < 1 || !(alpha > 0.0)) return -1;
    double x = (double)in * (double)out / (alpha * ((double)in + (double)out));
    int64_t r = (int64_t)floor(x);
    int64_t R = in < out ? in : out;
    if (r < 1) r = 1;
    if (r > R) r = R;
    return (int32_t)r;
}

/*
 * Rank search of Algorithm 1 (Section 2.1, Rank Optimization), given the measured step times.
 * t[i] is the step time of the layer decomposed at rank r_min + i, i = 0 .. r_max - r_min;
 * t_dense the step time of the original layer.  The listing cannot be run as printed (it uses
 * t(r-1) before it is measured, and indexes the 257 -> 256 drop at 257 while the rank it wants
 * is 256), so this follows the text around it:
 *   d(r) = t(r) - t(r-1) for r in (r_min, r_max]  -- the first derivative of step time vs rank;
 *   selection 0 (text): going down from r_max, the first r whose d(r) exceeds `noise` and is not
 *                  smaller than its neighbours d(r+1), d(r-1) ("first peak");
 *   selection 1 (listing): the r with the largest d(r) over the whole range (ties: the largest r),
 *                  accepted only if d(r) exceeds `noise`;
 *   the rank just below that drop is the optimum, R_opt = r - 1; without such an r the estimated
 *   rank stays, R_opt = r_max;
 *   the decomposed layer is used iff t(R_opt) < t_dense.
 * mode = selection, optionally + 4: an extension that is NOT in the paper's listing or text (one
 * reading of the caption's "more efficient computations"): a pick that is not faster than the
 * estimated rank itself is dropped and r_max stays.  Off unless the caller asks for it.
 * Returns 0, or -1 on invalid arguments (empty range, non-finite times, negative noise).
 */
int32_t lrd_ref_select_rank(const double* t, int32_t r_min, int32_t r_max, double t_dense, double noise,
                            int32_t mode, int32_t* r_opt, int32_t* keep_decomposed)
{
    const int32_t require_faster = mode & 4;
    mode &= ~4;
    if (!t || !r_opt || !keep_decomposed || r_min < 1 || r_max < r_min || (mode != 0 && mode != 1)) return -1;
    if (!(noise >= 0.0) || !isfinite(noise) || !isfinite(t_dense)) return -1;
    const int32_t n = r_max - r_min + 1;
    for (int32_t i = 0; i < n; ++i)
        if (!isfinite(t[i])) return -1;
    int32_t found = 0;                      /* the r of the drop, 0 if none */
    if (mode == 0) {
        for (int32_t r = r_max; r > r_min && !found; --r) {
            double d = t[r - r_min] - t[r - 1 - r_min];
            if (!(d > noise)) continue;
            int peak = 1;
            if (r < r_max) {
                double up = t[r + 1 - r_min] - t[r - r_min];
                if (d < up) peak = 0;
            }
            if (r - 1 > r_min) {
                double down = t[r - 1 - r_min] - t[r - 2 - r_min];
                if (d < down) peak = 0;
            }
            if (peak) found = r;
        }
    } else {
        double best = 0.0;
        for (int32_t r = r_max; r > r_min; --r) {
            double d = t[r - r_min] - t[r - 1 - r_min];
            if (d > noise && (!found || d > best)) {
                best = d;
                found = r;
            }
        }
    }
    *r_opt = found ? found - 1 : r_max;
    if (require_faster && !(t[*r_opt - r_min] < t[r_max - r_min])) *r_opt = r_max;
    *keep_decomposed = t[*r_opt - r_min] < t_dense ? 1 : 0;
    return 0;
}

/* ------------------------------------------------------------------------------------------ */
/* SVD-decomposed linear layer (Section 2, Fig. 1: one FC layer -> two consecutive FC layers)  */
/* ------------------------------------------------------------------------------------------ */

/* H[t,j] = sum_i X[t,i] V[j,i];  Y[t,o] = sum_j H[t,j] U[o,j] (+ bias[o]) */
void lrd_ref_linear_fwd(const double* X, const double* V, const double* U, const double* bias,
                        double* H, double* Y, int64_t T, int64_t in, int64_t out, int64_t r)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        for (int64_t j = 0; j < r; ++j) {
            double s = 0.0;
            for (int64_t i = 0; i < in; ++i) s += X[t * in + i] * V[j * in + i];
            H[t * r + j] = s;
        }
        for (int64_t o = 0; o < out; ++o) {
            double s = 0.0;
            for (int64_t j = 0; j < r; ++j) s += H[t * r + j] * U[o * r + j];
            Y[t * out + o] = s + (bias ? bias[o] : 0.0);
        }
    }
}

/*
 * Backward of the pair.  dH and dX are always produced (the gradient flows through frozen
 * factors).  dU[o,j] = sum_t dY[t,o] H[t,j] only when L_r(1) is trainable, dV[j,i] =
 * sum_t dH[t,j] X[t,i] only when L_r(0) is trainable; a frozen factor's buffer is not touched.
 * dbias (optional) = column sums of dY.
 */
void lrd_ref_linear_bwd(const double* dY, const double* X, const double* H, const double* V,
                        const double* U, double* dH, double* dX, double* dV, double* dU,
                        double* dbias, uint32_t mask, int64_t T, int64_t in, int64_t out, int64_t r)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        /* every sum runs over its index in ascending order; the innermost loop walks the
         * contiguous index of the output row so that memory is read in order */
        for (int64_t j = 0; j < r; ++j) dH[t * r + j] = 0.0;
        for (int64_t o = 0; o < out; ++o) {
            double g = dY[t * out + o];
            for (int64_t j = 0; j < r; ++j) dH[t * r + j] += g * U[o * r + j];
        }
        if (dX) {
            for (int64_t i = 0; i < in; ++i) dX[t * in + i] = 0.0;
            for (int64_t j = 0; j < r; ++j) {
                double g = dH[t * r + j];
                for (int64_t i = 0; i < in; ++i) dX[t * in + i] += g * V[j * in + i];
            }
        }
    }
    if (!(mask & LRD_REF_FREEZE_L1) && dU) {
#pragma omp parallel for schedule(static)
        for (int64_t o = 0; o < out; ++o) {
            for (int64_t j = 0; j < r; ++j) dU[o * r + j] = 0.0;
            for (int64_t t = 0; t < T; ++t) {
                double g = dY[t * out + o];
                for (int64_t j = 0; j < r; ++j) dU[o * r + j] += g * H[t * r + j];
            }
        }
    }
    if (!(mask & LRD_REF_FREEZE_L0) && dV) {
#pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < r; ++j) {
            for (int64_t i = 0; i < in; ++i) dV[j * in + i] = 0.0;
            for (int64_t t = 0; t < T; ++t) {
                double g = dH[t * r + j];
                for (int64_t i = 0; i < in; ++i) dV[j * in + i] += g * X[t * in + i];
            }
        }
    }
    if (dbias) {
        for (int64_t o = 0; o < out; ++o) {
            double s = 0.0;
            for (int64_t t = 0; t < T; ++t) s += dY[t * out + o];
            dbias[o] = s;
        }
    }
}

/* The undecomposed layer, for the "versus the original layer" comparison (Algorithm 1). */
void lrd_ref_dense_linear_fwd(const double* X, const double* W, const double* bias, double* Y,
                              int64_t T, int64_t in, int64_t out)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t)
        for (int64_t o = 0; o < out; ++o) {
            double s = 0.0;
            for (int64_t i = 0; i < in; ++i) s += X[t * in + i] * W[o * in + i];
            Y[t * out + o] = s + (bias ? bias[o] : 0.0);
        }
}

void lrd_ref_dense_linear_bwd(const double* dY, const double* X, const double* W, double* dX,
                              double* dW, int64_t T, int64_t in, int64_t out)
{
    if (dX) {
#pragma omp parallel for schedule(static)
        for (int64_t t = 0; t < T; ++t) {
            for (int64_t i = 0; i < in; ++i) dX[t * in + i] = 0.0;
            for (int64_t o = 0; o < out; ++o) {
                double g = dY[t * out + o];
                for (int64_t i = 0; i < in; ++i) dX[t * in + i] += g * W[o * in + i];
            }
        }
    }
    if (dW) {
#pragma omp parallel for schedule(static)
        for (int64_t o = 0; o < out; ++o) {
            for (int64_t i = 0; i < in; ++i) dW[o * in + i] = 0.0;
            for (int64_t t = 0; t < T; ++t) {
                double g = dY[t * out + o];
                for (int64_t i = 0; i < in; ++i) dW[o * in + i] += g * X[t * in + i];
            }
        }
    }
}

/* GELU in its erf form and its derivative Phi(x) + x phi(x): glue between stacked layers. */
void lrd_ref_gelu_fwd(const double* Z, double* A, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) A[i] = 0.5 * Z[i] * (1.0 + erf(Z[i] / sqrt(2.0)));
}

void lrd_ref_gelu_bwd(const double* dA, const double* Z, double* dZ, int64_t n)
{
    const double inv_sqrt_2pi = 0.3989422804014326779;
    for (int64_t i = 0; i < n; ++i) {
        double z = Z[i];
        double Phi = 0.5 * (1.0 + erf(z / sqrt(2.0)));
        double phi = inv_sqrt_2pi * exp(-0.5 * z * z);
        dZ[i] = dA[i] * (Phi + z * phi);
    }
}

/* ------------------------------------------------------------------------------------------ */
/* Convolutions: NHWC activations, weights [O][k][k][I], cross-correlation, zero padding        */
/* ------------------------------------------------------------------------------------------ */

static int64_t conv_out_dim(int64_t n, int32_t k, int32_t s, int32_t p)
{
    return (n + 2 * (int64_t)p - k) / s + 1;
}

/* Y[n,y,x,o] = sum_{u,v,i} X[n, y*s+u-p, x*s+v-p, i] W[o,u,v,i] */
void lrd_ref_conv_fwd(const double* X, const double* W, double* Y, int64_t N, int64_t Hh,
                      int64_t Ww, int64_t I, int64_t O, int32_t k, int32_t s, int32_t p)
{
    int64_t Ho = conv_out_dim(Hh, k, s, p), Wo = conv_out_dim(Ww, k, s, p);
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t y = 0; y < Ho; ++y)
            for (int64_t x = 0; x < Wo; ++x)
                for (int64_t o = 0; o < O; ++o) {
                    double acc = 0.0;
                    for (int32_t u = 0; u < k; ++u) {
                        int64_t yy = y * s + u - p;
                        if (yy < 0 || yy >= Hh) continue;
                        for (int32_t v = 0; v < k; ++v) {
                            int64_t xx = x * s + v - p;
                            if (xx < 0 || xx >= Ww) continue;
                            const double* xp = X + ((n * Hh + yy) * Ww + xx) * I;
                            const double* wp = W + ((o * k + u) * k + v) * I;
                            for (int64_t i = 0; i < I; ++i) acc += xp[i] * wp[i];
                        }
                    }
                    Y[((n * Ho + y) * Wo + x) * O + o] = acc;
                }
}

/* dX[n,a,b,i] = sum over (y,u,x,v,o) with y*s+u-p = a, x*s+v-p = b of dY[n,y,x,o] W[o,u,v,i] */
void lrd_ref_conv_dgrad(const double* dY, const double* W, double* dX, int64_t N, int64_t Hh,
                        int64_t Ww, int64_t I, int64_t O, int32_t k, int32_t s, int32_t p)
{
    int64_t Ho = conv_out_dim(Hh, k, s, p), Wo = conv_out_dim(Ww, k, s, p);
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t a = 0; a < Hh; ++a)
            for (int64_t b = 0; b < Ww; ++b) {
                double* dx = dX + ((n * Hh + a) * Ww + b) * I;
                for (int64_t i = 0; i < I; ++i) dx[i] = 0.0;
                for (int32_t u = 0; u < k; ++u) {
                    int64_t ys = a + p - u;
                    if (ys < 0 || ys % s != 0) continue;
                    int64_t y = ys / s;
                    if (y >= Ho) continue;
                    for (int32_t v = 0; v < k; ++v) {
                        int64_t xs = b + p - v;
                        if (xs < 0 || xs % s != 0) continue;
                        int64_t x = xs / s;
                        if (x >= Wo) continue;
                        const double* gp = dY + ((n * Ho + y) * Wo + x) * O;
                        for (int64_t o = 0; o < O; ++o) {
                            const double* wp = W + ((o * k + u) * k + v) * I;
                            for (int64_t i = 0; i < I; ++i) dx[i] += gp[o] * wp[i];
                        }
                    }
                }
            }
}

/* dW[o,u,v,i] = sum_{n,y,x} dY[n,y,x,o] X[n, y*s+u-p, x*s+v-p, i] */
void lrd_ref_conv_wgrad(const double* dY, const double* X, double* dW, int64_t N, int64_t Hh,
                        int64_t Ww, int64_t I, int64_t O, int32_t k, int32_t s, int32_t p)
{
    int64_t Ho = conv_out_dim(Hh, k, s, p), Wo = conv_out_dim(Ww, k, s, p);
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < O; ++o) {
        for (int64_t e = 0; e < (int64_t)k * k * I; ++e) dW[o * k * k * I + e] = 0.0;
        /* pixels in ascending (n,y,x) order for every weight entry */
        for (int64_t n = 0; n < N; ++n)
            for (int64_t y = 0; y < Ho; ++y)
                for (int64_t x = 0; x < Wo; ++x) {
                    double g = dY[((n * Ho + y) * Wo + x) * O + o];
                    for (int32_t u = 0; u < k; ++u) {
                        int64_t yy = y * s + u - p;
                        if (yy < 0 || yy >= Hh) continue;
                        for (int32_t v = 0; v < k; ++v) {
                            int64_t xx = x * s + v - p;
                            if (xx < 0 || xx >= Ww) continue;
                            const double* xp = X + ((n * Hh + yy) * Ww + xx) * I;
                            double* wp = dW + ((o * k + u) * k + v) * I;
                            for (int64_t i = 0; i < I; ++i) wp[i] += g * xp[i];
                        }
                    }
                }
    }
}

/* A pointwise (1x1) layer over P pixels: Out[p,o] = sum_i In[p,i] M[o,i]. */
static void pointwise_fwd(const double* In, const double* M, double* Out, int64_t P, int64_t I,
                          int64_t O)
{
#pragma omp parallel for schedule(static)
    for (int64_t q = 0; q < P; ++q)
        for (int64_t o = 0; o < O; ++o) {
            double s = 0.0;
            for (int64_t i = 0; i < I; ++i) s += In[q * I + i] * M[o * I + i];
            Out[q * O + o] = s;
        }
}

/* dIn[p,i] = sum_o dOut[p,o] M[o,i] */
static void pointwise_dgrad(const double* dOut, const double* M, double* dIn, int64_t P, int64_t I,
                            int64_t O)
{
#pragma omp parallel for schedule(static)
    for (int64_t q = 0; q < P; ++q) {
        for (int64_t i = 0; i < I; ++i) dIn[q * I + i] = 0.0;
        for (int64_t o = 0; o < O; ++o) {
            double g = dOut[q * O + o];
            for (int64_t i = 0; i < I; ++i) dIn[q * I + i] += g * M[o * I + i];
        }
    }
}

/* dM[o,i] = sum_p dOut[p,o] In[p,i] */
static void pointwise_wgrad(const double* dOut, const double* In, double* dM, int64_t P, int64_t I,
                            int64_t O)
{
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < O; ++o) {
        for (int64_t i = 0; i < I; ++i) dM[o * I + i] = 0.0;
        for (int64_t q = 0; q < P; ++q) {
            double g = dOut[q * O + o];
            for (int64_t i = 0; i < I; ++i) dM[o * I + i] += g * In[q * I + i];
        }
    }
}

/*
 * Tucker-2 decomposed k x k convolution (eq. 4; Section 2: "a 1x1 followed by a 3x3 and then
 * another 1x1").  Stride and padding act on the core; the 1x1 layers are stride 1, pad 0.
 * A [N,H,W,r1], B [N,Ho,Wo,r2], Y [N,Ho,Wo,S] are all returned.
 */
void lrd_ref_tucker_fwd(const double* X, const double* P1, const double* G, const double* P2,
                        double* A, double* B, double* Y, int64_t N, int64_t Hh, int64_t Ww,
                        int64_t C, int64_t S, int64_t r1, int64_t r2, int32_t k, int32_t s,
                        int32_t p)
{
    int64_t Ho = conv_out_dim(Hh, k, s, p), Wo = conv_out_dim(Ww, k, s, p);
    pointwise_fwd(X, P1, A, N * Hh * Ww, C, r1);
    lrd_ref_conv_fwd(A, G, B, N, Hh, Ww, r1, r2, k, s, p);
    pointwise_fwd(B, P2, Y, N * Ho * Wo, r2, S);
}

/*
 * Backward of the triple.  dB, dA, dX always; dP1 unless bit0, dG unless bit1, dP2 unless bit2.
 */
void lrd_ref_tucker_bwd(const double* dY, const double* X, const double* A, const double* B,
                        const double* P1, const double* G, const double* P2, double* dB,
                        double* dA, double* dX, double* dP1, double* dG, double* dP2,
                        uint32_t mask, int64_t N, int64_t Hh, int64_t Ww, int64_t C, int64_t S,
                        int64_t r1, int64_t r2, int32_t k, int32_t s, int32_t p)
{
    int64_t Ho = conv_out_dim(Hh, k, s, p), Wo = conv_out_dim(Ww, k, s, p);
    int64_t Pin = N * Hh * Ww, Pout = N * Ho * Wo;
    pointwise_dgrad(dY, P2, dB, Pout, r2, S);
    lrd_ref_conv_dgrad(dB, G, dA, N, Hh, Ww, r1, r2, k, s, p);
    if (dX) pointwise_dgrad(dA, P1, dX, Pin, C, r1);
    if (!(mask & LRD_REF_FREEZE_L2) && dP2) pointwise_wgrad(dY, B, dP2, Pout, r2, S);
    if (!(mask & LRD_REF_FREEZE_L1) && dG) lrd_ref_conv_wgrad(dB, A, dG, N, Hh, Ww, r1, r2, k, s, p);
    if (!(mask & LRD_REF_FREEZE_L0) && dP1) pointwise_wgrad(dA, X, dP1, Pin, C, r1);
}

/* ------------------------------------------------------------------------------------------ */
/* Optimizer step of the experiments (Section 3: SGD with momentum 0.9 and weight decay 1e-4)   */
/* ------------------------------------------------------------------------------------------ */

/*
 * One step of stochastic gradient descent with momentum and weight decay on n parameters, in the
 * usual form: g' = g + wd * w;  m <- mu * m + g';  w <- w - lr * m.  A momentum buffer that
 * starts at zero makes the first step m = g', the common initialisation.
 */
void lrd_ref_sgd_step(double* w, double* m, const double* g, int64_t n, double lr, double mu, double wd)
{
    for (int64_t i = 0; i < n; ++i) {
        double gi = g[i] + wd * w[i];
        m[i] = mu * m[i] + gi;
        w[i] = w[i] - lr * m[i];
    }
}

/* ------------------------------------------------------------------------------------------ */
/* One-time factorization (eq. 1, 2, 4)                                                         */
/* ------------------------------------------------------------------------------------------ */

/*
 * Singular value decomposition by one-sided (Hestenes) Jacobi rotations, eq. 1.
 * M is m x n, row-major.  On return, with R = min(m,n):
 *   Uo [m x R]  left singular vectors (columns), sig [R] descending, Vo [n x R] right vectors,
 *   so that M = Uo diag(sig) Vo^T.  Columns belonging to a zero singular value are left zero.
 * Returns the number of sweeps used, or -1 if it did not converge / ran out of memory.
 */
int lrd_ref_svd(const double* M, int64_t m, int64_t n, double* Uo, double* sig, double* Vo)
{
    /* Work on the orientation with at least as many rows as columns: B is mm x nn, mm >= nn. */
    int flip = m < n;
    int64_t mm = flip ? n : m, nn = flip ? m : n;
    /* Column-major copies make the column rotations contiguous. */
    double* B = (double*)malloc(sizeof(double) * (size_t)mm * (size_t)nn);
    double* Q = (double*)calloc((size_t)nn * (size_t)nn, sizeof(double));
    double* nrm = (double*)malloc(sizeof(double) * (size_t)nn);
    int64_t* ord = (int64_t*)malloc(sizeof(int64_t) * (size_t)nn);
    if (!B || !Q || !nrm || !ord) {
        free(B); free(Q); free(nrm); free(ord);
        return -1;
    }
    for (int64_t c = 0; c < nn; ++c)
        for (int64_t rr = 0; rr < mm; ++rr)
            B[c * mm + rr] = flip ? M[c * n + rr] : M[rr * n + c];
    for (int64_t c = 0; c < nn; ++c) Q[c * nn + c] = 1.0;

    const double tol = 1e-15;
    int sweeps = 0, converged = 0;
    for (sweeps = 1; sweeps <= 60 && !converged; ++sweeps) {
        converged = 1;
        for (int64_t a = 0; a < nn - 1; ++a)
            for (int64_t b = a + 1; b < nn; ++b) {
                double* ca = B + a * mm;
                double* cb = B + b * mm;
                double aa = 0.0, bb = 0.0, ab = 0.0;
                for (int64_t i = 0; i < mm; ++i) {
                    aa += ca[i] * ca[i];
                    bb += cb[i] * cb[i];
                    ab += ca[i] * cb[i];
                }
                if (ab == 0.0 || fabs(ab) <= tol * sqrt(aa * bb)) continue;
                converged = 0;
                /* Rotation angle that makes the two columns orthogonal. */
                double zeta = (bb - aa) / (2.0 * ab);
                double tt = (zeta >= 0.0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
                double cs = 1.0 / sqrt(1.0 + tt * tt), sn = cs * tt;
                for (int64_t i = 0; i < mm; ++i) {
                    double x = ca[i], y = cb[i];
                    ca[i] = cs * x - sn * y;
                    cb[i] = sn * x + cs * y;
                }
                double* qa = Q + a * nn;
                double* qb = Q + b * nn;
                for (int64_t i = 0; i < nn; ++i) {
                    double x = qa[i], y = qb[i];
                    qa[i] = cs * x - sn * y;
                    qb[i] = sn * x + cs * y;
                }
            }
    }
    sweeps -= 1;

    for (int64_t c = 0; c < nn; ++c) {
        double s = 0.0;
        for (int64_t i = 0; i < mm; ++i) s += B[c * mm + i] * B[c * mm + i];
        nrm[c] = sqrt(s);
        ord[c] = c;
    }
    /* Sort indices by descending singular value (insertion sort: nn is small). */
    for (int64_t i = 1; i < nn; ++i) {
        int64_t key = ord[i];
        int64_t j = i - 1;
        while (j >= 0 && nrm[ord[j]] < nrm[key]) {
            ord[j + 1] = ord[j];
            --j;
        }
        ord[j + 1] = key;
    }
    /* B = (left vectors of the working orientation) * diag(sigma); Q = its right vectors. */
    for (int64_t c = 0; c < nn; ++c) {
        int64_t src = ord[c];
        double sg = nrm[src];
        sig[c] = sg;
        for (int64_t i = 0; i < mm; ++i) {
            double left = sg > 0.0 ? B[src * mm + i] / sg : 0.0;
            if (flip) Vo[i * nn + c] = left; else Uo[i * nn + c] = left;
        }
        for (int64_t i = 0; i < nn; ++i) {
            double right = sg > 0.0 ? Q[src * nn + i] : 0.0;
            if (flip) Uo[i * nn + c] = right; else Vo[i * nn + c] = right;
        }
    }
    free(B); free(Q); free(nrm); free(ord);
    return converged ? sweeps : -1;
}

/*
 * Rank-r factor pair of a layer weight W [out x in] (eq. 2), singular values shared evenly:
 *   U [out x r] = (left vectors) diag(sqrt sigma),  V [r x in] = diag(sqrt sigma) (right vectors)^T.
 * sig_all (optional, length min(out,in)) receives every singular value (for eq. 3's error).
 */
int lrd_ref_svd_factors(const double* W, int64_t out, int64_t in, int64_t r, double* U, double* V,
                        double* sig_all)
{
    int64_t R = out < in ? out : in;
    if (r < 1 || r > R) return -1;
    double* Uo = (double*)malloc(sizeof(double) * (size_t)out * (size_t)R);
    double* Vo = (double*)malloc(sizeof(double) * (size_t)in * (size_t)R);
    double* sg = (double*)malloc(sizeof(double) * (size_t)R);
    if (!Uo || !Vo || !sg) { free(Uo); free(Vo); free(sg); return -1; }
    int rc = lrd_ref_svd(W, out, in, Uo, sg, Vo);
    if (rc >= 0) {
        for (int64_t j = 0; j < r; ++j) {
            double h = sqrt(sg[j]);
            for (int64_t o = 0; o < out; ++o) U[o * r + j] = Uo[o * R + j] * h;
            for (int64_t i = 0; i < in; ++i) V[j * in + i] = Vo[i * R + j] * h;
        }
        if (sig_all) memcpy(sig_all, sg, sizeof(double) * (size_t)R);
    }
    free(Uo); free(Vo); free(sg);
    return rc;
}

/*
 * Tucker-2 of a conv weight W [S][k][k][C] by truncated higher-order SVD on the two channel
 * modes (eq. 4; the spatial mode is left whole).  P1 [r1 x C]: leading left singular vectors of
 * the C-mode unfolding, transposed.  P2 [S x r2]: those of the S-mode unfolding.  Core
 * G [r2][k][k][r1] = W contracted with P1 on its C index and with P2 on its S index.
 * tau (optional, 2 doubles) gets the discarded squared singular values of each unfolding.
 */
int lrd_ref_tucker2(const double* W, int64_t S, int64_t C, int32_t k, int64_t r1, int64_t r2,
                    double* P1, double* G, double* P2, double* tau)
{
    int64_t kk = (int64_t)k * k;
    if (r1 < 1 || r1 > C || r2 < 1 || r2 > S) return -1;
    int rc = -1;
    /* Mode-C unfolding: rows = c, columns = (o,u,v). */
    int64_t nc = S * kk, ns = C * kk;
    int64_t Rc = C < nc ? C : nc, Rs = S < ns ? S : ns;
    if (r1 > Rc || r2 > Rs) return -1;
    double* Mc = (double*)malloc(sizeof(double) * (size_t)C * (size_t)nc);
    double* Ms = (double*)malloc(sizeof(double) * (size_t)S * (size_t)ns);
    double* Uc = (double*)malloc(sizeof(double) * (size_t)C * (size_t)Rc);
    double* Vc = (double*)malloc(sizeof(double) * (size_t)nc * (size_t)Rc);
    double* Us = (double*)malloc(sizeof(double) * (size_t)S * (size_t)Rs);
    double* Vs = (double*)malloc(sizeof(double) * (size_t)ns * (size_t)Rs);
    double* sc = (double*)malloc(sizeof(double) * (size_t)Rc);
    double* ss = (double*)malloc(sizeof(double) * (size_t)Rs);
    double* tmp = (double*)malloc(sizeof(double) * (size_t)S * (size_t)kk * (size_t)r1);
    if (Mc && Ms && Uc && Vc && Us && Vs && sc && ss && tmp) {
        for (int64_t o = 0; o < S; ++o)
            for (int64_t q = 0; q < kk; ++q)
                for (int64_t c = 0; c < C; ++c) {
                    double w = W[(o * kk + q) * C + c];
                    Mc[c * nc + (o * kk + q)] = w;
                    Ms[o * ns + (q * C + c)] = w;
                }
        int r_a = lrd_ref_svd(Mc, C, nc, Uc, sc, Vc);
        int r_b = lrd_ref_svd(Ms, S, ns, Us, ss, Vs);
        if (r_a >= 0 && r_b >= 0) {
            for (int64_t a = 0; a < r1; ++a)
                for (int64_t c = 0; c < C; ++c) P1[a * C + c] = Uc[c * Rc + a];
            for (int64_t o = 0; o < S; ++o)
                for (int64_t b = 0; b < r2; ++b) P2[o * r2 + b] = Us[o * Rs + b];
            /* tmp[o,q,a] = sum_c W[o,q,c] P1[a,c] */
            for (int64_t o = 0; o < S; ++o)
                for (int64_t q = 0; q < kk; ++q)
                    for (int64_t a = 0; a < r1; ++a) {
                        double s = 0.0;
                        for (int64_t c = 0; c < C; ++c) s += W[(o * kk + q) * C + c] * P1[a * C + c];
                        tmp[(o * kk + q) * r1 + a] = s;
                    }
            /* G[b,q,a] = sum_o P2[o,b] tmp[o,q,a] */
            for (int64_t b = 0; b < r2; ++b)
                for (int64_t q = 0; q < kk; ++q)
                    for (int64_t a = 0; a < r1; ++a) {
                        double s = 0.0;
                        for (int64_t o = 0; o < S; ++o) s += P2[o * r2 + b] * tmp[(o * kk + q) * r1 + a];
                        G[(b * kk + q) * r1 + a] = s;
                    }
            if (tau) {
                tau[0] = 0.0;
                tau[1] = 0.0;
                for (int64_t a = r1; a < Rc; ++a) tau[0] += sc[a] * sc[a];
                for (int64_t b = r2; b < Rs; ++b) tau[1] += ss[b] * ss[b];
            }
            rc = 0;
        }
    }
    free(Mc); free(Ms); free(Uc); free(Vc); free(Us); free(Vs); free(sc); free(ss); free(tmp);
    return rc;
}

/* Threads the loops above will use (1 when built without OpenMP). */
#ifdef _OPENMP
#include <omp.h>
int lrd_ref_threads(void) { return omp_get_max_threads(); }
void lrd_ref_set_threads(int n) { if (n > 0) omp_set_num_threads(n); }
#else
int lrd_ref_threads(void) { return 1; }
void lrd_ref_set_threads(int n) { (void)n; }
#endif
