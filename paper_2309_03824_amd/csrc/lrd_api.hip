// C-ABI entry points: argument validation, workspace carving, and the composition of each layer
// pass out of matrix products (see lrd.h for the contract of every call).
#include <algorithm>
#include <atomic>
#include <mutex>

#include "lrd.h"
#include "lrd_internal.hpp"
#include "lrd_measure.h"

namespace lrd {
namespace {

std::atomic<int> g_fusion{LRD_FUSION_AUTO};

// Whether the fused pair kernel should take this shape.  AUTO: measured on MI355X, two separate
// products are faster at every workload shape tried so far (the fused kernel runs one workgroup
// per compute unit and pays a barrier per K-step), so AUTO currently resolves to "no".
inline bool want_fusion(const ChainOp& ch)
{
    int mode = g_fusion.load(std::memory_order_relaxed);
    if (mode == LRD_FUSION_NEVER) return false;
    if (!mfma_chain_supported(ch)) return false;
    return mode == LRD_FUSION_ALWAYS;
}

hipError_t run_chain(const ChainOp& ch, hipStream_t st)
{
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    const int logged = log_begin(&ev0, &ev1);
    if (logged >= 0) (void)hipEventRecord(ev0, st);
    note_kernel("chain_kernel (pair through LDS)");
    hipError_t e = mfma_chain(ch, st);
    if (logged >= 0) {
        (void)hipEventRecord(ev1, st);
        log_end(logged, ch.role, 0, 0, 1, ch.M, ch.N2, ch.K1, 1);
    }
    return e;
}

// A bf16 rank that is not a multiple of 8 breaks 16-byte loads on every operand whose leading
// dimension is r.  Such a pair is evaluated at the padded rank r8 = ceil(r/8)*8 on zero-padded
// copies of the (small) factors and of H, so that the large activations keep the fast kernels;
// the rank then costs the padding copies and the padded MFMA work, not a different code path.
inline int64_t pad8(int64_t r) { return (r + 7) / 8 * 8; }
inline bool pads_rank(int64_t in, int64_t out, int64_t r, lrd_dtype dt)
{
    return dt == LRD_BF16 && r % 8 != 0 && in % 8 == 0 && out % 8 == 0;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round256(size_t b) { return (b + 255) & ~size_t(255); }
inline size_t esize(lrd_dtype dt) { return dt == LRD_BF16 ? 2 : 4; }
inline bool dtype_ok(lrd_dtype dt) { return dt == LRD_F32 || dt == LRD_BF16; }

// Bump allocator over the caller's workspace.
struct Carver {
    char* base;
    size_t cap, used = 0;
    bool ok = true;
    Carver(void* p, size_t n) : base((char*)p), cap(n) {}
    void* take(size_t bytes)
    {
        size_t b = round256(bytes);
        if (!base || used + b > cap) { ok = false; return nullptr; }
        void* p = base + used;
        used += b;
        return p;
    }
};

#define LRD_TRY(expr)                                   \
    do {                                                \
        hipError_t e__ = (expr);                        \
        if (e__ != hipSuccess) return LRD_ERR_RUNTIME;  \
    } while (0)

// C[M x N] = A[M x K] . B^T with row-major operands A [M x K], B [N x K].
MatOp nt(const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc, int64_t M,
         int64_t N, int64_t K, lrd_dtype dt, bool out_f32)
{
    MatOp op;
    op.A = A; op.a_sm = lda; op.a_sk = 1;
    op.B = B; op.b_sn = ldb; op.b_sk = 1;
    op.C = C; op.ldc = ldc;
    op.M = M; op.N = N; op.K = K;
    op.in_bf16 = dt == LRD_BF16;
    op.out_f32 = out_f32 || dt == LRD_F32;
    return op;
}

// C[M x N] = A[M x K] . B with row-major B [K x N].
MatOp nn(const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc, int64_t M,
         int64_t N, int64_t K, lrd_dtype dt)
{
    MatOp op = nt(A, lda, B, 0, C, ldc, M, N, K, dt, false);
    op.b_sn = 1; op.b_sk = ldb;
    return op;
}

// C[M x N] (fp32) = A^T . B with row-major A [K x M], B [K x N]: the weight-gradient shape.
MatOp tn(const void* A, int64_t lda, const void* B, int64_t ldb, float* C, int64_t ldc, int64_t M,
         int64_t N, int64_t K, lrd_dtype dt)
{
    MatOp op = nt(A, 0, B, 0, C, ldc, M, N, K, dt, true);
    op.a_sm = 1; op.a_sk = lda;
    op.b_sn = 1; op.b_sk = ldb;
    return op;
}

size_t partial_bytes(int64_t M, int64_t N, int64_t K, lrd_dtype dt)
{
    int s = choose_splits(M, N, K, dt == LRD_BF16);
    return s > 1 ? round256((size_t)s * (size_t)M * (size_t)N * sizeof(float)) : 0;
}

// The same for a product whose result is a narrow activation.
size_t act_partial_bytes(int64_t M, int64_t N, int64_t K, lrd_dtype dt)
{
    int s = choose_splits_act(M, N, K, dt == LRD_BF16);
    return s > 1 ? round256((size_t)s * (size_t)M * (size_t)N * sizeof(float)) : 0;
}

// Split products of one linear pass run one after the other on the stream and share one region.
size_t linear_partial_region(int64_t T, int64_t in, int64_t out, int64_t r, lrd_dtype dt, bool backward)
{
    const size_t h = act_partial_bytes(T, r, in, dt);   // H = X.V^T (forward, or recomputed in the backward)
    if (!backward) return h;
    return std::max(std::max(h, act_partial_bytes(T, r, out, dt)),
                    std::max(partial_bytes(out, r, T, dt), partial_bytes(r, in, T, dt)));
}

enum SplitKind { SPLIT_WGRAD, SPLIT_ACT };
void share_splits(MatOp& op, void* region, lrd_dtype dt, SplitKind kind)
{
    int s = kind == SPLIT_WGRAD ? choose_splits(op.M, op.N, op.K, dt == LRD_BF16)
                                : choose_splits_act(op.M, op.N, op.K, dt == LRD_BF16);
    if (s > 1 && region) {
        op.partial = (float*)region;
        op.splits = s;
    }
}

void attach_splits(MatOp& op, Carver& cv, lrd_dtype dt)
{
    int s = choose_splits(op.M, op.N, op.K, dt == LRD_BF16);
    if (s > 1) {
        op.partial = (float*)cv.take((size_t)s * (size_t)op.M * (size_t)op.N * sizeof(float));
        op.splits = op.partial ? s : 1;
    }
}

bool linear_dims_ok(int64_t T, int64_t in, int64_t out, int64_t r)
{
    return T >= 1 && in >= 1 && out >= 1 && r >= 1 && r <= std::min(in, out) &&
           T < (int64_t(1) << 31) && in < (int64_t(1) << 24) && out < (int64_t(1) << 24);
}

ConvShape core_shape(const lrd_conv_geom& g, int64_t I, int64_t O)
{
    ConvShape cs;
    cs.N = (int)g.N; cs.H = (int)g.H; cs.W = (int)g.W;
    cs.Ho = (int)((g.H + 2 * g.pad - g.k) / g.stride + 1);
    cs.Wo = (int)((g.W + 2 * g.pad - g.k) / g.stride + 1);
    cs.I = (int)I; cs.O = (int)O;
    cs.k = g.k; cs.stride = g.stride; cs.pad = g.pad;
    return cs;
}

bool geom_ok(const lrd_conv_geom* g, bool tucker)
{
    if (!g) return false;
    if (g->N < 1 || g->H < 1 || g->W < 1 || g->C < 1 || g->S < 1) return false;
    if (g->k < 1 || g->stride < 1 || g->pad < 0) return false;
    if (g->H + 2 * g->pad < g->k || g->W + 2 * g->pad < g->k) return false;
    if (tucker && (g->r1 < 1 || g->r1 > g->C || g->r2 < 1 || g->r2 > g->S)) return false;
    const int64_t lim = int64_t(1) << 31;
    int64_t widest = std::max(std::max(g->C, g->S), std::max(g->r1, g->r2));
    if (g->N * g->H * g->W >= lim / std::max<int64_t>(widest, 1)) return false;  // 32-bit pixel*channel index space
    return true;
}

}  // namespace
}  // namespace lrd

using namespace lrd;

extern "C" {

int32_t lrd_set_fusion(int32_t mode)
{
    if (mode != LRD_FUSION_AUTO && mode != LRD_FUSION_ALWAYS && mode != LRD_FUSION_NEVER) return -1;
    return g_fusion.exchange(mode);
}

// ------------------------------------------------------------------------------------ linear
size_t lrd_linear_workspace_bytes(int64_t T, int64_t in, int64_t out, int64_t r, lrd_dtype dt,
                                  uint32_t freeze_mask)
{
    (void)freeze_mask;
    if (!dtype_ok(dt) || !linear_dims_ok(T, in, out, r)) return 0;
    if (pads_rank(in, out, r, dt)) {
        const size_t r8 = (size_t)pad8(r);
        size_t pads = round256((size_t)out * r8 * 2) + round256(r8 * (size_t)in * 2) + round256((size_t)T * r8 * 2) +
                      round256((size_t)out * r8 * 4) + round256(r8 * (size_t)in * 4);
        return pads + lrd_linear_workspace_bytes(T, in, out, (int64_t)r8, dt, freeze_mask);
    }
    size_t act = round256((size_t)T * (size_t)r * esize(dt));
    // forward: H when not side-stored; backward: dH and a recomputed H; both: one split-K region
    size_t fwd = act + linear_partial_region(T, in, out, r, dt, false);
    size_t bwd = 2 * act + linear_partial_region(T, in, out, r, dt, true);
    return std::max(fwd, bwd);
}

lrd_status lrd_linear_fwd(const void* X, const void* V, const void* U, const float* bias, void* Y,
                          void* H_save, int64_t T, int64_t in, int64_t out, int64_t r,
                          lrd_dtype dt, void* ws, size_t ws_bytes, void* hip_stream)
{
    return lrd_linear_fwd_act(X, V, U, bias, Y, nullptr, H_save, LRD_ACT_NONE, T, in, out, r, dt, ws, ws_bytes,
                              hip_stream);
}

lrd_status lrd_linear_fwd_act(const void* X, const void* V, const void* U, const float* bias, void* Y,
                              void* Y_act, void* H_save, int32_t act, int64_t T, int64_t in, int64_t out,
                              int64_t r, lrd_dtype dt, void* ws, size_t ws_bytes, void* hip_stream)
{
    if (!dtype_ok(dt) || !linear_dims_ok(T, in, out, r) || !X || !V || !U || !Y) return LRD_ERR_INVALID_ARG;
    if ((act != LRD_ACT_NONE && act != LRD_ACT_GELU) || (act == LRD_ACT_GELU && !Y_act)) return LRD_ERR_INVALID_ARG;
    if (act == LRD_ACT_NONE) Y_act = nullptr;
    if (!aligned16(X) || !aligned16(V) || !aligned16(U) || !aligned16(Y) || !aligned16(H_save) || !aligned16(ws) ||
        !aligned16(bias) || !aligned16(Y_act))
        return LRD_ERR_ALIGNMENT;
    hipStream_t st = (hipStream_t)hip_stream;

    if (pads_rank(in, out, r, dt)) {
        const int64_t r8 = pad8(r);
        Carver cv(ws, ws_bytes);
        void* Up = cv.take((size_t)out * r8 * 2);
        void* Vp = cv.take((size_t)r8 * in * 2);
        void* Hp = cv.take((size_t)T * r8 * 2);
        if (!cv.ok) return LRD_ERR_WORKSPACE;
        LRD_TRY(copy2d(U, r, out, r, Up, r8, out, r8, 2, st));
        LRD_TRY(copy2d(V, in, r, in, Vp, in, r8, in, 2, st));
        lrd_status rc = lrd_linear_fwd_act(X, Vp, Up, bias, Y, Y_act, Hp, act, T, in, out, r8, dt, (char*)ws + cv.used,
                                           ws_bytes - cv.used, hip_stream);
        if (rc != LRD_OK) return rc;
        if (H_save) LRD_TRY(copy2d(Hp, r8, T, r, H_save, r, T, r, 2, st));
        return LRD_OK;
    }

    if (dt == LRD_BF16) {
        ChainOp ch;
        ch.A = X; ch.lda = in;
        ch.B1 = V; ch.b1_sn = in; ch.b1_sk = 1;
        ch.B2 = U; ch.b2_sn = r; ch.b2_sk = 1;
        ch.C = Y; ch.ldc = out;
        ch.mid_save = H_save; ch.ldmid = r;
        ch.bias = bias;
        ch.M = T; ch.K1 = in; ch.R = r; ch.N2 = out;
        ch.role = LRD_ROLE_FWD_DOWN;
        if (want_fusion(ch)) {
            LRD_TRY(run_chain(ch, st));
            if (Y_act) LRD_TRY(gelu_fwd(Y, Y_act, T * out, true, st));
            return LRD_OK;
        }
    }
    Carver cv(ws, ws_bytes);
    void* H = H_save ? H_save : cv.take((size_t)T * r * esize(dt));
    const size_t region_bytes = linear_partial_region(T, in, out, r, dt, false);
    void* region = region_bytes ? cv.take(region_bytes) : nullptr;
    if (!H || !cv.ok) return LRD_ERR_WORKSPACE;
    MatOp g1 = nt(X, in, V, in, H, r, T, r, in, dt, false);
    share_splits(g1, region, dt, SPLIT_ACT);
    MatOp g2 = nt(H, r, U, r, Y, out, T, out, r, dt, false);
    g2.bias = bias;
    g1.role = LRD_ROLE_FWD_DOWN;
    g2.role = LRD_ROLE_FWD_UP;
    if (Y_act) {
        g2.epilogue = EPI_ACT_STORE;
        g2.aux = Y_act;
        g2.ldaux = out;
    }
    LRD_TRY(run_matop(g1, st));
    LRD_TRY(run_matop(g2, st));
    return LRD_OK;
}

lrd_status lrd_linear_bwd(const void* dY, const void* X, const void* H, const void* V,
                          const void* U, void* dX, float* dV, float* dU, float* dbias,
                          uint32_t freeze_mask, int64_t T, int64_t in, int64_t out, int64_t r,
                          lrd_dtype dt, void* ws, size_t ws_bytes, void* hip_stream)
{
    return lrd_linear_bwd_act(dY, X, H, V, U, dX, dV, dU, dbias, freeze_mask, nullptr, LRD_ACT_NONE, T, in, out, r,
                              dt, ws, ws_bytes, hip_stream);
}

namespace {
// lrd_linear_bwd_act; with sgd_u / sgd_v the optimizer step of that factor is applied where its
// gradient is finished (no padded ranks then: their gradients are cropped first).
lrd_status linear_bwd_impl(const void* dY, const void* X, const void* H, const void* V, const void* U, void* dX, float* dV,
                           float* dU, float* dbias, uint32_t freeze_mask, const void* Z_in, int32_t act, int64_t T,
                           int64_t in, int64_t out, int64_t r, lrd_dtype dt, void* ws, size_t ws_bytes, void* hip_stream,
                           const SgdFuse* sgd_u, const SgdFuse* sgd_v)
{
    if (!dtype_ok(dt) || !linear_dims_ok(T, in, out, r) || !dY || !V || !U) return LRD_ERR_INVALID_ARG;
    if ((act != LRD_ACT_NONE && act != LRD_ACT_GELU) || (act == LRD_ACT_GELU && dX && !Z_in)) return LRD_ERR_INVALID_ARG;
    if (act == LRD_ACT_NONE || !dX) Z_in = nullptr;
    if (!aligned16(Z_in)) return LRD_ERR_ALIGNMENT;
    if (freeze_mask & ~uint32_t(LRD_FREEZE_L0 | LRD_FREEZE_L1)) return LRD_ERR_INVALID_ARG;
    const bool train_v = !(freeze_mask & LRD_FREEZE_L0), train_u = !(freeze_mask & LRD_FREEZE_L1);
    if (train_v && (!dV || !X)) return LRD_ERR_INVALID_ARG;
    if (train_u && (!dU || (!H && !X))) return LRD_ERR_INVALID_ARG;
    if (!aligned16(dY) || !aligned16(X) || !aligned16(H) || !aligned16(V) || !aligned16(U) || !aligned16(dX) ||
        !aligned16(ws) || (train_v && !aligned16(dV)) || (train_u && !aligned16(dU)) || !aligned16(dbias))
        return LRD_ERR_ALIGNMENT;
    hipStream_t st = (hipStream_t)hip_stream;
    if (pads_rank(in, out, r, dt)) {
        const int64_t r8 = pad8(r);
        Carver cvp(ws, ws_bytes);
        void* Up = cvp.take((size_t)out * r8 * 2);
        void* Vp = cvp.take((size_t)r8 * in * 2);
        void* Hp = cvp.take((size_t)T * r8 * 2);
        float* dUp = (float*)cvp.take((size_t)out * r8 * 4);
        float* dVp = (float*)cvp.take((size_t)r8 * in * 4);
        if (!cvp.ok) return LRD_ERR_WORKSPACE;
        LRD_TRY(copy2d(U, r, out, r, Up, r8, out, r8, 2, st));
        LRD_TRY(copy2d(V, in, r, in, Vp, in, r8, in, 2, st));
        const bool have_h = H && train_u;
        if (have_h) LRD_TRY(copy2d(H, r, T, r, Hp, r8, T, r8, 2, st));
        if (sgd_u || sgd_v) return LRD_ERR_INVALID_ARG;
        lrd_status rc = lrd_linear_bwd_act(dY, X, have_h ? Hp : nullptr, Vp, Up, dX, dVp, dUp, dbias, freeze_mask, Z_in, act, T,
                                           in, out, r8, dt, (char*)ws + cvp.used, ws_bytes - cvp.used, hip_stream);
        if (rc != LRD_OK) return rc;
        if (train_u) LRD_TRY(copy2d(dUp, r8, out, r, dU, r, out, r, 4, st));
        if (train_v) LRD_TRY(copy2d(dVp, in, r, in, dV, in, r, in, 4, st));
        return LRD_OK;
    }
    Carver cv(ws, ws_bytes);
    const size_t act_bytes = (size_t)T * r * esize(dt);
    const bool need_dH = dX || train_v;

    // Carve everything first so that a short workspace is reported before any launch.
    void* dH = need_dH ? cv.take(act_bytes) : nullptr;
    void* Hre = (train_u && !H) ? cv.take(act_bytes) : nullptr;
    const size_t region_bytes = linear_partial_region(T, in, out, r, dt, true);
    void* region = region_bytes ? cv.take(region_bytes) : nullptr;
    MatOp wu, wv;
    if (train_u) {
        wu = tn(dY, out, H ? H : Hre, r, dU, r, out, r, T, dt);
        wu.role = LRD_ROLE_WGRAD_U;
        wu.sgd = sgd_u;
        share_splits(wu, region, dt, SPLIT_WGRAD);
    }
    if (train_v) {
        wv = tn(dH, r, X, in, dV, in, r, in, T, dt);
        wv.role = LRD_ROLE_WGRAD_V;
        wv.sgd = sgd_v;
        share_splits(wv, region, dt, SPLIT_WGRAD);
    }
    if (!cv.ok) return LRD_ERR_WORKSPACE;

    if (need_dH) {
        bool fused = false;
        if (dt == LRD_BF16 && dX) {
            ChainOp ch;
            ch.A = dY; ch.lda = out;
            ch.B1 = U; ch.b1_sn = 1; ch.b1_sk = r;     // B1(j, o) = U[o][j]
            ch.B2 = V; ch.b2_sn = 1; ch.b2_sk = in;    // B2(i, j) = V[j][i]
            ch.C = dX; ch.ldc = in;
            ch.mid_save = train_v ? dH : nullptr; ch.ldmid = r;
            ch.M = T; ch.K1 = out; ch.R = r; ch.N2 = in;
            ch.role = LRD_ROLE_DGRAD_UP;
            if (want_fusion(ch)) {
                LRD_TRY(run_chain(ch, st));
                if (Z_in) LRD_TRY(gelu_bwd(dX, Z_in, dX, T * in, true, st));
                fused = true;
            }
        }
        if (!fused) {
            MatOp d1 = nn(dY, out, U, r, dH, r, T, r, out, dt);
            d1.role = LRD_ROLE_DGRAD_UP;
            share_splits(d1, region, dt, SPLIT_ACT);
            LRD_TRY(run_matop(d1, st));
            if (dX) {
                MatOp d2 = nn(dH, r, V, in, dX, in, T, in, r, dt);
                d2.role = LRD_ROLE_DGRAD_DOWN;
                if (Z_in) {
                    d2.epilogue = EPI_ACT_GRAD;
                    d2.aux = const_cast<void*>(Z_in);
                    d2.ldaux = in;
                }
                LRD_TRY(run_matop(d2, st));
            }
        }
    }
    if (train_u) {
        if (!H) {
            MatOp re = nt(X, in, V, in, Hre, r, T, r, in, dt, false);
            share_splits(re, region, dt, SPLIT_ACT);
            LRD_TRY(run_matop(re, st));
        }
        LRD_TRY(run_matop(wu, st));
    }
    if (train_v) LRD_TRY(run_matop(wv, st));
    if (dbias) LRD_TRY(column_sums(dY, dbias, T, out, dt == LRD_BF16, st));
    return LRD_OK;
}
}  // namespace

lrd_status lrd_linear_bwd_act(const void* dY, const void* X, const void* H, const void* V,
                              const void* U, void* dX, float* dV, float* dU, float* dbias,
                              uint32_t freeze_mask, const void* Z_in, int32_t act, int64_t T, int64_t in,
                              int64_t out, int64_t r, lrd_dtype dt, void* ws, size_t ws_bytes, void* hip_stream)
{
    return linear_bwd_impl(dY, X, H, V, U, dX, dV, dU, dbias, freeze_mask, Z_in, act, T, in, out, r, dt, ws, ws_bytes, hip_stream,
                           nullptr, nullptr);
}

// ------------------------------------------------------------------------------------ allocation-free backward
namespace {
// Scratch of lrd_linear_bwd_static.  In host code this name is only a handle for the symbol, not a
// device address: the address on each GPU comes from hipGetSymbolAddress, once per device.
static __device__ __align__(256) unsigned char scratch[LRD_STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
void* g_scratch_ptr[MAX_DEVICES] = {};
std::mutex g_scratch_mutex;

// Address of `scratch` on the current device, or nullptr if the runtime refuses.
void* scratch_on_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

int32_t lrd_linear_bwd_static_fits(int64_t T, int64_t in, int64_t out, int64_t r, lrd_dtype dt, uint32_t freeze_mask)
{
    const size_t need = lrd_linear_workspace_bytes(T, in, out, r, dt, freeze_mask);
    if (!dtype_ok(dt) || !linear_dims_ok(T, in, out, r)) return 0;
    return need <= LRD_STATIC_SCRATCH_BYTES ? 1 : 0;
}

lrd_status lrd_linear_bwd_static(const void* dY, const void* X, const void* H, const void* V, const void* U, void* dX,
                                 float* dV, float* dU, float* dbias, uint32_t freeze_mask, int64_t T, int64_t in,
                                 int64_t out, int64_t r, lrd_dtype dt, void* hip_stream)
{
    if (!dtype_ok(dt) || !linear_dims_ok(T, in, out, r)) return LRD_ERR_INVALID_ARG;
    if (!lrd_linear_bwd_static_fits(T, in, out, r, dt, freeze_mask)) return LRD_ERR_WORKSPACE;
    void* ws = scratch_on_current_device();
    if (!ws) return LRD_ERR_RUNTIME;
    return lrd_linear_bwd(dY, X, H, V, U, dX, dV, dU, dbias, freeze_mask, T, in, out, r, dt, ws, LRD_STATIC_SCRATCH_BYTES,
                          hip_stream);
}

// ------------------------------------------------------------------------------------ optimizer
lrd_status lrd_sgd_step(float* w_master, float* momentum_buf, const float* grad, void* w_copy, lrd_dtype copy_dt, int64_t n,
                        const lrd_sgd* opt, void* hip_stream)
{
    if (!w_master || !momentum_buf || !grad || !opt || n < 0 || !dtype_ok(copy_dt)) return LRD_ERR_INVALID_ARG;
    if (!(opt->lr >= 0.f) || !(opt->momentum >= 0.f) || !(opt->weight_decay >= 0.f)) return LRD_ERR_INVALID_ARG;
    LRD_TRY(sgd_step(w_master, momentum_buf, grad, w_copy, copy_dt == LRD_BF16, n, opt->lr, opt->momentum, opt->weight_decay,
                     (hipStream_t)hip_stream));
    return LRD_OK;
}

size_t lrd_linear_sgd_workspace_bytes(int64_t T, int64_t in, int64_t out, int64_t r, lrd_dtype dt, uint32_t freeze_mask)
{
    const size_t base = lrd_linear_workspace_bytes(T, in, out, r, dt, freeze_mask);
    if (!dtype_ok(dt) || !linear_dims_ok(T, in, out, r)) return 0;
    return base + round256((size_t)out * r * 4) + round256((size_t)r * in * 4);
}

lrd_status lrd_linear_bwd_sgd(const void* dY, const void* X, const void* H, void* V, void* U, void* dX, float* V_master,
                              float* U_master, float* V_momentum, float* U_momentum, float* dbias, uint32_t freeze_mask,
                              const void* Z_in, int32_t act, const lrd_sgd* opt, int64_t T, int64_t in, int64_t out, int64_t r,
                              lrd_dtype dt, void* ws, size_t ws_bytes, void* hip_stream)
{
    if (!dtype_ok(dt) || !linear_dims_ok(T, in, out, r) || !opt) return LRD_ERR_INVALID_ARG;
    if (freeze_mask & ~uint32_t(LRD_FREEZE_L0 | LRD_FREEZE_L1)) return LRD_ERR_INVALID_ARG;
    if (!(opt->lr >= 0.f) || !(opt->momentum >= 0.f) || !(opt->weight_decay >= 0.f)) return LRD_ERR_INVALID_ARG;
    const bool train_v = !(freeze_mask & LRD_FREEZE_L0), train_u = !(freeze_mask & LRD_FREEZE_L1);
    if (train_v && (!V_master || !V_momentum)) return LRD_ERR_INVALID_ARG;
    if (train_u && (!U_master || !U_momentum)) return LRD_ERR_INVALID_ARG;
    if (!aligned16(ws)) return LRD_ERR_ALIGNMENT;
    // the gradients of the trainable factors live in the workspace and never reach the caller
    Carver cv(ws, ws_bytes);
    float* dU = train_u ? (float*)cv.take((size_t)out * r * 4) : nullptr;
    float* dV = train_v ? (float*)cv.take((size_t)r * in * 4) : nullptr;
    if (!cv.ok) return LRD_ERR_WORKSPACE;
    if (pads_rank(in, out, r, dt)) {
        // padded ranks: the gradients are cropped to the caller's rank before the steps
        lrd_status rc = lrd_linear_bwd_act(dY, X, H, V, U, dX, dV, dU, dbias, freeze_mask, Z_in, act, T, in, out, r, dt,
                                           (char*)ws + cv.used, ws_bytes - cv.used, hip_stream);
        if (rc != LRD_OK) return rc;
        hipStream_t st = (hipStream_t)hip_stream;
        if (train_u) LRD_TRY(sgd_step(U_master, U_momentum, dU, U, true, out * r, opt->lr, opt->momentum, opt->weight_decay, st));
        if (train_v) LRD_TRY(sgd_step(V_master, V_momentum, dV, V, true, r * in, opt->lr, opt->momentum, opt->weight_decay, st));
        return LRD_OK;
    }
    // Each step is applied where its gradient is finished: in the sum over the split-K slices (the
    // gradient itself is then never stored), else by a kernel right after the product.  Both weight
    // gradients come after every product that reads V or U, and dV does not read U.
    SgdFuse su, sv;
    su.w = U_master; su.m = U_momentum; su.copy = U;
    sv.w = V_master; sv.m = V_momentum; sv.copy = V;
    su.copy_bf16 = sv.copy_bf16 = dt == LRD_BF16;
    su.lr = sv.lr = opt->lr; su.mu = sv.mu = opt->momentum; su.wd = sv.wd = opt->weight_decay;
    return linear_bwd_impl(dY, X, H, V, U, dX, dV, dU, dbias, freeze_mask, Z_in, act, T, in, out, r, dt, (char*)ws + cv.used,
                           ws_bytes - cv.used, hip_stream, train_u ? &su : nullptr, train_v ? &sv : nullptr);
}

// ------------------------------------------------------------------------------------ grouped linear
// G decomposed layers of equal shape reading the same input (the query / key / value projections of
// an attention block): their first factors are stacked into one [G*r x in] matrix, so the G
// products with X become one product of width G*r and the G data gradients one product of depth
// G*r; the second factors stay separate and address their r columns of the stacked intermediate
// through its leading dimension.
namespace {
inline bool group_dims_ok(int64_t T, int64_t in, int64_t out, int64_t r, int32_t groups)
{
    return groups >= 1 && groups <= 64 && linear_dims_ok(T, in, out, r) && (int64_t)groups * r < (int64_t(1) << 24);
}
inline const char* at(const void* p, int64_t elems, lrd_dtype dt) { return (const char*)p + elems * (int64_t)esize(dt); }

size_t group_partial_region(int64_t T, int64_t in, int64_t out, int64_t r, int32_t G, lrd_dtype dt, bool backward)
{
    const size_t h = act_partial_bytes(T, G * r, in, dt);
    if (!backward) return h;
    // the groups' second-factor gradients are one batched product: G sets of slices side by side
    return std::max(std::max(h, act_partial_bytes(T, r, out, dt)),
                    std::max((size_t)G * partial_bytes(out, r, T, dt), partial_bytes(G * r, in, T, dt)));
}
}  // namespace

size_t lrd_linear_group_workspace_bytes(int64_t T, int64_t in, int64_t out, int64_t r, int32_t groups, lrd_dtype dt,
                                        uint32_t freeze_mask)
{
    (void)freeze_mask;
    if (!dtype_ok(dt) || !group_dims_ok(T, in, out, r, groups)) return 0;
    const size_t act = round256((size_t)T * (size_t)groups * (size_t)r * esize(dt));
    const size_t fwd = act + group_partial_region(T, in, out, r, groups, dt, false);
    const size_t bwd = 2 * act + group_partial_region(T, in, out, r, groups, dt, true);
    return std::max(fwd, bwd);
}

lrd_status lrd_linear_group_fwd(const void* X, const void* V_cat, const void* U, const float* bias, void* Y, void* H_save,
                                int64_t T, int64_t in, int64_t out, int64_t r, int32_t groups, lrd_dtype dt, void* ws,
                                size_t ws_bytes, void* hip_stream)
{
    if (!dtype_ok(dt) || !group_dims_ok(T, in, out, r, groups) || !X || !V_cat || !U || !Y) return LRD_ERR_INVALID_ARG;
    if (!aligned16(X) || !aligned16(V_cat) || !aligned16(U) || !aligned16(Y) || !aligned16(H_save) || !aligned16(ws) ||
        !aligned16(bias))
        return LRD_ERR_ALIGNMENT;
    hipStream_t st = (hipStream_t)hip_stream;
    const int64_t gr = (int64_t)groups * r;
    Carver cv(ws, ws_bytes);
    void* H = H_save ? H_save : cv.take((size_t)T * gr * esize(dt));
    const size_t region_bytes = group_partial_region(T, in, out, r, groups, dt, false);
    void* region = region_bytes ? cv.take(region_bytes) : nullptr;
    if (!H || !cv.ok) return LRD_ERR_WORKSPACE;
    MatOp g1 = nt(X, in, V_cat, in, H, gr, T, gr, in, dt, false);
    g1.role = LRD_ROLE_FWD_DOWN;
    share_splits(g1, region, dt, SPLIT_ACT);
    LRD_TRY(run_matop(g1, st));
    // the groups' second products, one launch: group g reads columns g*r.. of H and its own U, writes its own Y
    MatOp g2 = nt(H, gr, U, r, Y, out, T, out, r, dt, false);
    g2.bias = bias;
    g2.role = LRD_ROLE_FWD_UP;
    g2.batch = groups;
    g2.a_bs = r; g2.b_bs = out * r; g2.c_bs = T * out; g2.bias_bs = out;
    LRD_TRY(run_matop(g2, st));
    return LRD_OK;
}

lrd_status lrd_linear_group_bwd(const void* dY, const void* X, const void* H, const void* V_cat, const void* U, void* dX,
                                float* dV_cat, float* dU, float* dbias, uint32_t freeze_mask, int64_t T, int64_t in, int64_t out,
                                int64_t r, int32_t groups, lrd_dtype dt, void* ws, size_t ws_bytes, void* hip_stream)
{
    if (!dtype_ok(dt) || !group_dims_ok(T, in, out, r, groups) || !dY || !V_cat || !U) return LRD_ERR_INVALID_ARG;
    if (freeze_mask & ~uint32_t(LRD_FREEZE_L0 | LRD_FREEZE_L1)) return LRD_ERR_INVALID_ARG;
    const bool train_v = !(freeze_mask & LRD_FREEZE_L0), train_u = !(freeze_mask & LRD_FREEZE_L1);
    if (train_v && (!dV_cat || !X)) return LRD_ERR_INVALID_ARG;
    if (train_u && (!dU || (!H && !X))) return LRD_ERR_INVALID_ARG;
    if (!aligned16(dY) || !aligned16(X) || !aligned16(H) || !aligned16(V_cat) || !aligned16(U) || !aligned16(dX) ||
        !aligned16(ws) || (train_v && !aligned16(dV_cat)) || (train_u && !aligned16(dU)) || !aligned16(dbias))
        return LRD_ERR_ALIGNMENT;
    hipStream_t st = (hipStream_t)hip_stream;
    const int64_t gr = (int64_t)groups * r;
    Carver cv(ws, ws_bytes);
    const size_t act_bytes = (size_t)T * gr * esize(dt);
    const bool need_dH = dX || train_v;
    void* dH = need_dH ? cv.take(act_bytes) : nullptr;
    void* Hre = (train_u && !H) ? cv.take(act_bytes) : nullptr;
    const size_t region_bytes = group_partial_region(T, in, out, r, groups, dt, true);
    void* region = region_bytes ? cv.take(region_bytes) : nullptr;
    if (!cv.ok) return LRD_ERR_WORKSPACE;

    if (need_dH) {
        if (choose_splits_act(T, r, out, dt == LRD_BF16) > 1) {
            // few tokens: each group's product is sliced along K and summed into its columns of dH
            for (int32_t g = 0; g < groups; ++g) {
                MatOp d1 = nn(at(dY, (int64_t)g * T * out, dt), out, at(U, (int64_t)g * out * r, dt), r, (void*)at(dH, g * r, dt), gr,
                              T, r, out, dt);
                d1.role = LRD_ROLE_DGRAD_UP;
                share_splits(d1, region, dt, SPLIT_ACT);
                LRD_TRY(run_matop(d1, st));
            }
        } else {
            MatOp d1 = nn(dY, out, U, r, dH, gr, T, r, out, dt);
            d1.role = LRD_ROLE_DGRAD_UP;
            d1.batch = groups;
            d1.a_bs = T * out; d1.b_bs = out * r; d1.c_bs = r;
            LRD_TRY(run_matop(d1, st));
        }
        if (dX) {
            MatOp d2 = nn(dH, gr, V_cat, in, dX, in, T, in, gr, dt);
            d2.role = LRD_ROLE_DGRAD_DOWN;
            LRD_TRY(run_matop(d2, st));
        }
    }
    if (train_u) {
        const void* Hs = H;
        if (!H) {
            MatOp re = nt(X, in, V_cat, in, Hre, gr, T, gr, in, dt, false);
            share_splits(re, region, dt, SPLIT_ACT);
            LRD_TRY(run_matop(re, st));
            Hs = Hre;
        }
        // one launch for the groups' gradients: group g contracts its dY with its columns of H
        MatOp wu = tn(dY, out, Hs, gr, dU, r, out, r, T, dt);
        wu.role = LRD_ROLE_WGRAD_U;
        wu.batch = groups;
        wu.a_bs = T * out; wu.b_bs = r; wu.c_bs = out * r;
        share_splits(wu, region, dt, SPLIT_WGRAD);
        LRD_TRY(run_matop(wu, st));
    }
    if (train_v) {
        MatOp wv = tn(dH, gr, X, in, dV_cat, in, gr, in, T, dt);
        wv.role = LRD_ROLE_WGRAD_V;
        share_splits(wv, region, dt, SPLIT_WGRAD);
        LRD_TRY(run_matop(wv, st));
    }
    if (dbias)
        for (int32_t g = 0; g < groups; ++g)
            LRD_TRY(column_sums(at(dY, (int64_t)g * T * out, dt), dbias + (int64_t)g * out, T, out, dt == LRD_BF16, st));
    return LRD_OK;
}

// ------------------------------------------------------------------------------------ deferred weight gradients
lrd_status lrd_linear_bwd_data(const void* dY, const void* V, const void* U, void* dX, void* dH_save, const void* Z_in,
                               int32_t act, int64_t T, int64_t in, int64_t out, int64_t r, lrd_dtype dt, void* ws,
                               size_t ws_bytes, void* hip_stream)
{
    if (!dtype_ok(dt) || !linear_dims_ok(T, in, out, r) || !dY || !V || !U || !dH_save) return LRD_ERR_INVALID_ARG;
    if ((act != LRD_ACT_NONE && act != LRD_ACT_GELU) || (act == LRD_ACT_GELU && dX && !Z_in)) return LRD_ERR_INVALID_ARG;
    if (act == LRD_ACT_NONE || !dX) Z_in = nullptr;
    if (!aligned16(dY) || !aligned16(V) || !aligned16(U) || !aligned16(dX) || !aligned16(dH_save) || !aligned16(Z_in) ||
        !aligned16(ws))
        return LRD_ERR_ALIGNMENT;
    hipStream_t st = (hipStream_t)hip_stream;
    Carver cv(ws, ws_bytes);
    const size_t region_bytes = act_partial_bytes(T, r, out, dt);
    void* region = region_bytes ? cv.take(region_bytes) : nullptr;
    if (!cv.ok) return LRD_ERR_WORKSPACE;
    MatOp d1 = nn(dY, out, U, r, dH_save, r, T, r, out, dt);
    d1.role = LRD_ROLE_DGRAD_UP;
    share_splits(d1, region, dt, SPLIT_ACT);
    LRD_TRY(run_matop(d1, st));
    if (!dX) return LRD_OK;
    MatOp d2 = nn(dH_save, r, V, in, dX, in, T, in, r, dt);
    d2.role = LRD_ROLE_DGRAD_DOWN;
    if (Z_in) {      // engines that do not fuse the epilogue run it as a pass of its own (run_matop)
        d2.epilogue = EPI_ACT_GRAD;
        d2.aux = const_cast<void*>(Z_in);
        d2.ldaux = in;
    }
    LRD_TRY(run_matop(d2, st));
    return LRD_OK;
}

lrd_status lrd_linear_group_bwd_data(const void* dY, const void* V_cat, const void* U, void* dX, void* dH_save, int64_t T,
                                     int64_t in, int64_t out, int64_t r, int32_t groups, lrd_dtype dt, void* ws,
                                     size_t ws_bytes, void* hip_stream)
{
    if (!dtype_ok(dt) || !group_dims_ok(T, in, out, r, groups) || !dY || !V_cat || !U || !dH_save) return LRD_ERR_INVALID_ARG;
    if (!aligned16(dY) || !aligned16(V_cat) || !aligned16(U) || !aligned16(dX) || !aligned16(dH_save) || !aligned16(ws))
        return LRD_ERR_ALIGNMENT;
    hipStream_t st = (hipStream_t)hip_stream;
    const int64_t gr = (int64_t)groups * r;
    Carver cv(ws, ws_bytes);
    const size_t region_bytes = act_partial_bytes(T, r, out, dt);
    void* region = region_bytes ? cv.take(region_bytes) : nullptr;
    if (!cv.ok) return LRD_ERR_WORKSPACE;
    if (choose_splits_act(T, r, out, dt == LRD_BF16) > 1) {
        for (int32_t g = 0; g < groups; ++g) {
            MatOp d1 = nn(at(dY, (int64_t)g * T * out, dt), out, at(U, (int64_t)g * out * r, dt), r, (void*)at(dH_save, g * r, dt),
                          gr, T, r, out, dt);
            d1.role = LRD_ROLE_DGRAD_UP;
            share_splits(d1, region, dt, SPLIT_ACT);
            LRD_TRY(run_matop(d1, st));
        }
    } else {
        MatOp d1 = nn(dY, out, U, r, dH_save, gr, T, r, out, dt);
        d1.role = LRD_ROLE_DGRAD_UP;
        d1.batch = groups;
        d1.a_bs = T * out; d1.b_bs = out * r; d1.c_bs = r;
        LRD_TRY(run_matop(d1, st));
    }
    if (dX) {
        MatOp d2 = nn(dH_save, gr, V_cat, in, dX, in, T, in, gr, dt);
        d2.role = LRD_ROLE_DGRAD_DOWN;
        LRD_TRY(run_matop(d2, st));
    }
    return LRD_OK;
}

namespace {
inline bool wgrad_batched_dims_ok(int64_t layers, int64_t T, int64_t in, int64_t out, int64_t r)
{
    return layers >= 1 && layers <= 1024 && T >= 1 && in >= 1 && out >= 1 && r >= 1 && T < (int64_t(1) << 31) &&
           in < (int64_t(1) << 24) && out < (int64_t(1) << 24) && r < (int64_t(1) << 24);
}
inline size_t batched_partial_bytes(int64_t M, int64_t N, int64_t K, int64_t batch)
{
    const int s = choose_splits_batched(M, N, K, batch);
    return s > 1 ? round256((size_t)s * (size_t)batch * (size_t)M * (size_t)N * sizeof(float)) : 0;
}
}  // namespace

size_t lrd_linear_wgrad_batched_workspace_bytes(int64_t layers, int64_t T, int64_t in, int64_t out, int64_t r, lrd_dtype dt,
                                                uint32_t freeze_mask)
{
    if (!dtype_ok(dt) || !wgrad_batched_dims_ok(layers, T, in, out, r)) return 0;
    size_t b = 0;
    if (!(freeze_mask & LRD_FREEZE_L1)) b = std::max(b, batched_partial_bytes(out, r, T, layers));
    if (!(freeze_mask & LRD_FREEZE_L0)) b = std::max(b, batched_partial_bytes(r, in, T, layers));
    return b;
}

lrd_status lrd_linear_wgrad_batched(const void* dY, int64_t dy_stride, const void* H, int64_t ldh, int64_t h_stride,
                                    const void* dH, int64_t lddh, int64_t dh_stride, const void* X, int64_t x_stride, float* dV,
                                    float* dU, uint32_t freeze_mask, int64_t layers, int64_t T, int64_t in, int64_t out, int64_t r,
                                    lrd_dtype dt, void* ws, size_t ws_bytes, void* hip_stream)
{
    if (!dtype_ok(dt) || !wgrad_batched_dims_ok(layers, T, in, out, r)) return LRD_ERR_INVALID_ARG;
    if (freeze_mask & ~uint32_t(LRD_FREEZE_L0 | LRD_FREEZE_L1)) return LRD_ERR_INVALID_ARG;
    const bool train_v = !(freeze_mask & LRD_FREEZE_L0), train_u = !(freeze_mask & LRD_FREEZE_L1);
    if (train_u && (!dY || !H || !dU || ldh < r || dy_stride % 8 || h_stride % 8 || dy_stride < 0 || h_stride < 0))
        return LRD_ERR_INVALID_ARG;
    if (train_v && (!dH || !X || !dV || lddh < r || dh_stride % 8 || x_stride % 8 || dh_stride < 0 || x_stride < 0))
        return LRD_ERR_INVALID_ARG;
    if (!aligned16(ws) || (train_u && (!aligned16(dY) || !aligned16(H) || !aligned16(dU))) ||
        (train_v && (!aligned16(dH) || !aligned16(X) || !aligned16(dV))))
        return LRD_ERR_ALIGNMENT;
    hipStream_t st = (hipStream_t)hip_stream;
    const size_t region_bytes = lrd_linear_wgrad_batched_workspace_bytes(layers, T, in, out, r, dt, freeze_mask);
    if (region_bytes > ws_bytes || (region_bytes && !ws)) return LRD_ERR_WORKSPACE;
    auto slice = [&](MatOp& op) {
        const int s = choose_splits_batched(op.M, op.N, op.K, layers);
        if (s > 1) {
            op.partial = (float*)ws;
            op.splits = s;
        }
    };
    if (train_u) {
        MatOp wu = tn(dY, out, H, ldh, dU, r, out, r, T, dt);
        wu.role = LRD_ROLE_WGRAD_U;
        wu.batch = (int)layers;
        wu.a_bs = dy_stride; wu.b_bs = h_stride; wu.c_bs = out * r;
        slice(wu);
        LRD_TRY(run_matop(wu, st));
    }
    if (train_v) {
        MatOp wv = tn(dH, lddh, X, in, dV, in, r, in, T, dt);
        wv.role = LRD_ROLE_WGRAD_V;
        wv.batch = (int)layers;
        wv.a_bs = dh_stride; wv.b_bs = x_stride; wv.c_bs = r * in;
        slice(wv);
        LRD_TRY(run_matop(wv, st));
    }
    return LRD_OK;
}

// ------------------------------------------------------------------------------------ dense linear
size_t lrd_dense_linear_workspace_bytes(int64_t T, int64_t in, int64_t out, lrd_dtype dt)
{
    if (!dtype_ok(dt) || T < 1 || in < 1 || out < 1) return 0;
    return partial_bytes(out, in, T, dt);
}

lrd_status lrd_dense_linear_fwd(const void* X, const void* W, const float* bias, void* Y, int64_t T,
                                int64_t in, int64_t out, lrd_dtype dt, void* ws, size_t ws_bytes,
                                void* hip_stream)
{
    (void)ws; (void)ws_bytes;
    if (!dtype_ok(dt) || !linear_dims_ok(T, in, out, 1) || !X || !W || !Y) return LRD_ERR_INVALID_ARG;
    if (!aligned16(X) || !aligned16(W) || !aligned16(Y) || !aligned16(bias)) return LRD_ERR_ALIGNMENT;
    MatOp g = nt(X, in, W, in, Y, out, T, out, in, dt, false);
    g.bias = bias;
    LRD_TRY(run_matop(g, (hipStream_t)hip_stream));
    return LRD_OK;
}

lrd_status lrd_dense_linear_bwd(const void* dY, const void* X, const void* W, void* dX, float* dW,
                                int64_t T, int64_t in, int64_t out, lrd_dtype dt, void* ws,
                                size_t ws_bytes, void* hip_stream)
{
    if (!dtype_ok(dt) || !linear_dims_ok(T, in, out, 1) || !dY || !W || (dW && !X)) return LRD_ERR_INVALID_ARG;
    if (!aligned16(dY) || !aligned16(X) || !aligned16(W) || !aligned16(dX) || !aligned16(dW) || !aligned16(ws))
        return LRD_ERR_ALIGNMENT;
    hipStream_t st = (hipStream_t)hip_stream;
    Carver cv(ws, ws_bytes);
    MatOp wg;
    if (dW) {
        wg = tn(dY, out, X, in, dW, in, out, in, T, dt);
        attach_splits(wg, cv, dt);
        if (!cv.ok) return LRD_ERR_WORKSPACE;
    }
    if (dX) LRD_TRY(run_matop(nn(dY, out, W, in, dX, in, T, in, out, dt), st));
    if (dW) LRD_TRY(run_matop(wg, st));
    return LRD_OK;
}

// ------------------------------------------------------------------------------------ Tucker conv
// Same rule for the Tucker triple: ranks that are not multiples of 8 run at the padded ranks on
// zero-padded copies of P1, G, P2 (and of saved A / B in the backward).
inline bool pads_tucker(const lrd_conv_geom& g, lrd_dtype dt)
{
    return dt == LRD_BF16 && (g.r1 % 8 != 0 || g.r2 % 8 != 0) && g.C % 8 == 0 && g.S % 8 == 0;
}

struct TuckerPads {
    lrd_conv_geom gp;
    size_t p1, gc, p2, a, b, dp1, dg, dp2;   // byte sizes of the padded copies
    size_t total() const { return p1 + gc + p2 + a + b + dp1 + dg + dp2; }
};

inline TuckerPads tucker_pads(const lrd_conv_geom& g)
{
    TuckerPads t;
    t.gp = g;
    t.gp.r1 = pad8(g.r1);
    t.gp.r2 = pad8(g.r2);
    ConvShape cs = core_shape(g, g.r1, g.r2);
    const size_t kk = (size_t)g.k * g.k, pin = (size_t)g.N * g.H * g.W, pout = (size_t)g.N * cs.Ho * cs.Wo;
    const size_t r1 = t.gp.r1, r2 = t.gp.r2;
    t.p1 = round256(r1 * g.C * 2);
    t.gc = round256(r2 * kk * r1 * 2);
    t.p2 = round256((size_t)g.S * r2 * 2);
    t.a = round256(pin * r1 * 2);
    t.b = round256(pout * r2 * 2);
    t.dp1 = round256(r1 * g.C * 4);
    t.dg = round256(r2 * kk * r1 * 4);
    t.dp2 = round256((size_t)g.S * r2 * 4);
    return t;
}

size_t lrd_tucker_conv_workspace_bytes(const lrd_conv_geom* g, lrd_dtype dt, uint32_t freeze_mask)
{
    (void)freeze_mask;
    if (!dtype_ok(dt) || !geom_ok(g, true)) return 0;
    if (pads_tucker(*g, dt)) {
        TuckerPads t = tucker_pads(*g);
        return t.total() + lrd_tucker_conv_workspace_bytes(&t.gp, dt, freeze_mask);
    }
    ConvShape cs = core_shape(*g, g->r1, g->r2);
    size_t pin = (size_t)g->N * g->H * g->W, pout = (size_t)g->N * cs.Ho * cs.Wo;
    size_t a = round256(pin * g->r1 * esize(dt)), b = round256(pout * g->r2 * esize(dt));
    size_t kk = (size_t)g->k * g->k;
    size_t part = std::max(std::max(partial_bytes(g->S, g->r2, pout, dt), partial_bytes(g->r2, kk * g->r1, pout, dt)),
                           partial_bytes(g->r1, g->C, pin, dt));
    part = std::max(part, round256(conv_direct_wgrad_bytes(cs, dt == LRD_BF16)));
    // forward: A and B when not side-stored; backward: dA, dB, recomputed A and B, partials, and the
    // flipped core weights of a stride-1 data gradient
    return 2 * (a + b) + part + round256(conv_dgrad_flip_bytes(cs, dt == LRD_BF16));
}

lrd_status lrd_tucker_conv_fwd(const void* X, const void* P1, const void* G, const void* P2,
                               void* Y, void* A_save, void* B_save, const lrd_conv_geom* g,
                               lrd_dtype dt, void* ws, size_t ws_bytes, void* hip_stream)
{
    if (!dtype_ok(dt) || !geom_ok(g, true) || !X || !P1 || !G || !P2 || !Y) return LRD_ERR_INVALID_ARG;
    if (!aligned16(X) || !aligned16(P1) || !aligned16(G) || !aligned16(P2) || !aligned16(Y) || !aligned16(A_save) ||
        !aligned16(B_save) || !aligned16(ws))
        return LRD_ERR_ALIGNMENT;
    hipStream_t st = (hipStream_t)hip_stream;
    ConvShape cs = core_shape(*g, g->r1, g->r2);
    const int64_t pin = g->N * g->H * g->W, pout = g->N * (int64_t)cs.Ho * cs.Wo;
    const int64_t kk = (int64_t)g->k * g->k;
    if (pads_tucker(*g, dt)) {
        TuckerPads t = tucker_pads(*g);
        const int64_t r1 = g->r1, r2 = g->r2, q1 = t.gp.r1, q2 = t.gp.r2;
        Carver cp(ws, ws_bytes);
        void* P1p = cp.take(t.p1);
        void* Gp = cp.take(t.gc);
        void* P2p = cp.take(t.p2);
        void* Ap = cp.take(t.a);
        void* Bp = cp.take(t.b);
        if (!cp.ok) return LRD_ERR_WORKSPACE;
        LRD_TRY(copy2d(P1, g->C, r1, g->C, P1p, g->C, q1, g->C, 2, st));
        LRD_TRY(copy2d(G, r1, r2 * kk, r1, Gp, q1, q2 * kk, q1, 2, st));
        LRD_TRY(copy2d(P2, r2, g->S, r2, P2p, q2, g->S, q2, 2, st));
        lrd_status rc = lrd_tucker_conv_fwd(X, P1p, Gp, P2p, Y, Ap, Bp, &t.gp, dt, (char*)ws + cp.used, ws_bytes - cp.used,
                                            hip_stream);
        if (rc != LRD_OK) return rc;
        if (A_save) LRD_TRY(copy2d(Ap, q1, pin, r1, A_save, r1, pin, r1, 2, st));
        if (B_save) LRD_TRY(copy2d(Bp, q2, pout, r2, B_save, r2, pout, r2, 2, st));
        return LRD_OK;
    }
    Carver cv(ws, ws_bytes);
    void* A = A_save ? A_save : cv.take((size_t)pin * g->r1 * esize(dt));
    void* B = B_save ? B_save : cv.take((size_t)pout * g->r2 * esize(dt));
    if (!A || !B) return LRD_ERR_WORKSPACE;

    LRD_TRY(run_matop(nt(X, g->C, P1, g->C, A, g->r1, pin, g->r1, g->C, dt, false), st));
    MatOp core = nt(A, g->r1, G, kk * g->r1, B, g->r2, pout, g->r2, kk * g->r1, dt, false);
    core.gather = GATHER_CONV_FWD;
    core.cs = cs;
    LRD_TRY(run_matop(core, st));
    LRD_TRY(run_matop(nt(B, g->r2, P2, g->r2, Y, g->S, pout, g->S, g->r2, dt, false), st));
    return LRD_OK;
}

lrd_status lrd_tucker_conv_bwd(const void* dY, const void* X, const void* A, const void* B,
                               const void* P1, const void* G, const void* P2, void* dX,
                               float* dP1, float* dG, float* dP2, uint32_t freeze_mask,
                               const lrd_conv_geom* g, lrd_dtype dt, void* ws, size_t ws_bytes,
                               void* hip_stream)
{
    if (!dtype_ok(dt) || !geom_ok(g, true) || !dY || !P1 || !G || !P2) return LRD_ERR_INVALID_ARG;
    if (freeze_mask & ~uint32_t(LRD_FREEZE_L0 | LRD_FREEZE_L1 | LRD_FREEZE_L2)) return LRD_ERR_INVALID_ARG;
    const bool t1 = !(freeze_mask & LRD_FREEZE_L0), tg = !(freeze_mask & LRD_FREEZE_L1),
               t2 = !(freeze_mask & LRD_FREEZE_L2);
    if ((t1 && (!dP1 || !X)) || (tg && !dG) || (t2 && !dP2)) return LRD_ERR_INVALID_ARG;
    const bool need_A = tg || (t2 && !B);            // A feeds dG, and B's recomputation
    if (((need_A && !A) || (t2 && !B)) && !X) return LRD_ERR_INVALID_ARG;
    if (!aligned16(dY) || !aligned16(X) || !aligned16(A) || !aligned16(B) || !aligned16(P1) || !aligned16(G) ||
        !aligned16(P2) || !aligned16(dX) || !aligned16(ws) || (t1 && !aligned16(dP1)) || (tg && !aligned16(dG)) ||
        (t2 && !aligned16(dP2)))
        return LRD_ERR_ALIGNMENT;
    hipStream_t st = (hipStream_t)hip_stream;
    ConvShape cs = core_shape(*g, g->r1, g->r2);
    const int64_t pin = g->N * g->H * g->W, pout = g->N * (int64_t)cs.Ho * cs.Wo;
    const int64_t kk = (int64_t)g->k * g->k;
    const int64_t r1 = g->r1, r2 = g->r2, C = g->C, S = g->S;
    if (pads_tucker(*g, dt)) {
        TuckerPads t = tucker_pads(*g);
        const int64_t q1 = t.gp.r1, q2 = t.gp.r2;
        Carver cp(ws, ws_bytes);
        void* P1p = cp.take(t.p1);
        void* Gp = cp.take(t.gc);
        void* P2p = cp.take(t.p2);
        void* Ap = cp.take(t.a);
        void* Bp = cp.take(t.b);
        float* dP1p = (float*)cp.take(t.dp1);
        float* dGp = (float*)cp.take(t.dg);
        float* dP2p = (float*)cp.take(t.dp2);
        if (!cp.ok) return LRD_ERR_WORKSPACE;
        LRD_TRY(copy2d(P1, C, r1, C, P1p, C, q1, C, 2, st));
        LRD_TRY(copy2d(G, r1, r2 * kk, r1, Gp, q1, q2 * kk, q1, 2, st));
        LRD_TRY(copy2d(P2, r2, S, r2, P2p, q2, S, q2, 2, st));
        const bool have_a = A && need_A, have_b = B && t2;
        if (have_a) LRD_TRY(copy2d(A, r1, pin, r1, Ap, q1, pin, q1, 2, st));
        if (have_b) LRD_TRY(copy2d(B, r2, pout, r2, Bp, q2, pout, q2, 2, st));
        lrd_status rc = lrd_tucker_conv_bwd(dY, X, have_a ? Ap : nullptr, have_b ? Bp : nullptr, P1p, Gp, P2p, dX, dP1p, dGp,
                                            dP2p, freeze_mask, &t.gp, dt, (char*)ws + cp.used, ws_bytes - cp.used,
                                            hip_stream);
        if (rc != LRD_OK) return rc;
        if (t1) LRD_TRY(copy2d(dP1p, C, r1, C, dP1, C, r1, C, 4, st));
        if (tg) LRD_TRY(copy2d(dGp, q1, r2 * kk, r1, dG, r1, r2 * kk, r1, 4, st));
        if (t2) LRD_TRY(copy2d(dP2p, q2, S, r2, dP2, r2, S, r2, 4, st));
        return LRD_OK;
    }
    Carver cv(ws, ws_bytes);
    const bool need_dA = dX || t1;
    const bool need_dB = need_dA || tg;

    void* dB = need_dB ? cv.take((size_t)pout * r2 * esize(dt)) : nullptr;
    void* dA = need_dA ? cv.take((size_t)pin * r1 * esize(dt)) : nullptr;
    void* Are = (need_A && !A) ? cv.take((size_t)pin * r1 * esize(dt)) : nullptr;
    void* Bre = (t2 && !B) ? cv.take((size_t)pout * r2 * esize(dt)) : nullptr;
    const void* Ause = A ? A : Are;
    const void* Buse = B ? B : Bre;
    MatOp w2, wg, w1;
    float* shared_partial = nullptr;
    size_t shared_bytes = 0;
    auto splits_for = [&](MatOp& op) {
        int s = choose_splits(op.M, op.N, op.K, dt == LRD_BF16);
        if (s <= 1) return;
        size_t need = (size_t)s * op.M * op.N * sizeof(float);
        if (need > shared_bytes) return;
        op.partial = shared_partial; op.splits = s;
    };
    if (t2) w2 = tn(dY, S, Buse, r2, dP2, r2, S, r2, pout, dt);
    if (tg) {
        wg = tn(dB, r2, Ause, r1, dG, kk * r1, r2, kk * r1, pout, dt);
        wg.gather = GATHER_CONV_WGRAD;
        wg.cs = cs;
    }
    if (t1) w1 = tn(dA, r1, X, C, dP1, C, r1, C, pin, dt);
    // one partial buffer, sized for the largest of the three products, used by them in turn
    shared_bytes = std::max(std::max(t2 ? partial_bytes(S, r2, pout, dt) : 0, tg ? partial_bytes(r2, kk * r1, pout, dt) : 0),
                            t1 ? partial_bytes(r1, C, pin, dt) : 0);
    if (tg) shared_bytes = std::max(shared_bytes, round256(conv_direct_wgrad_bytes(cs, dt == LRD_BF16)));
    if (shared_bytes) shared_partial = (float*)cv.take(shared_bytes);
    const size_t flip_bytes = need_dA ? conv_dgrad_flip_bytes(cs, dt == LRD_BF16) : 0;
    void* flip = flip_bytes ? cv.take(flip_bytes) : nullptr;
    if (!cv.ok) return LRD_ERR_WORKSPACE;
    if (t2) splits_for(w2);
    if (tg) {
        splits_for(wg);
        wg.scratch = shared_partial;
        wg.scratch_bytes = shared_bytes;
    }
    if (t1) splits_for(w1);

    if (need_dB) LRD_TRY(run_matop(nn(dY, S, P2, r2, dB, r2, pout, r2, S, dt), st));
    if (need_dA) {
        MatOp dg = nt(dB, r2, G, 0, dA, r1, pin, r1, kk * r2, dt, false);
        dg.gather = GATHER_CONV_DGRAD;
        dg.cs = cs;
        dg.scratch = flip;
        dg.scratch_bytes = flip_bytes;
        LRD_TRY(run_matop(dg, st));
    }
    if (dX) LRD_TRY(run_matop(nn(dA, r1, P1, C, dX, C, pin, C, r1, dt), st));
    if (Are) LRD_TRY(run_matop(nt(X, C, P1, C, Are, r1, pin, r1, C, dt, false), st));
    if (Bre) {
        MatOp core = nt(Ause, r1, G, kk * r1, Bre, r2, pout, r2, kk * r1, dt, false);
        core.gather = GATHER_CONV_FWD;
        core.cs = cs;
        LRD_TRY(run_matop(core, st));
    }
    if (t2) LRD_TRY(run_matop(w2, st));
    if (tg) LRD_TRY(run_matop(wg, st));
    if (t1) LRD_TRY(run_matop(w1, st));
    return LRD_OK;
}

// ------------------------------------------------------------------------------------ dense conv
size_t lrd_dense_conv_workspace_bytes(const lrd_conv_geom* g, lrd_dtype dt)
{
    if (!dtype_ok(dt) || !geom_ok(g, false)) return 0;
    ConvShape cs = core_shape(*g, g->C, g->S);
    return std::max(partial_bytes(g->S, (int64_t)g->k * g->k * g->C, g->N * (int64_t)cs.Ho * cs.Wo, dt),
                    round256(conv_direct_wgrad_bytes(cs, dt == LRD_BF16))) +
           round256(conv_dgrad_flip_bytes(cs, dt == LRD_BF16));
}

lrd_status lrd_dense_conv_fwd(const void* X, const void* W, void* Y, const lrd_conv_geom* g,
                              lrd_dtype dt, void* ws, size_t ws_bytes, void* hip_stream)
{
    (void)ws; (void)ws_bytes;
    if (!dtype_ok(dt) || !geom_ok(g, false) || !X || !W || !Y) return LRD_ERR_INVALID_ARG;
    if (!aligned16(X) || !aligned16(W) || !aligned16(Y)) return LRD_ERR_ALIGNMENT;
    ConvShape cs = core_shape(*g, g->C, g->S);
    const int64_t pout = g->N * (int64_t)cs.Ho * cs.Wo, K = (int64_t)g->k * g->k * g->C;
    MatOp op = nt(X, g->C, W, K, Y, g->S, pout, g->S, K, dt, false);
    op.gather = GATHER_CONV_FWD;
    op.cs = cs;
    LRD_TRY(run_matop(op, (hipStream_t)hip_stream));
    return LRD_OK;
}

lrd_status lrd_dense_conv_bwd(const void* dY, const void* X, const void* W, void* dX, float* dW,
                              const lrd_conv_geom* g, lrd_dtype dt, void* ws, size_t ws_bytes,
                              void* hip_stream)
{
    if (!dtype_ok(dt) || !geom_ok(g, false) || !dY || !W || (dW && !X)) return LRD_ERR_INVALID_ARG;
    if (!aligned16(dY) || !aligned16(X) || !aligned16(W) || !aligned16(dX) || !aligned16(dW) || !aligned16(ws))
        return LRD_ERR_ALIGNMENT;
    hipStream_t st = (hipStream_t)hip_stream;
    ConvShape cs = core_shape(*g, g->C, g->S);
    const int64_t pin = g->N * g->H * g->W, pout = g->N * (int64_t)cs.Ho * cs.Wo;
    const int64_t kk = (int64_t)g->k * g->k;
    Carver cv(ws, ws_bytes);
    MatOp wg;
    if (dW) {
        wg = tn(dY, g->S, X, g->C, dW, kk * g->C, g->S, kk * g->C, pout, dt);
        wg.gather = GATHER_CONV_WGRAD;
        wg.cs = cs;
        // the workgroup partials of the direct kernel, or split-K slices, in the same region
        const size_t direct = conv_direct_wgrad_bytes(cs, dt == LRD_BF16);
        if (direct) {
            wg.scratch = cv.take(direct);
            wg.scratch_bytes = direct;
        } else {
            attach_splits(wg, cv, dt);
        }
        if (!cv.ok) return LRD_ERR_WORKSPACE;
    }
    if (dX) {
        MatOp dg = nt(dY, g->S, W, 0, dX, g->C, pin, g->C, kk * g->S, dt, false);
        dg.gather = GATHER_CONV_DGRAD;
        dg.cs = cs;
        dg.scratch_bytes = conv_dgrad_flip_bytes(cs, dt == LRD_BF16);
        dg.scratch = dg.scratch_bytes ? cv.take(dg.scratch_bytes) : nullptr;
        if (!cv.ok) return LRD_ERR_WORKSPACE;
        LRD_TRY(run_matop(dg, st));
    }
    if (dW) LRD_TRY(run_matop(wg, st));
    return LRD_OK;
}

// ------------------------------------------------------------------------------------ glue
lrd_status lrd_gelu_fwd(const void* Z, void* A, int64_t n, lrd_dtype dt, void* hip_stream)
{
    if (!dtype_ok(dt) || n < 0 || !Z || !A) return LRD_ERR_INVALID_ARG;
    if (!aligned16(Z) || !aligned16(A)) return LRD_ERR_ALIGNMENT;
    LRD_TRY(gelu_fwd(Z, A, n, dt == LRD_BF16, (hipStream_t)hip_stream));
    return LRD_OK;
}

lrd_status lrd_gelu_bwd(const void* dA, const void* Z, void* dZ, int64_t n, lrd_dtype dt,
                        void* hip_stream)
{
    if (!dtype_ok(dt) || n < 0 || !dA || !Z || !dZ) return LRD_ERR_INVALID_ARG;
    if (!aligned16(dA) || !aligned16(Z) || !aligned16(dZ)) return LRD_ERR_ALIGNMENT;
    LRD_TRY(gelu_bwd(dA, Z, dZ, n, dt == LRD_BF16, (hipStream_t)hip_stream));
    return LRD_OK;
}

}  // extern "C"
