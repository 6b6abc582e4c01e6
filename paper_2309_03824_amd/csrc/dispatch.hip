// Engine selection for a single matrix product and the split-K policy.
#include <atomic>
#include <cstdio>
#include <mutex>
#include <vector>

#include "lrd_internal.hpp"
#include "lrd_measure.h"

namespace lrd {

// Weight-gradient products have a long K (tokens or pixels) and a small output; K is cut into
// slices so that the launch has enough workgroups to fill 256 compute units about twice over.
// Measured with cold operands at K = 8192 (kernel plus reduce): a 3072 x 192 gradient is fastest
// with 128 x 128 tiles and 10 slices (480 workgroups), a 768 x 192 one with 64 x 64 tiles and
// 12 slices (432); more slices only add partial-sum traffic.  The count depends only on the
// shape, so workspace queries and launches agree; the kernel launcher picks the tile from the
// resulting workgroup count.
int choose_splits(int64_t M, int64_t N, int64_t K, bool in_bf16)
{
    (void)in_bf16;
    const int64_t t128 = ceil_div(M, 128) * ceil_div(N, 128);
    const int64_t t64 = ceil_div(M, 64) * ceil_div(N, 64);
    int64_t s = t128 >= 24 ? ceil_div(480, t128) : ceil_div(432, t64);
    const int64_t by_k = K / 256;          // keep at least 256 reduction steps per slice
    if (s > by_k) s = by_k;
    if (s > 512) s = 512;
    return s < 2 ? 1 : (int)s;
}

// Products whose result is a [tokens x r] activation (H = X.V^T, dH = dY.U) have few output tiles
// when r is small and a long K when the wide side of the layer is the reduction.  While 64 x 64
// tiles still give every compute unit a workgroup (T = 8192, r = 192: 384 of them) the unsplit
// kernel is as fast as any split plus its reduce (27.7 us against 25.6-29 us at K = 3072, cold
// operands), so K is cut only below that, down to slices of 768.
int choose_splits_act(int64_t M, int64_t N, int64_t K, bool in_bf16)
{
    if (!in_bf16 || N % 8 != 0) return 1;           // only the aligned MFMA path reduces into bf16
    const int64_t t64 = ceil_div(M, 64) * ceil_div(N, 64);
    if (t64 >= 256) return 1;
    int64_t s = ceil_div(512, t64);
    const int64_t by_k = K / 768;
    if (s > by_k) s = by_k;
    if (s > 8) s = 8;
    return s < 2 ? 1 : (int)s;
}

// Weight gradients of `batch` layers of one shape in one launch.  256 x 256 tiles over all members
// already give most compute units a workgroup when there are a dozen layers; K is sliced only while
// they do not (12 x [1024 x 256] over 8192 tokens: 203 us unsliced, 78 us in 4 slices; 36 members:
// 213 us unsliced, 283 us in 2 slices).
int choose_splits_batched(int64_t M, int64_t N, int64_t K, int64_t batch)
{
    const int64_t tiles = ceil_div(M, 256) * ceil_div(N, 256) * batch;
    int64_t s = 224 / tiles;
    const int64_t by_k = K / 512;
    if (s > by_k) s = by_k;
    if (s > 64) s = 64;
    return s < 2 ? 1 : (int)s;
}

namespace {
std::mutex g_log_mutex;
std::atomic<bool> g_log_on{false};
void** g_log_events = nullptr;
int g_log_pairs = 0;
std::vector<lrd_profile_record> g_log;
thread_local const char* t_kernel = "";
}  // namespace

void note_kernel(const char* name) { t_kernel = name; }

int log_begin(hipEvent_t* start, hipEvent_t* stop)
{
    if (!g_log_on.load(std::memory_order_relaxed)) return -1;
    std::lock_guard<std::mutex> lock(g_log_mutex);
    if (!g_log_on.load() || (int)g_log.size() >= g_log_pairs) return -1;
    const int i = (int)g_log.size();
    g_log.push_back(lrd_profile_record{});
    *start = (hipEvent_t)g_log_events[2 * i];
    *stop = (hipEvent_t)g_log_events[2 * i + 1];
    t_kernel = "";
    return i;
}

void log_end(int index, int role, int gather, int epilogue, int splits, int64_t M, int64_t N, int64_t K, int64_t batch)
{
    std::lock_guard<std::mutex> lock(g_log_mutex);
    if (index < 0 || index >= (int)g_log.size()) return;
    lrd_profile_record& r = g_log[index];
    r.role = role; r.gather = gather; r.epilogue = epilogue; r.splits = splits;
    r.M = M; r.N = N; r.K = K; r.batch = batch;
    snprintf(r.kernel, sizeof(r.kernel), "%s", t_kernel);
}

// The activation epilogue as separate elementwise passes, for engines that do not fuse it.
// C and aux are dense [M x N] here (ldc = ldaux = N), which is all the layer passes produce.
hipError_t apply_epilogue(const MatOp& op, hipStream_t st)
{
    if (op.ldc != op.N || op.ldaux != op.N) return hipErrorInvalidValue;
    const int64_t n = op.M * op.N;
    if (op.epilogue == EPI_ACT_STORE) return gelu_fwd(op.C, op.aux, n, op.in_bf16, st);
    if (op.epilogue == EPI_ACT_GRAD) return gelu_bwd(op.C, op.aux, op.C, n, op.in_bf16, st);
    return hipSuccess;
}

size_t conv_dgrad_flip_bytes(const ConvShape& cs, bool bf16)
{
    if (!bf16 || cs.stride != 1 || cs.k < 2 || cs.pad > cs.k - 1 || cs.I % 8 != 0 || cs.O % 8 != 0) return 0;
    return (size_t)cs.k * cs.k * cs.I * cs.O * 2;
}

namespace {
// The data gradient of a stride-1 convolution as the forward convolution of dY [N][Ho][Wo][O] with
// wt[i][k*k - 1 - t][o] = w[o][t][i] and padding k - 1 - pad.  False if this op is not one of those.
bool conv_dgrad_as_fwd(const MatOp& op, MatOp* fwd)
{
    const ConvShape& cs = op.cs;
    const size_t need = conv_dgrad_flip_bytes(cs, op.in_bf16);
    if (op.gather != GATHER_CONV_DGRAD || op.out_f32 || !need || !op.scratch || op.scratch_bytes < need) return false;
    if (reinterpret_cast<uintptr_t>(op.scratch) & 15u) return false;
    MatOp f = op;
    f.gather = GATHER_CONV_FWD;
    f.cs.H = cs.Ho; f.cs.W = cs.Wo; f.cs.Ho = cs.H; f.cs.Wo = cs.W;
    f.cs.I = cs.O; f.cs.O = cs.I;
    f.cs.pad = cs.k - 1 - cs.pad;
    f.B = op.scratch;
    f.b_sn = (int64_t)cs.k * cs.k * cs.O;
    f.b_sk = 1;
    f.scratch = nullptr;
    f.scratch_bytes = 0;
    if (!mfma_gemm2_supported(f)) return false;
    *fwd = f;
    return true;
}
}  // namespace

hipError_t run_matop(const MatOp& op_in, hipStream_t st)
{
    if (op_in.batch > 1 && !mfma_gemm2_supported(op_in)) {
        // no engine takes this batch in one launch: one product at a time
        const int64_t ein = op_in.in_bf16 ? 2 : 4, eout = op_in.out_f32 ? 4 : ein;
        for (int b = 0; b < op_in.batch; ++b) {
            MatOp one = op_in;
            one.batch = 1;
            one.A = (const char*)op_in.A + b * op_in.a_bs * ein;
            one.B = (const char*)op_in.B + b * op_in.b_bs * ein;
            one.C = (char*)op_in.C + b * op_in.c_bs * eout;
            if (op_in.bias) one.bias = op_in.bias + b * op_in.bias_bs;
            if (op_in.aux) one.aux = (char*)op_in.aux + b * op_in.aux_bs * ein;
            hipError_t e = run_matop(one, st);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }
    MatOp op = op_in;
    if (!op.out_f32 && op.splits > 1 && !mfma_gemm2_supported(op)) {
        op.splits = 1;   // the other engines split K only towards fp32 results
        op.partial = nullptr;
    }
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    const int logged = log_begin(&ev0, &ev1);
    if (logged >= 0) (void)hipEventRecord(ev0, st);
    hipError_t e;
    bool epilogue_done = true;
    MatOp flipped;
    if (conv_direct_supported(op)) e = conv_direct(op, st);
    else if (conv_dgrad_as_fwd(op, &flipped)) {
        e = flip_conv_weights(op.B, op.scratch, op.cs.O, op.cs.I, op.cs.k, st);
        if (e == hipSuccess) e = mfma_gemm2(flipped, st);
    }
    else if (mfma_gemm2_supported(op)) e = mfma_gemm2(op, st);
    else {
        epilogue_done = op.epilogue == EPI_NONE;
        if (mfma_matop_supported(op)) e = mfma_matop(op, st);
        else e = generic_matop(op, st);
    }
    if (e == hipSuccess && op.sgd && !op.sgd->done) {
        // the engine stored the gradient whole: the step runs on it as a kernel of its own
        if (!op.out_f32 || op.ldc != op.N) e = hipErrorInvalidValue;
        else e = sgd_step(op.sgd->w, op.sgd->m, (const float*)op.C, op.sgd->copy, op.sgd->copy_bf16, op.M * op.N, op.sgd->lr,
                          op.sgd->mu, op.sgd->wd, st);
        op.sgd->done = true;
    }
    if (logged >= 0) {
        (void)hipEventRecord(ev1, st);
        log_end(logged, op.role, op.gather, op.epilogue, op.splits > 1 && op.partial ? op.splits : 1, op.M, op.N, op.K, op.batch);
    }
    if (e != hipSuccess || epilogue_done) return e;
    return apply_epilogue(op, st);
}

}  // namespace lrd

extern "C" {

lrd_status lrd_profile_log_start(void** events, int32_t n_pairs)
{
    if (!events || n_pairs < 1) return LRD_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(lrd::g_log_mutex);
    lrd::g_log.clear();
    lrd::g_log.reserve((size_t)n_pairs);
    lrd::g_log_events = events;
    lrd::g_log_pairs = n_pairs;
    lrd::g_log_on.store(true);
    return LRD_OK;
}

int32_t lrd_profile_log_stop(lrd_profile_record* out, int32_t capacity)
{
    std::lock_guard<std::mutex> lock(lrd::g_log_mutex);
    lrd::g_log_on.store(false);
    const int32_t n = (int32_t)lrd::g_log.size();
    if (out)
        for (int32_t i = 0; i < n && i < capacity; ++i) out[i] = lrd::g_log[i];
    return n;
}

}  // extern "C"
