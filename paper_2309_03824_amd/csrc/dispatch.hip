// Engine selection for a single matrix product and the split-K policy.
#include <atomic>

#include "lrd_internal.hpp"

namespace lrd {

// Weight-gradient products have a long K (tokens or pixels) and a small output; K is cut into
// slices so that the launch has enough workgroups to fill 256 compute units.  The count depends
// only on the shape, so workspace queries and launches agree.
int choose_splits(int64_t M, int64_t N, int64_t K, bool in_bf16)
{
    (void)in_bf16;
    const int64_t tiles = ceil_div(M, 128) * ceil_div(N, 128);
    int64_t s = ceil_div(256, tiles);
    const int64_t by_k = K / 256;          // keep at least 256 reduction steps per slice
    if (s > by_k) s = by_k;
    if (s > 64) s = 64;
    return s < 2 ? 1 : (int)s;
}

namespace {
std::atomic<int> g_probe_role{0};
hipEvent_t g_probe_start = nullptr, g_probe_stop = nullptr;
}  // namespace

void probe_arm(int role, hipEvent_t start, hipEvent_t stop)
{
    g_probe_role.store(0);
    g_probe_start = start;
    g_probe_stop = stop;
    g_probe_role.store(role);
}

bool probe_take(int role, hipEvent_t* start, hipEvent_t* stop)
{
    if (role == 0) return false;
    int expected = role;
    if (!g_probe_role.compare_exchange_strong(expected, 0)) return false;
    *start = g_probe_start;
    *stop = g_probe_stop;
    return true;
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

hipError_t run_matop(const MatOp& op, hipStream_t st)
{
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    const bool probed = probe_take(op.role, &ev0, &ev1);
    if (probed) (void)hipEventRecord(ev0, st);
    hipError_t e;
    bool epilogue_done = true;
    if (mfma_gemm2_supported(op)) e = mfma_gemm2(op, st);
    else {
        epilogue_done = op.epilogue == EPI_NONE;
        if (mfma_matop_supported(op)) e = mfma_matop(op, st);
        else e = generic_matop(op, st);
    }
    if (probed) (void)hipEventRecord(ev1, st);
    if (e != hipSuccess || epilogue_done) return e;
    return apply_epilogue(op, st);
}

}  // namespace lrd
