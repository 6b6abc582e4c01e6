// Engine selection for a single matrix product and the split-K policy.
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

hipError_t run_matop(const MatOp& op, hipStream_t st)
{
    if (mfma_gemm2_supported(op)) return mfma_gemm2(op, st);
    if (mfma_matop_supported(op)) return mfma_matop(op, st);
    return generic_matop(op, st);
}

}  // namespace lrd
