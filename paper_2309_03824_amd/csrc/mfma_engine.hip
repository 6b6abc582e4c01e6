// bf16 MFMA engine (placeholder until the tile kernels land: nothing is claimed as supported).
#include "lrd_internal.hpp"

namespace lrd {

bool mfma_matop_supported(const MatOp&) { return false; }
hipError_t mfma_matop(const MatOp&, hipStream_t) { return hipErrorNotSupported; }
bool mfma_chain_supported(const ChainOp&) { return false; }
hipError_t mfma_chain(const ChainOp&, hipStream_t) { return hipErrorNotSupported; }

}  // namespace lrd
