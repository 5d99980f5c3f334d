// MFMA forward path (placeholder until the matrix-core kernels land: nothing is supported, so the
// dispatcher always takes the vector-ALU path).
#include "llla_common.hpp"

namespace llla {

bool mfma_forward_supported(int, llla_dtype, bool) { return false; }
size_t mfma_forward_workspace_bytes(int, int, int, int, llla_dtype) { return 0; }
hipError_t mfma_forward(const Problem &) { return hipErrorNotSupported; }

}  // namespace llla
