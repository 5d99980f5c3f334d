// MFMA decode path (placeholder: nothing supported yet, the vector-ALU path serves decode).
#include "llla_common.hpp"

namespace llla {

bool mfma_decode_supported(int, llla_dtype) { return false; }
size_t mfma_decode_workspace_bytes(int, int, int, int, llla_dtype) { return 0; }
hipError_t mfma_decode(const Problem &) { return hipErrorNotSupported; }

}  // namespace llla
