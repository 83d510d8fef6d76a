// placeholder until the matrix-core kernels land
#include "m2rnn_kernels.hpp"
namespace m2rnn {
bool mfma_supported(int, int) { return false; }
int mfma_default_chunk(int, int) { return 16; }
int mfma_max_chunk(int, int) { return 16; }
size_t mfma_workspace_bytes(int, int, int, int, int, int, int, int) { return 0; }
hipError_t mfma_fwd(const FwdArgs &, hipStream_t) { return hipErrorNotSupported; }
hipError_t mfma_bwd(const BwdArgs &, hipStream_t) { return hipErrorNotSupported; }
}  // namespace m2rnn
