// Shape support, chunk limits and workspace sizing of the matrix-core path.
#include "m2rnn_kernels.hpp"
#include "m2rnn_mfma_common.hpp"

namespace m2rnn {

int mfma_pick_rb(int K, int V, int units);
int mfma_bwd_max_chunk(int K, int V);
size_t mfma_bwd_workspace_bytes(int B, int T, int N, int Nqk, int K, int V);

bool mfma_supported(int K, int V) { return mfma_pick_rb(K, V, 1 << 20) != 0; }

// The chunk is bounded by the backward's on-chip stash; the default is the
// largest that fits (fewest checkpoint bytes).
int mfma_max_chunk(int K, int V) { return mfma_bwd_max_chunk(K, V); }
int mfma_default_chunk(int K, int V) { return mfma_bwd_max_chunk(K, V); }

size_t mfma_workspace_bytes(int B, int T, int N, int Nqk, int K, int V, int C, int bwd) {
  (void)C;
  const int rb = mfma_pick_rb(K, V, B * N);
  if (rb == 0) return bwd ? mfma_bwd_workspace_bytes(B, T, N, Nqk, K, V) : 0;  // no tiling: the
      // register-resident kernels serve the shape (their forward needs no workspace)
  const int P = K / (16 * rb);
  const size_t fwd = P > 1 ? align256((size_t)P * B * T * N * V * 4) : 0;
  if (!bwd) return fwd;
  return mfma_bwd_workspace_bytes(B, T, N, Nqk, K, V);
}

}  // namespace m2rnn
