// Placeholder until the matrix-core kernels land: bf16 / head_dim 128 runs the vector-ALU path.
#include "kernels.hpp"
namespace roco {
hipError_t launch_prefill_attention_mfma(const PrefillArgs& a, hipStream_t s) {
  return launch_prefill_attention_simple(1, 128, a, s);
}
}  // namespace roco
