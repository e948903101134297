// bf16 causal attention on the matrix cores (placeholder: not yet enabled).
#include "kernels.h"

namespace po {

bool attention_mfma_supported(int s, int h, int n_heads) {
  (void)s;
  (void)h;
  (void)n_heads;
  return false;
}

bool attention_forward_mfma(const void*, void*, float*, int, int, int, hipStream_t) {
  set_error("attention_forward_mfma: not available");
  return false;
}

bool attention_backward_mfma(const void*, const void*, const float*, const void*, void*, float*, int, int, int,
                             hipStream_t) {
  set_error("attention_backward_mfma: not available");
  return false;
}

}  // namespace po
