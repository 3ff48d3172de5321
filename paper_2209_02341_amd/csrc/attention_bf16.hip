// bf16 packed causal attention.
#include "attention_rowwise.h"

namespace energon {

hipError_t launch_attention_bf16(const bf16_t* qkv, bf16_t* out, const int32_t* cu, int32_t B, int32_t max_len,
                                 int32_t nh, int32_t d, hipStream_t s) {
  return launch_attention_rowwise<bf16_t>(qkv, out, cu, B, max_len, nh, d, s);
}

}  // namespace energon
