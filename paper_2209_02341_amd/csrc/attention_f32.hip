// fp32 storage path of the packed causal attention (small fp32 workload): the row-wise
// vector-ALU kernel, instantiated for float.
#include "attention_rowwise.h"

namespace energon {

hipError_t launch_attention_f32(const float* qkv, float* out, const int32_t* cu, int32_t B, int32_t max_len,
                                int32_t nh, int32_t d, hipStream_t s) {
  return launch_attention_rowwise<float>(qkv, out, cu, B, max_len, nh, d, s);
}

}  // namespace energon
