// The two layout kernels of the paper's own attention path (Sec. 4.3): the attention core
// stays padded there, so padding is rebuilt in front of it and removed behind it, each fused
// with the head transpose.
//   rebuild:  packed [T, 3A] (Q | K | V, head-major)  ->  q, k, v  [B, nh, S, d], zeros at pads
//   remove :  padded [B, nh, S, d]                    ->  packed [T, A]
// Both are plain copies in 16-byte vectors, one wavefront per padded position (b, s); a head's
// d elements (128 or 256 bytes) stay contiguous on both sides.  HBM-bound:
// rebuild moves T*3A*e + B*S*3A*e bytes, remove 2*T*A*e.
#include "common.h"

namespace energon {

// hv = 16-byte vectors per head (d * e / 16)
__global__ __launch_bounds__(256) void rebuild_qkv_kernel(const uint4* __restrict__ qkv, uint4* __restrict__ q,
                                                          uint4* __restrict__ k, uint4* __restrict__ v,
                                                          const int32_t* __restrict__ cu, int32_t B, int32_t S,
                                                          int32_t nh, int32_t hv) {
  const int64_t p = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);  // padded position
  if (p >= (int64_t)B * S) return;
  const int lane = threadIdx.x & 63;
  const int32_t b = (int32_t)(p / S), s = (int32_t)(p % S);
  const int32_t c0 = cu[b], len = cu[b + 1] - c0;
  const int32_t third = nh * hv;  // vectors per third of a packed row
  const uint4* src = qkv + (size_t)(c0 + s) * 3 * third;
  const uint4 zero = make_uint4(0, 0, 0, 0);
  for (int32_t i = lane; i < 3 * third; i += 64) {
    const int32_t which = i / third, r = i - which * third, h = r / hv, c = r - h * hv;
    uint4* dst = which == 0 ? q : which == 1 ? k : v;
    dst[((size_t)(b * nh + h) * S + s) * hv + c] = s < len ? src[i] : zero;
  }
}

__global__ __launch_bounds__(256) void remove_padding_heads_kernel(const uint4* __restrict__ o, uint4* __restrict__ out,
                                                                   const int32_t* __restrict__ cu, int32_t B, int32_t S,
                                                                   int32_t nh, int32_t hv) {
  const int64_t p = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (p >= (int64_t)B * S) return;
  const int lane = threadIdx.x & 63;
  const int32_t b = (int32_t)(p / S), s = (int32_t)(p % S);
  const int32_t c0 = cu[b], len = cu[b + 1] - c0;
  if (s >= len) return;
  const int32_t rowv = nh * hv;
  uint4* dst = out + (size_t)(c0 + s) * rowv;
  for (int32_t i = lane; i < rowv; i += 64) {
    const int32_t h = i / hv, c = i - h * hv;
    dst[i] = o[((size_t)(b * nh + h) * S + s) * hv + c];
  }
}

hipError_t launch_rebuild_qkv(const void* qkv, void* q, void* k, void* v, const int32_t* cu, int32_t B, int32_t S,
                              int32_t nh, int32_t head_bytes, hipStream_t s) {
  const int64_t blocks = ((int64_t)B * S + 3) / 4;
  rebuild_qkv_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(static_cast<const uint4*>(qkv), static_cast<uint4*>(q),
                                                                static_cast<uint4*>(k), static_cast<uint4*>(v), cu, B,
                                                                S, nh, head_bytes / 16);
  return hipGetLastError();
}

hipError_t launch_remove_padding_heads(const void* o, void* out, const int32_t* cu, int32_t B, int32_t S, int32_t nh,
                                       int32_t head_bytes, hipStream_t s) {
  const int64_t blocks = ((int64_t)B * S + 3) / 4;
  remove_padding_heads_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(static_cast<const uint4*>(o),
                                                                         static_cast<uint4*>(out), cu, B, S, nh,
                                                                         head_bytes / 16);
  return hipGetLastError();
}

}  // namespace energon
