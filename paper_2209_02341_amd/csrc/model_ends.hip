// The two ends of the model around the layer stack, on the packed (padding-free) layout of
// Sec. 4.3; the paper names the embedding layer (Sec. 2.2) without describing it.
//  * embed_packed_kernel: row t of the packed activations = token embedding of ids[t] + learned
//    position embedding of t's position inside its sequence (found from cu_seqlens by bisection);
//    one wavefront per row, 16-byte vectors, one rounding.  HBM-bound: 3 * H * e bytes per token.
//  * cache_fill_kernel: the K and V columns of a prefill's packed QKV rows scattered into the
//    per-sequence cache rows that later generation steps read (the padded positions of the cache
//    are never written and never read).
//  * last_rows_kernel: the row of every sequence's last valid token (what next-token logits are
//    computed from), a zero row for an empty sequence.
#include "common.h"

namespace energon {

namespace {

template <typename E>
__global__ __launch_bounds__(256) void embed_packed_kernel(const int32_t* __restrict__ ids,
                                                           const int32_t* __restrict__ cu,
                                                           const int32_t* __restrict__ positions, int32_t B, int64_t T,
                                                           const E* __restrict__ wte, int32_t V,
                                                           const E* __restrict__ wpe, int32_t P, int32_t H,
                                                           E* __restrict__ x) {
  const int lane = threadIdx.x & 63;
  const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  int32_t pos;
  if (positions != nullptr) {
    pos = positions[t];                        // a generation step: the position is given per row
  } else {
    // sequence of row t: the last b with cu[b] <= t
    int32_t lo = 0, hi = B;  // invariant: cu[lo] <= t < cu[hi]
    while (hi - lo > 1) {
      const int32_t mid = (lo + hi) >> 1;
      if (cu[mid] <= t) lo = mid; else hi = mid;
    }
    pos = (int32_t)(t - cu[lo]);
  }
  pos = pos < 0 ? 0 : (pos < P ? pos : P - 1);  // out-of-range inputs stay inside the tables
  int32_t id = ids[t];
  id = id < 0 ? 0 : (id < V ? id : V - 1);
  const vec8<E>* a = reinterpret_cast<const vec8<E>*>(wte + (size_t)id * H);
  const vec8<E>* p = reinterpret_cast<const vec8<E>*>(wpe + (size_t)pos * H);
  vec8<E>* o = reinterpret_cast<vec8<E>*>(x + (size_t)t * H);
  for (int32_t v = lane; v < H / 8; v += 64) {
    const vec8<E> a8 = a[v], p8 = p[v];
    vec8<E> r;
#pragma unroll
    for (int e = 0; e < 8; ++e) r[e] = static_cast<E>(static_cast<float>(a8[e]) + static_cast<float>(p8[e]));
    o[v] = r;
  }
}

__global__ __launch_bounds__(256) void last_rows_kernel(const uint4* __restrict__ x, const int32_t* __restrict__ cu,
                                                        int32_t B, int32_t row_vecs, uint4* __restrict__ out) {
  const int lane = threadIdx.x & 63;
  const int32_t b = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (b >= B) return;
  const int32_t end = cu[b + 1], len = end - cu[b];
  const uint4* src = x + (size_t)(len > 0 ? end - 1 : 0) * row_vecs;
  for (int32_t v = lane; v < row_vecs; v += 64) out[(size_t)b * row_vecs + v] = len > 0 ? src[v] : make_uint4(0, 0, 0, 0);
}

// K and V thirds of the packed QKV rows of a prefill -> rows 0 .. len-1 of each sequence's cache
// [B, S_cap, A]; one wavefront per packed row, 16-byte vectors.
__global__ __launch_bounds__(256) void cache_fill_kernel(const uint4* __restrict__ qkv, const int32_t* __restrict__ cu,
                                                         int32_t B, int64_t T, int32_t a_vecs, int32_t S_cap,
                                                         uint4* __restrict__ kc, uint4* __restrict__ vc) {
  const int lane = threadIdx.x & 63;
  const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  int32_t lo = 0, hi = B;  // invariant: cu[lo] <= t < cu[hi]
  while (hi - lo > 1) {
    const int32_t mid = (lo + hi) >> 1;
    if (cu[mid] <= t) lo = mid; else hi = mid;
  }
  const int32_t pos = (int32_t)(t - cu[lo]);
  if (pos >= S_cap) return;   // a sequence longer than the cache: the tail is not stored
  const uint4* src = qkv + (size_t)t * 3 * a_vecs;
  const size_t dst = ((size_t)lo * S_cap + pos) * a_vecs;
  for (int32_t v = lane; v < a_vecs; v += 64) {
    kc[dst + v] = src[a_vecs + v];
    vc[dst + v] = src[2 * a_vecs + v];
  }
}

}  // namespace

hipError_t launch_cache_fill(const void* qkv, const int32_t* cu, int32_t B, int64_t T, int64_t a_bytes, int32_t S_cap,
                             void* kc, void* vc, hipStream_t s) {
  if (T <= 0) return hipSuccess;
  cache_fill_kernel<<<dim3((unsigned)((T + 3) / 4)), dim3(256), 0, s>>>((const uint4*)qkv, cu, B, T, (int32_t)(a_bytes / 16),
                                                                       S_cap, (uint4*)kc, (uint4*)vc);
  return hipGetLastError();
}

// cu != nullptr: positions from the packed layout; else positions[t] is row t's position
hipError_t launch_embed_packed(const int32_t* ids, const int32_t* cu, const int32_t* positions, int32_t B, int64_t T,
                               const void* wte, int32_t V, const void* wpe, int32_t P, int32_t H, int dtype, void* x,
                               hipStream_t s) {
  if (T <= 0) return hipSuccess;
  const dim3 grid((unsigned)((T + 3) / 4)), block(256);
  if (dtype == 1)
    embed_packed_kernel<bf16_t><<<grid, block, 0, s>>>(ids, cu, positions, B, T, (const bf16_t*)wte, V, (const bf16_t*)wpe, P,
                                                       H,
                                                       (bf16_t*)x);
  else
    embed_packed_kernel<f16_t><<<grid, block, 0, s>>>(ids, cu, positions, B, T, (const f16_t*)wte, V, (const f16_t*)wpe, P, H,
                                                      (f16_t*)x);
  return hipGetLastError();
}

hipError_t launch_last_rows(const void* x, const int32_t* cu, int32_t B, int64_t row_bytes, void* out, hipStream_t s) {
  if (B <= 0) return hipSuccess;
  last_rows_kernel<<<dim3((unsigned)((B + 3) / 4)), dim3(256), 0, s>>>((const uint4*)x, cu, B, (int32_t)(row_bytes / 16),
                                                                      (uint4*)out);
  return hipGetLastError();
}

}  // namespace energon
