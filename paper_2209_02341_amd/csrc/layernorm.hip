// Row-wise LayerNorm on packed tokens (one of the position-wise operations that the paper,
// Sec. 4.3, runs on the compacted rows).  One 256-thread group per row; the row is read
// once from HBM into registers as 16-byte vectors, mean and (biased) variance are taken in
// two register passes in fp32, and the normalised row is written once: 2*H*e bytes per row.
#include "common.h"

namespace energon {

constexpr int kLnThreads = 256;

__device__ inline float block_sum(float v, float* red) {
  v = wave_sum(v);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  __syncthreads();  // red may still be read from the previous reduction
  if (lane == 0) red[wave] = v;
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int w = 0; w < kLnThreads / kWave; ++w) t += red[w];
  return t;
}

// VPT = 16-byte vectors held per thread; needs row_vecs <= kLnThreads * VPT.
template <typename T, int VPT>
__global__ __launch_bounds__(kLnThreads) void layernorm_kernel(const T* __restrict__ x, const T* __restrict__ gamma,
                                                               const T* __restrict__ beta, T* __restrict__ y,
                                                               int32_t H, float eps) {
  constexpr int VEC = Elem<T>::VEC;
  __shared__ float red[kLnThreads / kWave];
  const int32_t row_vecs = H / VEC;
  const size_t row = blockIdx.x;
  const Vec16<T>* xr = reinterpret_cast<const Vec16<T>*>(x + row * H);
  float v[VPT][VEC];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < VPT; ++i) {
    const int32_t c = threadIdx.x + i * kLnThreads;
    if (c < row_vecs) {
      const Vec16<T> t = xr[c];
#pragma unroll
      for (int e = 0; e < VEC; ++e) { v[i][e] = Elem<T>::to_f32(t.v[e]); s += v[i][e]; }
    } else {
#pragma unroll
      for (int e = 0; e < VEC; ++e) v[i][e] = 0.f;
    }
  }
  const float inv_h = 1.0f / (float)H;
  const float mean = block_sum(s, red) * inv_h;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < VPT; ++i) {
    const int32_t c = threadIdx.x + i * kLnThreads;
    if (c < row_vecs) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) { const float dlt = v[i][e] - mean; q += dlt * dlt; }
    }
  }
  const float rstd = rsqrtf(block_sum(q, red) * inv_h + eps);
  Vec16<T>* yr = reinterpret_cast<Vec16<T>*>(y + row * H);
  const Vec16<T>* gr = reinterpret_cast<const Vec16<T>*>(gamma);
  const Vec16<T>* br = reinterpret_cast<const Vec16<T>*>(beta);
#pragma unroll
  for (int i = 0; i < VPT; ++i) {
    const int32_t c = threadIdx.x + i * kLnThreads;
    if (c < row_vecs) {
      const Vec16<T> g = gr[c], b = br[c];
      Vec16<T> o;
#pragma unroll
      for (int e = 0; e < VEC; ++e)
        o.v[e] = Elem<T>::from_f32((v[i][e] - mean) * rstd * Elem<T>::to_f32(g.v[e]) + Elem<T>::to_f32(b.v[e]));
      yr[c] = o;
    }
  }
}

template <typename T>
static hipError_t dispatch(const void* x, const void* g, const void* b, void* y, int64_t T_, int32_t H, float eps,
                           hipStream_t s) {
  const int32_t row_vecs = H / Elem<T>::VEC;
  const int vpt = (row_vecs + kLnThreads - 1) / kLnThreads;
  const dim3 grid((unsigned)T_), block(kLnThreads);
#define LN_CASE(V)                                                                                       \
  layernorm_kernel<T, V><<<grid, block, 0, s>>>((const T*)x, (const T*)g, (const T*)b, (T*)y, H, eps); \
  break;
  switch (vpt <= 1 ? 1 : vpt <= 2 ? 2 : vpt <= 4 ? 4 : vpt <= 8 ? 8 : vpt <= 16 ? 16 : 0) {
    case 1: LN_CASE(1)
    case 2: LN_CASE(2)
    case 4: LN_CASE(4)
    case 8: LN_CASE(8)
    case 16: LN_CASE(16)
    default: return hipErrorInvalidValue;
  }
#undef LN_CASE
  return hipGetLastError();
}

// Largest H one launch handles (16 vectors of 8 or 4 elements in each of 256 threads).
hipError_t launch_layernorm(const void* x, const void* gamma, const void* beta, void* y, int64_t T, int32_t H,
                            float eps, int dtype, hipStream_t s) {
  if (T <= 0) return hipSuccess;
  return dtype == 1 ? dispatch<bf16_t>(x, gamma, beta, y, T, H, eps, s)
       : dtype == 2 ? dispatch<f16_t>(x, gamma, beta, y, T, H, eps, s)
                    : dispatch<float>(x, gamma, beta, y, T, H, eps, s);
}

}  // namespace energon
