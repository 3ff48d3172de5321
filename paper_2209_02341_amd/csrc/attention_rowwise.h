// Row-wise causal attention over each sequence's real length, on packed rows (the paper,
// Sec. 4.3, keeps attention on the padded layout; here it runs on the packed rows, so no
// padding is rebuilt inside a layer).  One wavefront per (sequence, head, query); keys are
// taken 64 at a time, one key per lane, with a running max / running sum (online softmax),
// so no score row is ever stored.  All arithmetic in fp32 on the vector ALU.
#pragma once
#include "common.h"

namespace energon {

constexpr int kQPerBlock = 4;

template <typename T>
__global__ __launch_bounds__(kQPerBlock* kWave) void attention_rowwise_kernel(const T* __restrict__ qkv,
                                                                              T* __restrict__ out,
                                                                              const int32_t* __restrict__ cu,
                                                                              int32_t nh, int32_t d) {
  constexpr int VEC = Elem<T>::VEC;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int32_t b = blockIdx.z, h = blockIdx.y;
  const int32_t c0 = cu[b], len = cu[b + 1] - c0;
  const int32_t i = blockIdx.x * kQPerBlock + wave;
  if (i >= len) return;  // whole wavefront leaves; nothing below synchronises across wavefronts
  const int32_t A = nh * d;
  const size_t ld = (size_t)3 * A;
  const float scale = rsqrtf((float)d);
  const Vec16<T>* qv = reinterpret_cast<const Vec16<T>*>(qkv + (size_t)(c0 + i) * ld + (size_t)h * d);
  float m = -INFINITY, l = 0.f, o[2] = {0.f, 0.f};
  for (int32_t j0 = 0; j0 <= i; j0 += kWave) {
    const int32_t j = j0 + lane;
    const bool valid = j <= i;
    float s = -INFINITY;
    if (valid) {
      const Vec16<T>* kv = reinterpret_cast<const Vec16<T>*>(qkv + (size_t)(c0 + j) * ld + A + (size_t)h * d);
      float dot = 0.f;
      for (int32_t c = 0; c < d / VEC; ++c) {
        const Vec16<T> qa = qv[c], ka = kv[c];
#pragma unroll
        for (int e = 0; e < VEC; ++e) dot += Elem<T>::to_f32(qa.v[e]) * Elem<T>::to_f32(ka.v[e]);
      }
      s = dot * scale;
    }
    const float m_new = fmaxf(m, wave_max(s));
    const float p = valid ? expf(s - m_new) : 0.f;
    const float corr = expf(m - m_new);
    l = l * corr + wave_sum(p);
    o[0] *= corr;
    o[1] *= corr;
    const int32_t n = min(kWave, i - j0 + 1);
    for (int32_t jj = 0; jj < n; ++jj) {
      const float pj = __shfl(p, jj, kWave);
      const T* vrow = qkv + (size_t)(c0 + j0 + jj) * ld + 2 * (size_t)A + (size_t)h * d;
      if (lane < d) o[0] += pj * Elem<T>::to_f32(vrow[lane]);
      if (lane + kWave < d) o[1] += pj * Elem<T>::to_f32(vrow[lane + kWave]);
    }
    m = m_new;
  }
  T* orow = out + (size_t)(c0 + i) * A + (size_t)h * d;
  const float inv = 1.0f / l;
  if (lane < d) orow[lane] = Elem<T>::from_f32(o[0] * inv);
  if (lane + kWave < d) orow[lane + kWave] = Elem<T>::from_f32(o[1] * inv);
}

template <typename T>
hipError_t launch_attention_rowwise(const T* qkv, T* out, const int32_t* cu, int32_t B, int32_t max_len, int32_t nh,
                                    int32_t d, hipStream_t s) {
  if (B <= 0 || max_len <= 0) return hipSuccess;
  const dim3 grid((unsigned)((max_len + kQPerBlock - 1) / kQPerBlock), (unsigned)nh, (unsigned)B);
  attention_rowwise_kernel<T><<<grid, kQPerBlock * kWave, 0, s>>>(qkv, out, cu, nh, d);
  return hipGetLastError();
}

}  // namespace energon
