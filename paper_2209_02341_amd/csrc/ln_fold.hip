// LayerNorm folded into the linear that follows it (16-bit element types).  The paper (Sec. 5.5)
// names the fusion of LayerNorm with the QKV contractions and the bias as what the comparison
// system gains over unfused operators; here the fusion is algebraic, so the contraction keeps
// reading the un-normalised rows straight into LDS and the normalised matrix is never written:
//   LayerNorm(x) W^T + b = r (x Wf^T - mu c) + bf,
//   Wf = W gamma (per input feature),  c[n] = sum_k Wf[n,k],  bf = b + W beta,
// with mu, r = mean and 1 / sqrt(var + eps) of the row.  Three small kernels around the GEMM:
//   * fold_weights_kernel: once per weight matrix; Wf is rounded to the element type and c is
//     summed from the ROUNDED values, so the identity holds for the weights the GEMM really uses;
//   * row_stats_kernel: (mu, r) of every row, the row read once into registers (H*e bytes/row,
//     half of what a LayerNorm pass moves);
//   * merge_partials_kernel: (mu, r) from the per-128-column (sum, squared deviations) pairs that a
//     residual epilogue left behind (Chan's pairwise update, fixed order: deterministic), so a
//     LayerNorm that follows a residual add costs no pass over the rows at all.
#include "common.h"

namespace energon {

// ---- weights ------------------------------------------------------------------------------
// One wavefront per output row n.
template <typename E>
__global__ __launch_bounds__(256) void fold_weights_kernel(const E* __restrict__ w, const E* __restrict__ b,
                                                           const E* __restrict__ gamma, const E* __restrict__ beta,
                                                           int32_t N, int32_t K, E* __restrict__ wf,
                                                           float* __restrict__ colsum, float* __restrict__ bias_f) {
  const int lane = threadIdx.x & 63;
  const int32_t n = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (n >= N) return;
  const vec8<E>* wr = reinterpret_cast<const vec8<E>*>(w + (size_t)n * K);
  const vec8<E>* gr = reinterpret_cast<const vec8<E>*>(gamma);
  const vec8<E>* br = reinterpret_cast<const vec8<E>*>(beta);
  vec8<E>* orow = reinterpret_cast<vec8<E>*>(wf + (size_t)n * K);
  float c = 0.f, wb = 0.f;
  for (int32_t v = lane; v < K / 8; v += 64) {
    const vec8<E> w8 = wr[v], g8 = gr[v], b8 = br[v];
    vec8<E> o;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const float wv = static_cast<float>(w8[q]);
      o[q] = static_cast<E>(wv * static_cast<float>(g8[q]));
      c += static_cast<float>(o[q]);
      wb = fmaf(wv, static_cast<float>(b8[q]), wb);
    }
    orow[v] = o;
  }
  c = wave_sum(c);
  wb = wave_sum(wb);
  if (lane == 0) {
    colsum[n] = c;
    bias_f[n] = wb + (b != nullptr ? static_cast<float>(b[n]) : 0.f);
  }
}

hipError_t launch_fold_weights(const void* w, const void* b, const void* gamma, const void* beta, int32_t N, int32_t K,
                               int dtype, void* wf, float* colsum, float* bias_f, hipStream_t s) {
  if (N <= 0) return hipSuccess;
  const dim3 grid((unsigned)((N + 3) / 4)), block(256);
  if (dtype == 1)
    fold_weights_kernel<bf16_t><<<grid, block, 0, s>>>((const bf16_t*)w, (const bf16_t*)b, (const bf16_t*)gamma,
                                                       (const bf16_t*)beta, N, K, (bf16_t*)wf, colsum, bias_f);
  else
    fold_weights_kernel<f16_t><<<grid, block, 0, s>>>((const f16_t*)w, (const f16_t*)b, (const f16_t*)gamma,
                                                      (const f16_t*)beta, N, K, (f16_t*)wf, colsum, bias_f);
  return hipGetLastError();
}

// ---- row statistics -----------------------------------------------------------------------
constexpr int kStatThreads = 256;

__device__ inline float block_sum256(float v, float* red) {
  v = wave_sum(v);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  __syncthreads();  // red may still be read from the previous reduction
  if (lane == 0) red[wave] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

// VPT = 16-byte vectors held per thread; needs K / 8 <= kStatThreads * VPT.  Two passes over the
// registers: mean, then squared deviations (no cancellation for rows far from zero).
template <typename E, int VPT>
__global__ __launch_bounds__(kStatThreads) void row_stats_kernel(const E* __restrict__ x, int32_t K, float eps,
                                                                 float* __restrict__ stats) {
  __shared__ float red[kStatThreads / kWave];
  const int32_t row_vecs = K / 8;
  const size_t row = blockIdx.x;
  const vec8<E>* xr = reinterpret_cast<const vec8<E>*>(x + row * K);
  float v[VPT][8];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < VPT; ++i) {
    const int32_t c = threadIdx.x + i * kStatThreads;
    if (c < row_vecs) {
      const vec8<E> t = xr[c];
#pragma unroll
      for (int e = 0; e < 8; ++e) { v[i][e] = static_cast<float>(t[e]); s += v[i][e]; }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[i][e] = 0.f;
    }
  }
  const float inv_k = 1.0f / (float)K;
  const float mean = block_sum256(s, red) * inv_k;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < VPT; ++i) {
    const int32_t c = threadIdx.x + i * kStatThreads;
    if (c < row_vecs) {
#pragma unroll
      for (int e = 0; e < 8; ++e) { const float d = v[i][e] - mean; q += d * d; }
    }
  }
  const float rstd = rsqrtf(block_sum256(q, red) * inv_k + eps);
  if (threadIdx.x == 0) *reinterpret_cast<float2*>(stats + 2 * row) = make_float2(mean, rstd);
}

template <typename E>
static hipError_t stats_dispatch(const void* x, int64_t M, int32_t K, float eps, float* stats, hipStream_t s) {
  const int32_t row_vecs = K / 8;
  const int vpt = (row_vecs + kStatThreads - 1) / kStatThreads;
  const dim3 grid((unsigned)M), block(kStatThreads);
#define STAT_CASE(V) row_stats_kernel<E, V><<<grid, block, 0, s>>>((const E*)x, K, eps, stats); break;
  switch (vpt <= 1 ? 1 : vpt <= 2 ? 2 : vpt <= 4 ? 4 : vpt <= 8 ? 8 : vpt <= 16 ? 16 : 0) {
    case 1: STAT_CASE(1)
    case 2: STAT_CASE(2)
    case 4: STAT_CASE(4)
    case 8: STAT_CASE(8)
    case 16: STAT_CASE(16)
    default: return hipErrorInvalidValue;
  }
#undef STAT_CASE
  return hipGetLastError();
}

hipError_t launch_row_stats(const void* x, int64_t M, int32_t K, float eps, int dtype, float* stats, hipStream_t s) {
  if (M <= 0) return hipSuccess;
  return dtype == 1 ? stats_dispatch<bf16_t>(x, M, K, eps, stats, s) : stats_dispatch<f16_t>(x, M, K, eps, stats, s);
}

// ---- statistics from a residual epilogue's partials ------------------------------------------
// partial[m][p] = (sum, sum of squared deviations from the segment's own mean) of columns
// 128 p .. 128 p + 127 of row m.  16 lanes per row; every lane walks the segments p = lane % 16,
// + 16, ... twice (row mean first, then the squared deviations with the between-segment term).
__global__ __launch_bounds__(256) void merge_partials_kernel(const float* __restrict__ partial, int64_t M, int32_t P,
                                                             float eps, float* __restrict__ stats) {
  const int64_t m = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
  const int sub = threadIdx.x & 15;
  const bool live = m < M;
  const float2* pr = reinterpret_cast<const float2*>(partial) + (live ? m : 0) * P;
  float s = 0.f;
  for (int32_t p = sub; p < P; p += 16) s += pr[p].x;
#pragma unroll
  for (int o = 1; o < 16; o <<= 1) s += __shfl_xor(s, o, 64);
  const float inv_n = 1.0f / ((float)P * (float)kStatSeg);
  const float mean = s * inv_n;
  float q = 0.f;
  for (int32_t p = sub; p < P; p += 16) {
    const float2 t = pr[p];
    const float d = t.x * (1.0f / kStatSeg) - mean;
    q += t.y + (float)kStatSeg * d * d;
  }
#pragma unroll
  for (int o = 1; o < 16; o <<= 1) q += __shfl_xor(q, o, 64);
  if (live && sub == 0) *reinterpret_cast<float2*>(stats + 2 * m) = make_float2(mean, rsqrtf(q * inv_n + eps));
}

hipError_t launch_merge_partials(const float* partial, int64_t M, int32_t P, float eps, float* stats, hipStream_t s) {
  if (M <= 0) return hipSuccess;
  merge_partials_kernel<<<dim3((unsigned)((M + 15) / 16)), dim3(256), 0, s>>>(partial, M, P, eps, stats);
  return hipGetLastError();
}

}  // namespace energon
