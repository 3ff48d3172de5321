// fp32 linear layer  y = epilogue(x W^T + b)  on packed rows (paper Sec. 4.3: the linear
// layers see only valid tokens).  This is the fp32 storage path, used by the small fp32
// workload; it runs on the vector ALU with a 64x64 LDS tile and a 4x4 register tile per
// lane.  The bf16 path (MFMA) lives in gemm_bf16.hip.
#include "common.h"

namespace energon {

constexpr int kTile = 64, kTileK = 16;

__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ x, const float* __restrict__ w,
                                                       const float* __restrict__ bias, const float* res,
                                                       float* y, int64_t M, int32_t N, int32_t K, int epi) {
  __shared__ float xs[kTileK][kTile + 1];
  __shared__ float ws[kTileK][kTile + 1];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int64_t m0 = (int64_t)blockIdx.x * kTile;
  const int32_t n0 = blockIdx.y * kTile;
  const int lr = tid >> 2, lk = (tid & 3) * 4;  // this lane stages row lr, k offsets lk..lk+3
  float acc[4][4] = {};
  for (int32_t k0 = 0; k0 < K; k0 += kTileK) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int32_t k = k0 + lk + e;
      xs[lk + e][lr] = (m0 + lr < M && k < K) ? x[(size_t)(m0 + lr) * K + k] : 0.f;
      ws[lk + e][lr] = (n0 + lr < N && k < K) ? w[(size_t)(n0 + lr) * K + k] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kTileK; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = xs[k][ty * 4 + i]; b[i] = ws[k][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int32_t n = n0 + tx * 4 + j;
      if (n >= N) continue;
      float v = acc[i][j] + (bias ? bias[n] : 0.f);
      if (epi == EPI_BIAS_GELU) v = gelu_erf(v);
      if (epi == EPI_BIAS_RESIDUAL) v += res[(size_t)m * N + n];
      y[(size_t)m * N + n] = v;
    }
  }
}

hipError_t launch_gemm_f32(const float* x, const float* w, const float* bias, const float* res, float* y, int64_t M,
                           int32_t N, int32_t K, int epi, hipStream_t s) {
  if (M <= 0) return hipSuccess;
  const dim3 grid((unsigned)((M + kTile - 1) / kTile), (unsigned)((N + kTile - 1) / kTile));
  gemm_f32_kernel<<<grid, 256, 0, s>>>(x, w, bias, res, y, M, N, K, epi);
  return hipGetLastError();
}

}  // namespace energon
