// bf16 linear layer  y[M,N] = epilogue(x[M,K] W[N,K]^T + b)  on packed rows: the dense
// contractions that the paper (Sec. 4.3, Sec. 5.5) reports as >95 % of a large layer's time
// and that the padding removal shrinks from B*S rows to T rows.
//
// Design for gfx950:
//  * both operands are contiguous along K, so x rows feed the MFMA A operand and W rows the
//    B operand with the same 16-byte loads; v_mfma_f32_32x32x16_bf16, fp32 accumulators;
//  * a BM x BN output tile per workgroup, K walked in slabs of 64 (128 bytes per row);
//    slabs are double-buffered in LDS, the next slab is fetched from HBM into registers
//    while the MFMAs of the current one run, one barrier per slab;
//  * LDS rows are 8 chunks of 16 bytes, chunk c of row r stored at c ^ swz(r): the 32 rows a
//    wavefront reads for one MFMA operand then fall in distinct banks;
//  * workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2, so the id is
//    remapped to give every XCD a contiguous run of tiles, ordered in bands of 8 row tiles
//    so that tiles resident together share x slabs and W slabs in that L2;
//  * ragged M (T is arbitrary) and ragged N: loads clamp the row index, stores are predicated;
//  * epilogue in fp32 on the accumulators: + bias, GeLU(erf) or + residual, one rounding.
#include "common.h"

namespace energon {

constexpr int BK = 64;            // K elements per slab
constexpr int kChunks = BK / 8;   // 16-byte chunks per LDS row
constexpr int kXcds = 8;
constexpr int kGroupM = 8;        // row tiles per band

__device__ __forceinline__ int swz(int row) { return (row & 7) ^ ((row >> 3) & 1); }

template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(WM* WN * 64) void gemm_bf16_kernel(const bf16_t* __restrict__ x,
                                                                const bf16_t* __restrict__ w,
                                                                const bf16_t* __restrict__ bias, const bf16_t* res,
                                                                bf16_t* y, int64_t M, int32_t N, int32_t K, int epi,
                                                                int32_t tiles_m, int32_t tiles_n) {
  constexpr int NT = WM * WN * 64;
  constexpr int WTM = BM / WM, WTN = BN / WN;  // wavefront tile
  constexpr int TM = WTM / 32, TN = WTN / 32;  // 32x32 MFMA tiles per wavefront
  constexpr int CA = BM * kChunks / NT, CB = BN * kChunks / NT;
  static_assert(BM * kChunks % NT == 0 && BN * kChunks % NT == 0, "staging must divide evenly");
  extern __shared__ uint4 smem[];  // [2][BM + BN][kChunks]

  // ---- tile of this workgroup (XCD-aware order) ----
  const int32_t total = tiles_m * tiles_n;
  const int32_t per_xcd = (total + kXcds - 1) / kXcds;
  const int32_t idx = (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
  if (idx >= total) return;
  const int32_t band = idx / (kGroupM * tiles_n);
  const int32_t first_m = band * kGroupM;
  const int32_t band_m = min(kGroupM, tiles_m - first_m);
  const int32_t r = idx - band * kGroupM * tiles_n;
  const int32_t pm = first_m + r % band_m, pn = r / band_m;
  const int64_t m0 = (int64_t)pm * BM;
  const int32_t n0 = pn * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave / WN) * WTM, wn0 = (wave % WN) * WTN;

  // ---- staging assignments: chunk q = tid + i*NT -> (row q/8, chunk q%8) ----
  const uint4* ga[CA];
  const uint4* gb[CB];
  int sa[CA], sb[CB];
#pragma unroll
  for (int i = 0; i < CA; ++i) {
    const int q = tid + i * NT, row = q >> 3, c = q & 7;
    int64_t gr = m0 + row; if (gr > M - 1) gr = M - 1;
    ga[i] = reinterpret_cast<const uint4*>(x + (size_t)gr * K) + c;
    sa[i] = row * kChunks + (c ^ swz(row));
  }
#pragma unroll
  for (int i = 0; i < CB; ++i) {
    const int q = tid + i * NT, row = q >> 3, c = q & 7;
    int32_t gr = n0 + row; if (gr > N - 1) gr = N - 1;
    gb[i] = reinterpret_cast<const uint4*>(w + (size_t)gr * K) + c;
    sb[i] = BM * kChunks + row * kChunks + (c ^ swz(row));
  }
  // fragment addresses (chunk index without the k-step part)
  const int lrow = lane & 31, lhalf = lane >> 5;
  int fa[TM], fb[TN], fsa[TM], fsb[TN];
#pragma unroll
  for (int t = 0; t < TM; ++t) { const int row = wm0 + t * 32 + lrow; fa[t] = row * kChunks; fsa[t] = swz(row); }
#pragma unroll
  for (int t = 0; t < TN; ++t) { const int row = wn0 + t * 32 + lrow; fb[t] = (BM + row) * kChunks; fsb[t] = swz(row); }

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  constexpr int kStage = (BM + BN) * kChunks;
  const int KT = K / BK;
  uint4 ra[CA], rb[CB];
#pragma unroll
  for (int i = 0; i < CA; ++i) ra[i] = ga[i][0];
#pragma unroll
  for (int i = 0; i < CB; ++i) rb[i] = gb[i][0];
#pragma unroll
  for (int i = 0; i < CA; ++i) smem[sa[i]] = ra[i];
#pragma unroll
  for (int i = 0; i < CB; ++i) smem[sb[i]] = rb[i];
  __syncthreads();

  for (int kt = 0; kt < KT; ++kt) {
    const uint4* cur = smem + (kt & 1) * kStage;
    uint4* nxt = smem + ((kt + 1) & 1) * kStage;
    // the slab after the last one does not exist: fetch the last slab again (never read)
    const int knext = (kt + 1 < KT ? kt + 1 : kt) * kChunks;
#pragma unroll
    for (int i = 0; i < CA; ++i) ra[i] = ga[i][knext];
#pragma unroll
    for (int i = 0; i < CB; ++i) rb[i] = gb[i][knext];
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 af[TM], bfr[TN];
      const int c = ks * 2 + lhalf;
#pragma unroll
      for (int t = 0; t < TM; ++t) af[t] = *reinterpret_cast<const bf16x8*>(&cur[fa[t] + (c ^ fsa[t])]);
#pragma unroll
      for (int t = 0; t < TN; ++t) bfr[t] = *reinterpret_cast<const bf16x8*>(&cur[fb[t] + (c ^ fsb[t])]);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < CA; ++i) nxt[sa[i]] = ra[i];
#pragma unroll
    for (int i = 0; i < CB; ++i) nxt[sb[i]] = rb[i];
    __syncthreads();
  }

  // ---- epilogue: lane holds column (lane & 31), rows 8*(e/4) + 4*(lane/32) + e%4 of each tile ----
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int32_t n = n0 + wn0 + j * 32 + lrow;
    const bool n_ok = n < N;
    const float bv = (bias != nullptr && n_ok) ? static_cast<float>(bias[n]) : 0.f;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int64_t m = m0 + wm0 + i * 32 + (e >> 2) * 8 + lhalf * 4 + (e & 3);
        if (n_ok && m < M) {
          float v = acc[i][j][e] + bv;
          if (epi == EPI_BIAS_GELU) v = gelu_erf(v);
          if (epi == EPI_BIAS_RESIDUAL) v += static_cast<float>(res[(size_t)m * N + n]);
          y[(size_t)m * N + n] = static_cast<bf16_t>(v);
        }
      }
    }
  }
}

template <int BM, int BN, int WM, int WN>
static hipError_t launch_cfg(const bf16_t* x, const bf16_t* w, const bf16_t* bias, const bf16_t* res, bf16_t* y,
                             int64_t M, int32_t N, int32_t K, int epi, hipStream_t s) {
  auto kern = gemm_bf16_kernel<BM, BN, WM, WN>;
  constexpr size_t lds = 2 * (size_t)(BM + BN) * kChunks * sizeof(uint4);
  static bool attr_set = false;  // per instantiation; the attribute is idempotent, a race only repeats it
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int32_t tiles_m = (int32_t)((M + BM - 1) / BM), tiles_n = (N + BN - 1) / BN;
  const int64_t total = (int64_t)tiles_m * tiles_n;
  const int64_t grid = (total + kXcds - 1) / kXcds * kXcds;
  kern<<<dim3((unsigned)grid), dim3(WM * WN * 64), lds, s>>>(x, w, bias, res, y, M, N, K, epi, tiles_m, tiles_n);
  return hipGetLastError();
}

hipError_t launch_gemm_bf16(const bf16_t* x, const bf16_t* w, const bf16_t* bias, const bf16_t* res, bf16_t* y,
                            int64_t M, int32_t N, int32_t K, int epi, hipStream_t s) {
  if (M <= 0) return hipSuccess;
  return launch_cfg<256, 256, 2, 4>(x, w, bias, res, y, M, N, K, epi, s);
}

}  // namespace energon
