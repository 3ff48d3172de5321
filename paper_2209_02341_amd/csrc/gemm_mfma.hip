// 16-bit (bf16 or fp16) linear layer  y[M,N] = epilogue(x[M,K] W[N,K]^T + b)  on packed rows: the dense
// contractions that the paper (Sec. 3.1, Sec. 5.5) reports as >95 % of a large layer's time
// and that the padding removal (Sec. 4.3) shrinks from B*S rows to T rows.
//
// Design for gfx950:
//  * both operands are contiguous along K, so x rows feed the MFMA A operand and W rows the
//    B operand with the same 16-byte chunks; fp32 accumulators;
//  * a BM x BN output tile per workgroup, K walked in slabs of 64 (128 bytes per row), two
//    slab buffers in LDS, filled straight from global memory (global_load_lds_dwordx4);
//  * an LDS row is 8 chunks of 16 bytes; chunk c of row r is stored in slot c ^ swizzle(r), chosen
//    per MFMA form so that a wavefront's operand read meets no bank conflict (measured).  Slabs
//    are moved in 1 KiB groups = 8 rows x 8 slots in lane order, the lane that lands in slot s of
//    row r fetching chunk s ^ swizzle(r): full 128-byte lines on the global side;
//  * workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2, so the id is
//    remapped to give every XCD a contiguous run of tiles, ordered in bands of 8 row tiles:
//    the 32 tiles resident on an XCD form an 8 x 4 block that shares x and W slabs in that L2;
//  * epilogue in fp32: + bias, GeLU(erf) or + residual, one rounding to the storage type.
// Two kernels:
//  * gemm_mfma_sched_kernel, 256x256 tile, 4 wavefronts x 128x128 = 8 x 8 tiles of
//    v_mfma_f32_16x16x32 with the 256 accumulators in AGPRs; the slab loop is hand-scheduled
//    (MFMA, LDS reads and the next slab's loads interleaved in asm); edge tiles are shifted
//    inwards, so nothing is clamped or predicated; the epilogue goes through LDS and leaves as
//    16-byte non-temporal stores;
//  * gemm_mfma_tile_kernel, compiler-scheduled, v_mfma_f32_32x32x16, clamped loads and predicated
//    stores: used with 128x128 tiles for everything the first kernel does not take (small or
//    ragged-below-one-tile problems, odd slab counts).
#include "common.h"
#include <algorithm>
#include <vector>

namespace energon {

constexpr int BK = 64;            // K elements per slab
constexpr int kChunks = BK / 8;   // 16-byte chunks per LDS row
constexpr int kXcds = 8;
constexpr int kGroupM = 8;        // row tiles per band

typedef __attribute__((address_space(1))) const void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

__device__ __forceinline__ int swz(int row) { return (row & 7) ^ ((row >> 3) & 1); }
// The same for the 16-row operand tiles of the 16x16x32 form, where lane l reads row l % 16, chunk
// 4 ks + l / 16: row bits 1, 2, 3 go to slot bits 0, 2, 1 (measured: zero bank conflicts; with the
// function above every such read takes two passes).
__device__ __forceinline__ int swz16(int row) {
  return ((row >> 1) & 1) | (((row >> 2) & 1) << 2) | (((row >> 3) & 1) << 1);
}

// XCD-aware tile order; false if this workgroup is one of the (< 8) padding ids.
template <int BM, int BN>
__device__ __forceinline__ bool tile_origin(int32_t tiles_m, int32_t tiles_n, int64_t& m0, int32_t& n0) {
  const int32_t total = tiles_m * tiles_n;
  const int32_t per_xcd = (total + kXcds - 1) / kXcds;
  const int32_t idx = (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
  if (idx >= total) return false;
  const int32_t band = idx / (kGroupM * tiles_n);
  const int32_t first_m = band * kGroupM;
  const int32_t band_m = min(kGroupM, tiles_m - first_m);
  const int32_t r = idx - band * kGroupM * tiles_n;
  m0 = (int64_t)(first_m + r % band_m) * BM;
  n0 = (r / band_m) * BN;
  return true;
}

// Epilogue of one wavefront: TM x TN accumulator tiles of 32x32 whose top-left element is
// (mw, nw).  In each tile the lane holds column (lane & 31), rows 8*(e/4) + 4*(lane/32) + e%4.
// FOLD: the LayerNorm-folded epilogues are compiled into their own instantiation, so that the plain
// one stays as small as it was (small problems are sensitive to it: 5 us per launch measured).
template <typename E, int TM, int TN, bool FOLD>
__device__ __forceinline__ void store_tile(const f32x16 (&acc)[TM][TN], const E* __restrict__ bias,
                                           const E* res, E* y, int64_t M, int32_t N, int epi, int64_t mw,
                                           int32_t nw, int lane, const LnFold& lf) {
  const int lrow = lane & 31, lhalf = lane >> 5;
  constexpr bool fold = FOLD;
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int32_t n = nw + j * 32 + lrow;
    const bool n_ok = n < N;
    float bv = 0.f, cv = 0.f;
    if constexpr (fold) {
      if (n_ok) { bv = lf.bias[n]; cv = lf.colsum[n]; }
    } else {
      if (bias != nullptr && n_ok) bv = static_cast<float>(bias[n]);
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int64_t m = mw + i * 32 + (e >> 2) * 8 + lhalf * 4 + (e & 3);
        if (n_ok && m < M) {
          float v = acc[i][j][e];
          if constexpr (fold) {
            const float2 st = *reinterpret_cast<const float2*>(lf.stats + 2 * m);
            v = st.y * (v - st.x * cv);
          }
          v += bv;
          if (epi == EPI_BIAS_GELU || epi == EPI_LNFOLD_GELU) v = gelu_erf(v);
          if (epi == EPI_BIAS_RESIDUAL) v += static_cast<float>(res[(size_t)m * N + n]);
          y[(size_t)m * N + n] = static_cast<E>(v);
        }
      }
    }
  }
}

// Split-K mode of the tile kernel: the raw fp32 sums of this workgroup's part of K, to
// part[m][n] of its own [M, N] slice; a second kernel adds the slices in order and applies the epilogue.
template <int TM, int TN>
__device__ __forceinline__ void store_partial(const f32x16 (&acc)[TM][TN], float* __restrict__ part, int64_t M,
                                              int32_t N, int64_t mw, int32_t nw, int lane) {
  const int lrow = lane & 31, lhalf = lane >> 5;
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int32_t n = nw + j * 32 + lrow;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int64_t m = mw + i * 32 + (e >> 2) * 8 + lhalf * 4 + (e & 3);
        if (n < N && m < M) part[(size_t)m * N + n] = acc[i][j][e];
      }
  }
}

// Epilogue of one wavefront's 128x128 tile (8 x 8 accumulator tiles of 16x16; in each the lane
// holds column lane % 16, rows 4 * (lane / 16) + e) through LDS, for tiles that lie wholly
// inside the matrix.  The accumulators go to LDS as fp32, 64 rows at a time, rows padded to 132
// floats so that the four lane groups of a store (4 rows apart) hit different banks; each lane
// then owns 8 consecutive columns of a row: bias, GeLU / residual are applied there in fp32 and the
// row segment leaves as one 16-byte store, 16 lanes per 256-byte row segment.  One rounding,
// full-line writes, marked non-temporal: y is not read again by this kernel and would only push
// x / W slabs out of the L2 (measured: 1.4 % faster).
constexpr int kEpiLd = 132;
constexpr int kEpiWaveFloats = 64 * kEpiLd;

// Sum over the 16 lanes of a DPP row (lanes 16 k .. 16 k + 15), left in every one of them:
// neighbour, other pair of the quad, other quad of the half row, other half row.
__device__ __forceinline__ float row16_sum(float v) {
  v += __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
  v += __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
  v += __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), 0x141, 0xF, 0xF, true));  // row_half_mirror
  v += __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), 0x140, 0xF, 0xF, true));  // row_mirror
  return v;
}

// MODE selects what is compiled in, so that each instantiation carries only the registers of the
// epilogues it serves (compiled all together they push a hundred accumulators out to scratch memory
// after every tile):
//   0  the plain epilogues (bias, bias + GeLU, bias + residual);
//   1  the LayerNorm-folded epilogues (EPI_LNFOLD, EPI_LNFOLD_GELU): row statistics read, no residual;
//   2  bias + residual with the row statistics of the rounded result written to lf.partial.
constexpr int kEpiPlain = 0, kEpiFolded = 1, kEpiResidualStats = 2;
template <typename E, int MODE>
__device__ __forceinline__ void store_tile_coalesced(const f32x4 (&acc)[8][8], const E* __restrict__ bias,
                                                     const E* res, E* y, int32_t N, int epi, int64_t mw,
                                                     int32_t nw, int lane, float* stage, const LnFold& lf,
                                                     float* raw = nullptr) {
  // raw (plain mode only): the workgroup holds a piece of a tile cut along K; its fp32 sums go, without
  // any epilogue, to raw[256][256] (row-major, this wavefront's quadrant at the offsets it has in the
  // tile), through the same staging, 32 bytes per lane and row.
  constexpr bool fold = MODE == kEpiFolded;
  constexpr bool stats = MODE == kEpiResidualStats;
  const bool residual = MODE == kEpiResidualStats || (MODE == kEpiPlain && epi == EPI_BIAS_RESIDUAL);
  const bool gelu = MODE == kEpiFolded ? epi == EPI_LNFOLD_GELU : (MODE == kEpiPlain && epi == EPI_BIAS_GELU);
  const int lrow = lane & 15, lq = lane >> 4;
  const int rr = lane >> 4, c8 = (lane & 15) * 8;
  float bv[8], cv[8];
#pragma unroll
  for (int q = 0; q < 8; ++q) cv[q] = 0.f;
  if (fold) {
    const float4 b0 = *reinterpret_cast<const float4*>(lf.bias + nw + c8), b1 = *reinterpret_cast<const float4*>(lf.bias + nw + c8 + 4);
    const float4 c0 = *reinterpret_cast<const float4*>(lf.colsum + nw + c8), c1 = *reinterpret_cast<const float4*>(lf.colsum + nw + c8 + 4);
    bv[0] = b0.x; bv[1] = b0.y; bv[2] = b0.z; bv[3] = b0.w; bv[4] = b1.x; bv[5] = b1.y; bv[6] = b1.z; bv[7] = b1.w;
    cv[0] = c0.x; cv[1] = c0.y; cv[2] = c0.z; cv[3] = c0.w; cv[4] = c1.x; cv[5] = c1.y; cv[6] = c1.z; cv[7] = c1.w;
  } else if (bias != nullptr) {
    const vec8<E> b8 = *reinterpret_cast<const vec8<E>*>(bias + nw + c8);
#pragma unroll
    for (int q = 0; q < 8; ++q) bv[q] = static_cast<float>(b8[q]);
  } else {
#pragma unroll
    for (int q = 0; q < 8; ++q) bv[q] = 0.f;
  }
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    // What the rows of this pass need from global memory (residual segments, row statistics) is
    // requested before the staging, so that its latency passes behind the barriers and the LDS
    // traffic instead of stalling every row of the loop below.
    vec8<E> rpre[16];
    float2 spre[16];
    if (residual && raw == nullptr) {
#pragma unroll
      for (int it = 0; it < 16; ++it)
        rpre[it] = *reinterpret_cast<const vec8<E>*>(res + (size_t)(mw + pass * 64 + it * 4 + rr) * N + nw + c8);
    }
    if (fold) {
#pragma unroll
      for (int it = 0; it < 16; ++it)
        spre[it] = *reinterpret_cast<const float2*>(lf.stats + 2 * (mw + pass * 64 + it * 4 + rr));
    }
    __syncthreads();  // the slab buffers (first pass) / the previous pass's rows are no longer read
#pragma unroll
    for (int ii = 0; ii < 4; ++ii)
#pragma unroll
      for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          stage[(ii * 16 + lq * 4 + e) * kEpiLd + j * 16 + lrow] = acc[pass * 4 + ii][j][e];
    __syncthreads();
#pragma unroll
    for (int it = 0; it < 16; ++it) {
      const int r = it * 4 + rr;
      const float4 lo = *reinterpret_cast<const float4*>(&stage[r * kEpiLd + c8]);
      const float4 hi = *reinterpret_cast<const float4*>(&stage[r * kEpiLd + c8 + 4]);
      if (MODE == kEpiPlain && raw != nullptr) {
        float* dst = raw + (size_t)(pass * 64 + r) * 256 + c8;
        *reinterpret_cast<float4*>(dst) = lo;
        *reinterpret_cast<float4*>(dst + 4) = hi;
        continue;
      }
      float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
      const size_t off = (size_t)(mw + pass * 64 + r) * N + nw + c8;
      if (fold) {  // r (v - mu c) + b as two multiply-adds
        const float rmu = spre[it].y * spre[it].x;
#pragma unroll
        for (int q = 0; q < 8; ++q) v[q] = fmaf(spre[it].y, v[q], fmaf(-rmu, cv[q], bv[q]));
      } else {
#pragma unroll
        for (int q = 0; q < 8; ++q) v[q] += bv[q];
      }
      if (gelu) {
#pragma unroll
        for (int q = 0; q < 8; ++q) v[q] = gelu_erf(v[q]);
      }
      if (residual) {
#pragma unroll
        for (int q = 0; q < 8; ++q) v[q] += static_cast<float>(rpre[it][q]);
      }
      vec8<E> o;
#pragma unroll
      for (int q = 0; q < 8; ++q) o[q] = static_cast<E>(v[q]);
      __builtin_nontemporal_store(o, reinterpret_cast<vec8<E>*>(y + off));
      if (stats) {  // the 16 lanes of this row hold one 128-column segment of it
        float s1 = 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q) s1 += static_cast<float>(o[q]);
        s1 = row16_sum(s1);
        const float seg_mean = s1 * (1.0f / kStatSeg);
        float s2 = 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q) { const float d = static_cast<float>(o[q]) - seg_mean; s2 += d * d; }
        s2 = row16_sum(s2);
        if ((lane & 15) == 0)
          *reinterpret_cast<float2*>(lf.partial + ((size_t)(mw + pass * 64 + r) * (N / kStatSeg) + nw / kStatSeg) * 2) =
              make_float2(s1, s2);
      }
    }
  }
}

// ---- compiler-scheduled tile kernel ---------------------------------------------------------
// MODE 0: plain epilogues; 1: the LayerNorm-folded epilogues; 2: split K, gridDim.y parts, fp32 sums
// of part blockIdx.y to lf.partial + blockIdx.y * M * N (lf.partial is the caller's scratch here).
template <typename E, int BM, int BN, int WM, int WN, int MODE>
__global__ __launch_bounds__(WM* WN * 64) void gemm_mfma_tile_kernel(const E* __restrict__ x,
                                                                     const E* __restrict__ w,
                                                                     const E* __restrict__ bias,
                                                                     const E* res, E* y, int64_t M,
                                                                     int32_t N, int32_t K, int epi, int32_t tiles_m,
                                                                     int32_t tiles_n, LnFold lf) {
  constexpr int NW = WM * WN;
  constexpr int WTM = BM / WM, WTN = BN / WN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int GA = BM / 8 / NW, GB = BN / 8 / NW;  // 8-row groups (1 KiB of LDS) per wavefront
  static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "row groups must divide evenly");
  extern __shared__ uint4 smem[];  // [2][BM + BN][kChunks]

  int64_t m0;
  int32_t n0;
  if (!tile_origin<BM, BN>(tiles_m, tiles_n, m0, n0)) return;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm0 = (wave / WN) * WTM, wn0 = (wave % WN) * WTN;

  // One direct-to-LDS load fills 1 KiB = 8 rows x 8 chunks; lane l lands at row l/8, slot l%8 of
  // the group, so it must fetch the chunk that the swizzle puts in that slot.
  // Byte offsets from the tile's first row (uniform base pointer + 32-bit lane offset).
  const int KT = MODE == 2 ? K / BK / (int)gridDim.y : K / BK;                   // slabs of this workgroup
  const size_t k0 = MODE == 2 ? (size_t)blockIdx.y * KT * (BK * sizeof(E)) : 0;   // byte offset of its first slab
  const char* xbase = reinterpret_cast<const char*>(x + (size_t)m0 * K) + k0;
  const char* wbase = reinterpret_cast<const char*>(w + (size_t)n0 * K) + k0;
  uint32_t oa[GA], ob[GB];
#pragma unroll
  for (int i = 0; i < GA; ++i) {
    const int row = (wave + i * NW) * 8 + (lane >> 3), c = (lane & 7) ^ swz(row);
    const int64_t lim = M - 1 - m0;
    const uint32_t rr = (uint32_t)(row < lim ? row : lim);
    oa[i] = (rr * (uint32_t)K + c * 8) * 2u;
  }
#pragma unroll
  for (int i = 0; i < GB; ++i) {
    const int row = (wave + i * NW) * 8 + (lane >> 3), c = (lane & 7) ^ swz(row);
    const int32_t lim = N - 1 - n0;
    const uint32_t rr = (uint32_t)(row < lim ? row : lim);
    ob[i] = (rr * (uint32_t)K + c * 8) * 2u;
  }
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

  constexpr int kStage = (BM + BN) * kChunks;  // in uint4

  auto issue = [&](int kt, int stage) {
    uint4* base = smem + stage * kStage;
    const char* xk = xbase + (size_t)kt * (BK * 2);
    const char* wk = wbase + (size_t)kt * (BK * 2);
#pragma unroll
    for (int i = 0; i < GA; ++i)
      __builtin_amdgcn_global_load_lds((gptr_t)(xk + oa[i]), (lptr_t)(base + (wave + i * NW) * 64), 16, 0, 0);
#pragma unroll
    for (int i = 0; i < GB; ++i)
      __builtin_amdgcn_global_load_lds((gptr_t)(wk + ob[i]), (lptr_t)(base + BM * kChunks + (wave + i * NW) * 64), 16,
                                       0, 0);
  };

  issue(0, 0);
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the LDS writes of this wavefront have landed
  __syncthreads();

  for (int kt = 0; kt < KT; ++kt) {
    const uint4* cur = smem + (kt & 1) * kStage;
    if (kt + 1 < KT) issue(kt + 1, (kt + 1) & 1);
    vec8<E> af[2][TM], bfr[2][TN];
#pragma unroll
    for (int t = 0; t < TM; ++t) af[0][t] = *reinterpret_cast<const vec8<E>*>(&cur[fa[t] + (lhalf ^ fsa[t])]);
#pragma unroll
    for (int t = 0; t < TN; ++t) bfr[0][t] = *reinterpret_cast<const vec8<E>*>(&cur[fb[t] + (lhalf ^ fsb[t])]);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      const int p = ks & 1;
      if (ks + 1 < BK / 16) {
        const int c = (ks + 1) * 2 + lhalf;
#pragma unroll
        for (int t = 0; t < TM; ++t) af[p ^ 1][t] = *reinterpret_cast<const vec8<E>*>(&cur[fa[t] + (c ^ fsa[t])]);
#pragma unroll
        for (int t = 0; t < TN; ++t) bfr[p ^ 1][t] = *reinterpret_cast<const vec8<E>*>(&cur[fb[t] + (c ^ fsb[t])]);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = Mfma<E>::m32x32x16(af[p][i], bfr[p][j], acc[i][j]);
      // issue order: one LDS read of the next step's operands after every two MFMAs of this step
      if (ks + 1 < BK / 16) {
#pragma unroll
        for (int q = 0; q < TM + TN; ++q) {
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, (TM * TN) / (TM + TN), 0);
        }
      }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
  }

  if constexpr (MODE == 2)
    store_partial<TM, TN>(acc, lf.partial + (size_t)blockIdx.y * M * N, M, N, m0 + wm0, n0 + wn0, lane);
  else
    store_tile<E, TM, TN, MODE == 1>(acc, bias, res, y, M, N, epi, m0 + wm0, n0 + wn0, lane, lf);
}

// ---- hand-scheduled 256x256 kernel ----------------------------------------------------------
// Work decomposition.  The kernel is persistent: 8 * wgs workgroups (one per CU: 128 KiB of LDS each),
// workgroup id b running on XCD b % 8 as its workgroup j = b / 8.  Every XCD owns a fixed sequence
// of tiles, and its workgroups walk it in rounds: workgroup j takes tiles j, j + wgs, j + 2 wgs, ...
// so the tiles resident on an XCD at one time are wgs consecutive ones of its sequence, a compact
// block that shares x and W slabs in that XCD's L2.
//   raster 0: the tiles in bands of kGroupM row tiles, column by column inside a band, cut in 8 equal
//             runs, one per XCD (resident block: 8 x 4 tiles);
//   raster 1: XCD x owns row tiles [x R, (x + 1) R), R = tiles_m / 8, walked in bands of at most
//             kGroupM rows, column by column inside a band (resident block: min(R, 8) rows x wgs /
//             min(R, 8) columns), all XCDs moving through the columns of W together, so that a W slab
//             comes from HBM once and reaches the other seven L2s from the memory-side cache; the
//             tiles_m % 8 leftover row tiles are dealt column-wise, 1/8 to each XCD, at the end.
// With pieces = P > 1 the tiles of an XCD beyond its last full round (fewer than wgs) are not run as
// one more, partly empty round: each is cut along K into P chunks of the same even length (the last
// one shorter), chunk borders at the same slabs for every tile, and the rem * P pieces are dealt to
// the XCD's workgroups chunk by chunk (piece q = chunk * rem + tile, workgroup j takes q = j, j + wgs,
// ...).  Workgroups of a round thus walk the same slabs at the same time and keep sharing x and W
// slabs in the L2, as whole tiles do.  (Cutting the remainder's slabs into wgs equal contiguous
// shares, the textbook stream-K cut, balances better but starts every workgroup at a different K
// offset: measured on the tensor-parallel shard's QKV shape it took the L2 hit rate down far enough
// to make the launch 1.7 times slower than with whole tiles.)  A piece leaves its fp32 accumulators
// (row-major 256 x 256) in the caller's scratch, slot tile * P + chunk of its XCD; a second kernel adds the P pieces of
// every cut tile in ascending K order and applies the epilogue: deterministic, no atomics, no
// workgroup waits for another.  The tail of a launch is then a short, well filled round instead of
// a long, partly empty one: that matters where a tile is long and rounds are few (the
// tensor-parallel shard: 312 tiles of 192 slabs on 256 CUs).
struct SchedPlan {
  int32_t tiles_m, tiles_n, kt;   // kt: slabs of 64 along K per tile
  int32_t wgs;                    // workgroups per XCD
  int32_t raster;                 // 0 / 1, see above
  int32_t pieces;                 // P: 1 = remainder tiles run whole
};
struct XcdShare { int32_t n_tiles, dp_rounds, rem, chunk; };   // chunk: slabs per piece

__host__ __device__ inline int32_t sched_chunk(int32_t kt, int32_t pieces) {
  int32_t c = (kt + pieces - 1) / pieces;
  return c + (c & 1);
}

__host__ __device__ inline XcdShare xcd_share(const SchedPlan& p, int32_t x) {
  XcdShare s;
  if (p.raster == 1) {
    const int32_t rows = p.tiles_m / kXcds, left = (p.tiles_m - kXcds * rows) * p.tiles_n;
    const int32_t q = (left + kXcds - 1) / kXcds;
    const int32_t mine = left - x * q;
    s.n_tiles = rows * p.tiles_n + (mine < 0 ? 0 : (mine > q ? q : mine));
  } else {
    const int32_t total = p.tiles_m * p.tiles_n, per = (total + kXcds - 1) / kXcds;
    const int32_t mine = total - x * per;
    s.n_tiles = mine < 0 ? 0 : (mine > per ? per : mine);
  }
  if (p.pieces > 1) {
    s.dp_rounds = s.n_tiles / p.wgs;
    s.rem = s.n_tiles - s.dp_rounds * p.wgs;
    s.chunk = sched_chunk(p.kt, p.pieces);
  } else {
    s.dp_rounds = (s.n_tiles + p.wgs - 1) / p.wgs;   // the last one possibly not full
    s.rem = 0;
    s.chunk = p.kt;
  }
  return s;
}

// Tile l of XCD x's sequence -> (row tile, column tile).
__host__ __device__ inline void sched_tile(const SchedPlan& p, int32_t x, int32_t l, int32_t& tm, int32_t& tn) {
  if (p.raster == 1) {
    const int32_t rows = p.tiles_m / kXcds, main_n = rows * p.tiles_n;
    if (l < main_n) {   // the XCD's rows in bands of kGroupM, column by column inside a band
      const int32_t band = l / (kGroupM * p.tiles_n);
      const int32_t first = band * kGroupM;
      const int32_t band_m = rows - first < kGroupM ? rows - first : kGroupM;
      const int32_t r = l - band * kGroupM * p.tiles_n;
      tn = r / band_m;
      tm = x * rows + first + (r - tn * band_m);
    } else {
      const int32_t left_rows = p.tiles_m - kXcds * rows;
      const int32_t q = (left_rows * p.tiles_n + kXcds - 1) / kXcds;
      const int32_t g = x * q + (l - main_n);
      tn = g / left_rows;
      tm = kXcds * rows + (g - tn * left_rows);
    }
  } else {
    const int32_t total = p.tiles_m * p.tiles_n, per = (total + kXcds - 1) / kXcds;
    const int32_t idx = x * per + l;
    const int32_t band = idx / (kGroupM * p.tiles_n);
    const int32_t first_m = band * kGroupM;
    const int32_t band_m = p.tiles_m - first_m < kGroupM ? p.tiles_m - first_m : kGroupM;
    const int32_t r = idx - band * kGroupM * p.tiles_n;
    tn = r / band_m;
    tm = first_m + (r - tn * band_m);
  }
}

// The work of workgroup `wg` of XCD `xcd`, in the order it is done: whole tiles first, then pieces of
// the XCD's cut tiles.  next() yields tile l of the XCD's sequence, the slabs [kb, kb + n) of it, and
// the scratch slot of the piece inside the XCD's 2 * wgs slots (-1: the whole tile, finished by this
// workgroup).  Shared by the kernel and the host-side check of the decomposition.
struct SchedWalker {
  XcdShare share;
  int32_t wgs, wg, kt, pieces, n_whole, n_chunks, q_stop, done, q;
  __host__ __device__ SchedWalker(const SchedPlan& p, int32_t xcd, int32_t wg_) {
    share = xcd_share(p, xcd);
    wgs = p.wgs; wg = wg_; kt = p.kt; pieces = p.pieces;
    if (p.pieces > 1) n_whole = share.dp_rounds;
    else n_whole = share.n_tiles > wg ? (share.n_tiles - wg + wgs - 1) / wgs : 0;
    n_chunks = (kt + share.chunk - 1) / share.chunk;   // <= pieces
    q_stop = share.rem * n_chunks;
    done = 0;
    q = wg;
  }
  __host__ __device__ bool next(int32_t& l, int32_t& kb, int32_t& n, int32_t& slot) {
    if (done < n_whole) {
      l = done * wgs + wg;
      kb = 0;
      n = kt;
      slot = -1;
      ++done;
      return true;
    }
    if (q < q_stop) {
      const int32_t c = q / share.rem, t = q - c * share.rem;
      l = share.dp_rounds * wgs + t;
      kb = c * share.chunk;
      n = kt - kb < share.chunk ? kt - kb : share.chunk;
      slot = t * pieces + c;
      q += wgs;
      return true;
    }
    return false;
  }
};

constexpr int kPartFloats = 256 * 256;   // one piece's accumulators

// The slab loop is written as ordered inline-asm statements so that the issue order is exactly
// the one below (the compiler otherwise re-serialises LDS reads and MFMAs, and it must not copy
// or spill a register whose load is still in flight).  One wavefront per SIMD, 128x128 per
// wavefront = 8 x 8 tiles of v_mfma_f32_16x16x32_bf16 (measured on random operands under the
// chip's power limit: 16 % more flops per second than the 32x32x16 form).
// A slab of 64 along K is two MFMA steps of 32; a step is four quadrants of 16 MFMAs, one half
// (4 fragments) of the A operands against one half of the B operands.  There is ONE set of
// operand registers: the quadrants are walked in an order in which each half is released at
// least one quadrant before its successor is needed,
//   even step:  (aL,bL) (aL,bH) (aH,bH) (aH,bL)      odd step:  (aL,bH) (aL,bL) (aH,bL) (aH,bH)
// and every quadrant carries the 4 LDS reads that refill the half released last, 2 global loads
// and 2 LDS writes of staged chunks (see ENERGON_QUAD and ENERGON_SLAB): LDS and memory traffic
// is even over the loop.  One barrier per slab; a fetched chunk has 1.75 slab times to arrive.
// What the compiler cannot see inside asm statements it cannot guard: this code itself keeps
// the wait states between an MFMA and the first read of its result (end of the slab loop) and
// between a register write and an MFMA reading it (accumulator zeroing).
#define ENERGON_DS_READ(dst, addr, off) \
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(off) : "memory")
#define ENERGON_MFMA(acc, a, b)                                                                          \
  do {                                                                                                   \
    if constexpr (__is_same(E, bf16_t))                                                                  \
      asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));              \
    else                                                                                                 \
      asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));               \
  } while (0)

template <typename E, int BM, int BN, int WM, int WN, int MODE>
__global__ __launch_bounds__(WM* WN * 64) void gemm_mfma_sched_kernel(const E* __restrict__ x,
                                                                    const E* __restrict__ w,
                                                                    const E* __restrict__ bias,
                                                                    const E* res, E* y, int64_t M,
                                                                    int32_t N, int32_t K, int epi, SchedPlan plan,
                                                                    float* __restrict__ part, LnFold lf) {
  constexpr int NW = WM * WN;
  constexpr int WTM = BM / WM, WTN = BN / WN;
  constexpr int TM = WTM / 16, TN = WTN / 16;
  constexpr int GA = BM / 8 / NW, GB = BN / 8 / NW;
  static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "row groups must divide evenly");
  static_assert((BM + BN) * 128 == 65536, "stage stride is assumed to be 64 KiB");
  static_assert(TM == 8 && TN == 8 && GA + GB == 16, "the hand schedule is written for 4 x (128x128)");
  static_assert(BM * BN == kPartFloats, "a piece's accumulators");
  extern __shared__ uint4 smem[];  // [2][BM + BN][kChunks]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, kept in an SGPR
  const int wm0 = (wave / WN) * WTM, wn0 = (wave % WN) * WTN;

  // This workgroup's share: whole tiles first, then its pieces of the XCD's cut tiles.
  const int32_t xcd = blockIdx.x % kXcds;
  SchedWalker walk(plan, xcd, blockIdx.x / kXcds);

  for (;;) {
    // ---- next piece of work: tile l of the XCD's sequence, slabs [kb, kb + KT) of it ----
    int32_t l, kb, KT, slot;
    if (!walk.next(l, kb, KT, slot)) break;
    // non-null: the piece does not cover its tile
    float* const piece_out = slot < 0 ? nullptr : part + ((size_t)xcd * (2 * plan.wgs) + (size_t)slot) * kPartFloats;
    int32_t tm, tn;
    sched_tile(plan, xcd, l, tm, tn);
    int64_t m0 = (int64_t)tm * BM;
    int32_t n0 = tn * BN;
    // Ragged edges: the last tile of a row / column of tiles is shifted back so that it ends at
    // M / N (needs M >= BM, N >= BN).  It overlaps its neighbour; both compute bit-identical values
    // for the shared elements, so no load is clamped and no store is predicated.
    if (m0 > M - BM) m0 = M - BM;
    if (n0 > N - BN) n0 = N - BN;

    // Per-lane addresses are derived afresh for every piece from an opaque copy of the lane id: kept
    // alive across the epilogue instead, they would cost it registers it does not have.
    int lane_i = lane;
    asm volatile("" : "+v"(lane_i));
    // MFMA operand fragment of a 16-row tile for the step ks (32 along K = chunks 4 ks .. 4 ks + 3
    // of the slab row): lane l holds row l % 16, chunk 4 ks + l / 16.  LDS byte address of that
    // chunk for tile 0; tile t adds t * 2048 (16 rows), and swz depends on row % 16 only.
    const int lrow = lane_i & 15, lq = lane_i >> 4;
    uint32_t aaddr[2], baddr[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const uint32_t chunk = (uint32_t)((ks * 4 + lq) ^ swz16(lrow)) * 16u;
      aaddr[ks] = (uint32_t)(wm0 + lrow) * 128u + chunk;
      baddr[ks] = (uint32_t)(BM + wn0 + lrow) * 128u + chunk;
    }
    // Slab loads go straight from global memory to LDS (global_load_lds_dwordx4: no staging
    // register, no LDS store instruction; LDS stores from registers would occupy the LDS pipeline
    // longer than all the operand reads).  One instruction moves a row group: 8 rows x 128 bytes =
    // 1 KiB of LDS in lane order, lane l landing in slot l % 8 of row l / 8 and fetching the chunk
    // that the swizzle puts there.  The 64 row groups of a slab fall in four classes by the operand
    // half that reads them -- AL / AH: x rows 0..63 / 64..127 of each wavefront row, BL / BH likewise
    // for W -- and every wavefront moves 4 groups of each class, of its own parity (swz(row) depends
    // on row % 16 = 8 * (group parity) + l / 8, so one per-lane offset serves all its groups).
    const uint32_t voff = ((uint32_t)(lane_i >> 3) * (uint32_t)K +
                           (uint32_t)(((lane_i & 7) ^ swz16((wave & 1) * 8 + (lane_i >> 3))) * 8)) * 2u;

    f32x4 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;
    // The compiler sees no MFMA (they are inside asm statements) and so adds no wait states between
    // a register write and an MFMA that reads it: have the zeros written here, before the prologue.
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) asm volatile("" : "+a"(acc[i][j]));

    const char* gsrc[4][4];  // [class AL, BH, BL, AH][j]: global address of the group's first row, slab kb
    uint32_t ldst[4][4];     // its LDS byte offset in buffer 0
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const bool is_a = (c == 0 || c == 3), high = (c == 1 || c == 3);
        const int gl = 2 * ((wave >> 1) * 4 + j) + (wave & 1);           // 0..15 within the class
        const int g = gl + (gl >= 8 ? 8 : 0) + (high ? 8 : 0);            // row group within the operand's 32
        gsrc[c][j] = reinterpret_cast<const char*>((is_a ? x + (size_t)m0 * K : w + (size_t)n0 * K) + (size_t)(8 * g) * K) +
                     (size_t)kb * (BK * 2);
        ldst[c][j] = (uint32_t)((is_a ? 0 : BM * 128) + g * 1024);
      }
#define ENERGON_DMA(c, j, kt_, buf)                                                                     \
  __builtin_amdgcn_global_load_lds((gptr_t)(gsrc[c][j] + (size_t)(kt_) * (BK * 2) + voff),              \
                                   (lptr_t)(reinterpret_cast<char*>(smem) + (buf) * 0x10000 + ldst[c][j]), 16, 0, 0)

    vec8<E> fa[TM], fb[TN];  // the operand fragments: x-row tiles, W-row tiles
#define ENERGON_RA(t, ks) ENERGON_DS_READ(fa[t], aaddr[ks], (t) * 2048)
#define ENERGON_RB(t, ks) ENERGON_DS_READ(fb[t], baddr[ks], (t) * 2048)
#define ENERGON_MF(i, j) ENERGON_MFMA(acc[i][j], fa[i], fb[j])
#define ENERGON_NONE do { } while (0)
// Wait for this wavefront's LDS reads and for all but its newest `n` slab loads, then meet the
// other wavefronts: what they have read may now be overwritten, what they have fetched may be read.
#define ENERGON_SYNC(n)                                                   \
  do {                                                                    \
    asm volatile("s_waitcnt vmcnt(" #n ") lgkmcnt(0)" ::: "memory");      \
    __builtin_amdgcn_s_barrier();                                         \
  } while (0)

// One quadrant: the 16 MFMAs of A tiles ai..ai+3 against B tiles bj..bj+3 (rows walked back and
// forth, so that consecutive MFMAs share an operand: measurably less power) with, slotted between
// them, four LDS reads R0..R3 (fragments of a half that the previous quadrants have released) and
// up to four slab loads D0..D3; TAIL is the synchronisation that ends it (the reads are back on
// leaving in any case).
#define ENERGON_QUAD(ai, bj, R0, R1, R2, R3, D0, D1, D2, D3, TAIL)                              \
  do {                                                                                         \
    ENERGON_MF(ai + 0, bj + 0); R0; ENERGON_MF(ai + 0, bj + 1); R1;                             \
    ENERGON_MF(ai + 0, bj + 2); R2; ENERGON_MF(ai + 0, bj + 3); R3;                             \
    ENERGON_MF(ai + 1, bj + 3); D0; ENERGON_MF(ai + 1, bj + 2); D1;                             \
    ENERGON_MF(ai + 1, bj + 1); D2; ENERGON_MF(ai + 1, bj + 0); D3;                             \
    ENERGON_MF(ai + 2, bj + 0); ENERGON_MF(ai + 2, bj + 1); ENERGON_MF(ai + 2, bj + 2); ENERGON_MF(ai + 2, bj + 3); \
    ENERGON_MF(ai + 3, bj + 3); ENERGON_MF(ai + 3, bj + 2); ENERGON_MF(ai + 3, bj + 1); ENERGON_MF(ai + 3, bj + 0); \
    TAIL;                                                                                      \
  } while (0)
#define ENERGON_READS_BACK asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory")

    const int klast = KT - 1;
    // Prologue: slab 0 into buffer 0 (waited for), slab 1 into buffer 1 (in flight), the fragments
    // of the first quadrant in registers.  Load order within a slab is AL, BH, BL, AH throughout.
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
      for (int j = 0; j < 4; ++j) ENERGON_DMA(c, j, 0, 0);
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
      for (int j = 0; j < 4; ++j) ENERGON_DMA(c, j, (1 < klast ? 1 : klast), 1);
    asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    ENERGON_RA(0, 0); ENERGON_RA(1, 0); ENERGON_RA(2, 0); ENERGON_RA(3, 0);
    ENERGON_RB(0, 0); ENERGON_RB(1, 0); ENERGON_RB(2, 0); ENERGON_RB(3, 0);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");

    // Slab kt is consumed from buffer kt & 1 while slab kt+1 (other buffer) is landing.  Quadrants
    // 2, 3, 4, 5 hold the last reads of the classes AL, BH, BL, AH of slab kt; the barrier that
    // ends each of them frees that class's rows in the current buffer, and the loads of the same
    // class of slab kt+2 follow in the next two quadrants.  Reads of slab kt+1 start in quadrant 6
    // (AL), 7 (BL), then 0 (BH) and 1 (AH) of the next slab: the barriers ending quadrants 5, 6 and
    // 0 are preceded by waits for exactly those classes (loads return in order; the count is the
    // number of loads issued after the class's last).  A load thus has 8 to 10 quadrants, a good
    // slab time, to arrive, and loads are issued in every quadrant but three.
#define ENERGON_SLAB(kt_, cur, nxt)                                                                     \
  {                                                                                                     \
    const int kl2 = (kt_) + 2 < KT ? (kt_) + 2 : klast;                                                 \
    ENERGON_QUAD(0, 0, ENERGON_RB(4, 0), ENERGON_RB(5, 0), ENERGON_RB(6, 0), ENERGON_RB(7, 0),           \
                 ENERGON_NONE, ENERGON_NONE, ENERGON_NONE, ENERGON_NONE, ENERGON_SYNC(16));             \
    ENERGON_QUAD(0, 4, ENERGON_RA(4, 0), ENERGON_RA(5, 0), ENERGON_RA(6, 0), ENERGON_RA(7, 0),           \
                 ENERGON_NONE, ENERGON_NONE, ENERGON_NONE, ENERGON_NONE, ENERGON_READS_BACK);           \
    ENERGON_QUAD(4, 4, ENERGON_RA(0, 1), ENERGON_RA(1, 1), ENERGON_RA(2, 1), ENERGON_RA(3, 1),           \
                 ENERGON_NONE, ENERGON_NONE, ENERGON_NONE, ENERGON_NONE, ENERGON_SYNC(16));             \
    ENERGON_QUAD(4, 0, ENERGON_RB(4, 1), ENERGON_RB(5, 1), ENERGON_RB(6, 1), ENERGON_RB(7, 1),           \
                 ENERGON_DMA(0, 0, kl2, cur), ENERGON_DMA(0, 1, kl2, cur), ENERGON_NONE, ENERGON_NONE,   \
                 ENERGON_SYNC(18));                                                                     \
    ENERGON_QUAD(0, 4, ENERGON_RB(0, 1), ENERGON_RB(1, 1), ENERGON_RB(2, 1), ENERGON_RB(3, 1),           \
                 ENERGON_DMA(0, 2, kl2, cur), ENERGON_DMA(0, 3, kl2, cur), ENERGON_DMA(1, 0, kl2, cur),  \
                 ENERGON_DMA(1, 1, kl2, cur), ENERGON_SYNC(22));                                        \
    ENERGON_QUAD(0, 0, ENERGON_RA(4, 1), ENERGON_RA(5, 1), ENERGON_RA(6, 1), ENERGON_RA(7, 1),           \
                 ENERGON_DMA(1, 2, kl2, cur), ENERGON_DMA(1, 3, kl2, cur), ENERGON_DMA(2, 0, kl2, cur),  \
                 ENERGON_DMA(2, 1, kl2, cur), ENERGON_SYNC(22));                                        \
    _Pragma("unroll") for (int ks = 0; ks < 2; ++ks) { aaddr[ks] ^= 0x10000u; baddr[ks] ^= 0x10000u; }  \
    ENERGON_QUAD(4, 0, ENERGON_RA(0, 0), ENERGON_RA(1, 0), ENERGON_RA(2, 0), ENERGON_RA(3, 0),           \
                 ENERGON_DMA(2, 2, kl2, cur), ENERGON_DMA(2, 3, kl2, cur), ENERGON_DMA(3, 0, kl2, cur),  \
                 ENERGON_DMA(3, 1, kl2, cur), ENERGON_SYNC(18));                                        \
    ENERGON_QUAD(4, 4, ENERGON_RB(0, 0), ENERGON_RB(1, 0), ENERGON_RB(2, 0), ENERGON_RB(3, 0),           \
                 ENERGON_DMA(3, 2, kl2, cur), ENERGON_DMA(3, 3, kl2, cur), ENERGON_NONE, ENERGON_NONE,   \
                 ENERGON_READS_BACK);                                                                   \
  }
    for (int kt = 0; kt < KT; kt += 2) {  // KT is even (K % 128 == 0 and chunks of even length)
      ENERGON_SLAB(kt, 0, 1)
      ENERGON_SLAB(kt + 1, 1, 0)
      // Last trip only: let the MFMA pipeline run empty before control leaves the loop.  Past this
      // point the compiler moves accumulators between registers as it pleases, and it knows of no
      // MFMA in flight (they are inside asm statements), so it would add none of the wait states
      // that a read of a matrix-core result needs.
      asm volatile("s_cmp_lt_i32 %0, %1\n\t"
                   "s_cbranch_scc1 .Lenergon_more_%=\n\t"
                   "s_nop 15\n\ts_nop 15\n\ts_nop 15\n"
                   ".Lenergon_more_%=:"
                   :
                   : "s"(kt + 2), "s"(KT)
                   : "scc", "memory");
    }
#undef ENERGON_SLAB
    // Outstanding loads (the clamped refetches of the last slabs) still write to LDS.
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
#undef ENERGON_DMA
#undef ENERGON_QUAD
#undef ENERGON_SYNC
#undef ENERGON_READS_BACK
#undef ENERGON_NONE
#undef ENERGON_RA
#undef ENERGON_RB
#undef ENERGON_MF

    // The epilogue's per-lane addresses must not be computed (and kept live) above the slab loop,
    // where every VGPR is spoken for: route the lane id through an ordered asm statement.
    int lane_e = lane;
    asm volatile("" : "+v"(lane_e));
    // a piece of a cut tile leaves its raw sums (piece_out != nullptr), everything else its results
    store_tile_coalesced<E, MODE>(acc, bias, res, y, N, epi, m0 + wm0, n0 + wn0, lane_e,
                                  reinterpret_cast<float*>(smem) + wave * kEpiWaveFloats, lf,
                                  piece_out != nullptr ? piece_out + (size_t)wm0 * 256 + wn0 : nullptr);
    // the slab buffers (or the staging rows over them) are reused by the next piece's first loads
    __syncthreads();
  }
}

// Second kernel of a launch that cut tiles.  A workgroup finishes 16 rows of one cut tile (16 strips
// per tile): every thread owns 8 consecutive columns of a row, adds the P pieces' sums for them in
// ascending K order (all loads issued before the first add), applies bias, GeLU / residual in fp32,
// rounds once and stores 16 bytes.  blockIdx.x % 8 is the XCD that wrote the pieces.
constexpr int kFixStrips = 16;
template <typename E>
__global__ __launch_bounds__(512) void gemm_mfma_fixup_kernel(const float* __restrict__ part,
                                                             const E* __restrict__ bias, const E* res, E* y,
                                                             int64_t M, int32_t N, int epi, SchedPlan plan) {
  const int32_t xcd = blockIdx.x % kXcds, rest = blockIdx.x / kXcds;
  const int32_t t = rest / kFixStrips, strip = rest % kFixStrips;
  const XcdShare share = xcd_share(plan, xcd);
  if (t >= share.rem) return;
  const int32_t n_chunks = (plan.kt + share.chunk - 1) / share.chunk;
  const int tid = threadIdx.x;
  const int r = strip * 16 + (tid >> 5), c8 = (tid & 31) * 8;   // row and first column inside the tile
  const float* src = part + ((size_t)xcd * (2 * plan.wgs) + (size_t)t * plan.pieces) * kPartFloats + (size_t)r * 256 + c8;
  float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int32_t c0 = 0; c0 < n_chunks; c0 += 4) {   // four pieces' loads in flight at a time
    float4 lo[4], hi[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const bool live = c0 + c < n_chunks;
      const float* p = src + (size_t)(live ? c0 + c : c0) * kPartFloats;
      lo[c] = *reinterpret_cast<const float4*>(p);
      hi[c] = *reinterpret_cast<const float4*>(p + 4);
      if (!live) { lo[c] = make_float4(0.f, 0.f, 0.f, 0.f); hi[c] = lo[c]; }
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      v[0] += lo[c].x; v[1] += lo[c].y; v[2] += lo[c].z; v[3] += lo[c].w;
      v[4] += hi[c].x; v[5] += hi[c].y; v[6] += hi[c].z; v[7] += hi[c].w;
    }
  }
  int32_t tm, tn;
  sched_tile(plan, xcd, share.dp_rounds * plan.wgs + t, tm, tn);
  int64_t m0 = (int64_t)tm * 256;
  int32_t n0 = tn * 256;
  if (m0 > M - 256) m0 = M - 256;
  if (n0 > N - 256) n0 = N - 256;
  const int32_t n = n0 + c8;
  if (bias != nullptr) {
    const vec8<E> b8 = *reinterpret_cast<const vec8<E>*>(bias + n);
#pragma unroll
    for (int q = 0; q < 8; ++q) v[q] += static_cast<float>(b8[q]);
  }
  if (epi == EPI_BIAS_GELU) {
#pragma unroll
    for (int q = 0; q < 8; ++q) v[q] = gelu_erf(v[q]);
  }
  const size_t off = (size_t)(m0 + r) * N + n;
  if (epi == EPI_BIAS_RESIDUAL) {
    const vec8<E> r8 = *reinterpret_cast<const vec8<E>*>(res + off);
#pragma unroll
    for (int q = 0; q < 8; ++q) v[q] += static_cast<float>(r8[q]);
  }
  vec8<E> o;
#pragma unroll
  for (int q = 0; q < 8; ++q) o[q] = static_cast<E>(v[q]);
  *reinterpret_cast<vec8<E>*>(y + off) = o;
}

template <typename E, typename Kern>
static hipError_t launch_tiles(Kern kern, LdsAttrOnce& attr_set, int BM, int BN, int threads, size_t lds, const E* x,
                               const E* w, const E* bias, const E* res, E* y, int64_t M, int32_t N,
                               int32_t K, int epi, const LnFold& lf, hipStream_t s, int32_t ks = 1) {
  {
    hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), lds, attr_set);
    if (e != hipSuccess) return e;
  }
  const int32_t tiles_m = (int32_t)((M + BM - 1) / BM), tiles_n = (N + BN - 1) / BN;
  const int64_t total = (int64_t)tiles_m * tiles_n;
  const int64_t grid = (total + kXcds - 1) / kXcds * kXcds;
  kern<<<dim3((unsigned)grid, (unsigned)ks), dim3(threads), lds, s>>>(x, w, bias, res, y, M, N, K, epi, tiles_m, tiles_n,
                                                                       lf);
  return hipGetLastError();
}

// The 256x256 kernel needs whole tiles to shift at the edges, an even number of slabs, and enough
// tiles for most of the 256 CUs.  Shifted edge tiles overlap their neighbours: with the residual
// aliasing y, an overlapped element could be read after the neighbour's write, so that case
// needs whole tiles.
static bool takes_sched_kernel(int64_t M, int32_t N, int32_t K, bool res_aliases_y) {
  const int64_t big_tiles = ((M + 255) / 256) * ((N + 255) / 256);
  const bool overlap_safe = !res_aliases_y || (M % 256 == 0 && N % 256 == 0);
  return M >= 256 && N >= 256 && K % 128 == 0 && big_tiles >= 192 && overlap_safe;
}

// Row partials come from the 256x256 kernel's epilogue, one per 128-column segment, and a
// shifted column tile would count its overlap twice: whole column tiles only.
bool gemm_emits_row_partials(int64_t M, int32_t N, int32_t K, bool res_aliases_y) {
  return takes_sched_kernel(M, N, K, res_aliases_y) && N % 256 == 0;
}

// Workgroups per XCD for the persistent 256x256 kernel: one per CU (MI355X: 256 CUs in 8 XCDs).
static int32_t sched_wgs_per_xcd() {
  static int32_t cached[32] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 32;
  const bool tracked = dev >= 0 && dev < 32;
  if (tracked && cached[dev] > 0) return cached[dev];
  int cus = 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < kXcds) cus = 256;
  const int32_t v = cus / kXcds;
  if (tracked) cached[dev] = v;
  return v;
}

// Decomposition of a launch of the 256x256 kernel.  Raster: a row band per XCD once every XCD gets
// at least two row tiles (all XCDs then stream the same W columns at the same time), band order
// otherwise.  Pieces: the P in 1..8 (P rem <= 2 wgs: the scratch has 2 wgs slots per XCD) with the
// least expected time, in slab units of a busy chip (a 256x256x64 slab step takes about 1.55 us
// under the sustained power limit): the remainder's rounds of pieces, plus, for P > 1, each piece's
// start-up and accumulator store and the second kernel (it reads every piece once at about 3 TB/s
// including its own stores, after a launch gap).  P > 1 has to win by 3 % of the launch.
static SchedPlan sched_plan(int64_t M, int32_t N, int32_t K, bool can_split, int32_t wgs) {
  SchedPlan p;
  p.tiles_m = (int32_t)((M + 255) / 256);
  p.tiles_n = (N + 255) / 256;
  p.kt = K / BK;
  p.wgs = wgs;
  p.raster = p.tiles_m >= 2 * kXcds ? 1 : 0;
  p.pieces = 1;
  if (!can_split) return p;
  // per XCD: full rounds and remainder tiles (they differ by a tile between XCDs)
  int32_t full[kXcds], rem[kXcds], rem_max = 0;
  for (int32_t x = 0; x < kXcds; ++x) {
    const int32_t n = xcd_share(p, x).n_tiles;
    full[x] = n / wgs;
    rem[x] = n - full[x] * wgs;
    rem_max = rem[x] > rem_max ? rem[x] : rem_max;
  }
  if (rem_max == 0) return p;
  const double slab_us = 1.55, piece_us = 6.0;
  auto launch_time = [&](int32_t P, int32_t chunk) {   // the slowest XCD sets the time
    double worst = 0;
    for (int32_t x = 0; x < kXcds; ++x) {
      const int32_t rounds = (rem[x] * P + wgs - 1) / wgs;
      const double t = (double)full[x] * p.kt * slab_us + rounds * (chunk * slab_us + (P > 1 ? piece_us : 0.0));
      worst = t > worst ? t : worst;
    }
    return worst;
  };
  const double whole = launch_time(1, p.kt);
  double best = whole;
  for (int32_t P = 2; P <= 8 && P * rem_max <= 2 * wgs; ++P) {
    const int32_t chunk = sched_chunk(p.kt, P), n_chunks = (p.kt + chunk - 1) / chunk;
    if (n_chunks != P || chunk < 8) continue;
    int32_t cut_tiles = 0;
    for (int32_t x = 0; x < kXcds; ++x) cut_tiles += rem[x];
    const double fix_us = 8.0 + (double)cut_tiles * P * (kPartFloats * 4.0) / 3.0e6;
    const double t = launch_time(P, chunk) + fix_us;
    if (t < best && whole - t > 0.03 * whole) {
      best = t;
      p.pieces = P;
    }
  }
  return p;
}

// the most cut tiles any XCD has under a plan
static int32_t sched_max_rem(const SchedPlan& p) {
  int32_t m = 0;
  for (int32_t x = 0; x < kXcds; ++x) {
    const int32_t r = xcd_share(p, x).rem;
    m = r > m ? r : m;
  }
  return m;
}

size_t gemm_sched_scratch_bytes(int64_t M, int32_t N, int32_t K) {
  if (!takes_sched_kernel(M, N, K, false)) return 0;
  const int32_t wgs = sched_wgs_per_xcd();
  if (sched_plan(M, N, K, true, wgs).pieces == 1) return 0;
  return (size_t)2 * kXcds * wgs * kPartFloats * sizeof(float);
}

// Tile size and number of K parts for the split path of the compiler-scheduled kernel: enough
// workgroups (>= 512 where K allows), every part at least 16 slabs long.
void gemm_split_plan(int64_t M, int32_t N, int32_t K, int32_t* tile, int32_t* ks) {
  const int64_t tiles128 = ((M + 127) / 128) * ((N + 127) / 128);
  const int32_t t = tiles128 < 128 ? 64 : 128;
  const int64_t tiles = ((M + t - 1) / t) * ((N + t - 1) / t);
  const int32_t KT = K / BK;
  int32_t k = 1;
  while (k < 16 && tiles * k < 512 && KT % (2 * k) == 0 && KT / (2 * k) >= 16) k *= 2;
  *tile = t;
  *ks = k;
}

size_t gemm_split_scratch_bytes(int64_t M, int32_t N, int32_t K) {
  if (takes_sched_kernel(M, N, K, false)) return gemm_sched_scratch_bytes(M, N, K);
  int32_t tile, ks;
  gemm_split_plan(M, N, K, &tile, &ks);
  return ks > 1 ? (size_t)ks * (size_t)M * N * sizeof(float) : 0;
}

// Host-side check of the decomposition for one shape (what the kernels would do, replayed with the
// same functions): every tile is either finished whole by exactly one workgroup or cut into pieces
// whose slab ranges are even, start where the previous one ended and add up to the tile; the pieces of
// a tile occupy the slots its second-kernel workgroups read, in ascending K order; no slot is used
// twice or lies outside the XCD's 2 * wgs.  0 if all of that holds, else a positive code naming the
// first violation; -1 if the 256x256 kernel does not take the shape.
int gemm_sched_selfcheck(int64_t M, int32_t N, int32_t K, int32_t wgs, int32_t can_split, int32_t* pieces_out) {
  if (!takes_sched_kernel(M, N, K, false) || wgs < 1) return -1;
  const SchedPlan p = sched_plan(M, N, K, can_split != 0, wgs);
  if (pieces_out) *pieces_out = p.pieces;
  const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
  std::vector<int32_t> covered(tiles, 0);     // slabs covered so far (pieces must arrive in K order per tile)
  std::vector<int8_t> whole(tiles, 0);
  for (int32_t x = 0; x < kXcds; ++x) {
    const XcdShare sh = xcd_share(p, x);
    std::vector<int8_t> slot_used(2 * (size_t)wgs, 0);
    // pieces of one tile are produced by different workgroups: collect (tile, kb, n, slot) and sort by kb
    struct Piece { int64_t tile; int32_t kb, n, slot; };
    std::vector<Piece> pieces;
    int64_t seen = 0;
    for (int32_t wg = 0; wg < wgs; ++wg) {
      SchedWalker walk(p, x, wg);
      int32_t l, kb, n, slot;
      while (walk.next(l, kb, n, slot)) {
        if (l < 0 || l >= sh.n_tiles) return 1;
        int32_t tm, tn;
        sched_tile(p, x, l, tm, tn);
        if (tm < 0 || tm >= p.tiles_m || tn < 0 || tn >= p.tiles_n) return 2;
        const int64_t tile = (int64_t)tm * p.tiles_n + tn;
        if (n <= 0 || (n & 1) || (kb & 1) || kb < 0 || kb + n > p.kt) return 3;
        if (slot < 0) {
          if (kb != 0 || n != p.kt || whole[tile] || covered[tile]) return 4;
          whole[tile] = 1;
          covered[tile] = p.kt;
        } else {
          if (slot >= 2 * wgs || slot_used[slot]) return 5;
          slot_used[slot] = 1;
          pieces.push_back({tile, kb, n, slot});
        }
        ++seen;
      }
    }
    std::sort(pieces.begin(), pieces.end(), [](const Piece& a, const Piece& b) { return a.tile != b.tile ? a.tile < b.tile : a.kb < b.kb; });
    for (const Piece& q : pieces) {
      if (whole[q.tile] || covered[q.tile] != q.kb) return 6;
      covered[q.tile] += q.n;
    }
    // what the second kernel reads: cut tile t of this XCD = tile dp_rounds * wgs + t, slots t * P + c, c ascending
    const int32_t n_chunks = (p.kt + sh.chunk - 1) / sh.chunk;
    for (int32_t t = 0; t < sh.rem; ++t) {
      int32_t tm, tn;
      sched_tile(p, x, sh.dp_rounds * wgs + t, tm, tn);
      const int64_t tile = (int64_t)tm * p.tiles_n + tn;
      int32_t kb = 0;
      for (int32_t c = 0; c < n_chunks; ++c) {
        bool found = false;
        for (const Piece& q : pieces)
          if (q.slot == t * p.pieces + c) { found = q.tile == tile && q.kb == kb; kb += q.n; break; }
        if (!found) return 7;
      }
      if (kb != p.kt) return 8;
    }
    if (sh.rem > wgs || (p.pieces > 1 && sh.rem * p.pieces > 2 * wgs)) return 9;
    (void)seen;
  }
  for (int64_t t = 0; t < tiles; ++t)
    if (covered[t] != p.kt) return 10;
  return 0;
}

template <typename E, int MODE>
static hipError_t launch_sched(const E* x, const E* w, const E* bias, const E* res, E* y, int64_t M, int32_t N,
                               int32_t K, int epi, const LnFold& lf, hipStream_t s, float* scratch) {
  constexpr size_t slabs = 2 * (size_t)(256 + 256) * kChunks * sizeof(uint4);
  constexpr size_t epi_stage = 4 * (size_t)kEpiWaveFloats * sizeof(float);
  constexpr size_t lds = slabs > epi_stage ? slabs : epi_stage;
  static LdsAttrOnce attr_main;   // per element type and MODE
  auto kern = gemm_mfma_sched_kernel<E, 256, 256, 2, 2, MODE>;
  hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), lds, attr_main);
  if (e != hipSuccess) return e;
  const int32_t wgs = sched_wgs_per_xcd();
  // the LayerNorm-folded epilogues and the row statistics live in the main kernel only: no cutting there
  const SchedPlan plan = sched_plan(M, N, K, scratch != nullptr && MODE == kEpiPlain, wgs);
  kern<<<dim3((unsigned)(kXcds * wgs)), dim3(256), lds, s>>>(x, w, bias, res, y, M, N, K, epi, plan, scratch, lf);
  e = hipGetLastError();
  if (e != hipSuccess || plan.pieces == 1) return e;
  const int32_t max_rem = sched_max_rem(plan);
  gemm_mfma_fixup_kernel<E><<<dim3((unsigned)(kXcds * max_rem * kFixStrips)), dim3(512), 0, s>>>(scratch, bias, res, y, M, N,
                                                                                                  epi, plan);
  return hipGetLastError();
}

template <typename E>
static hipError_t launch_gemm_mfma(const E* x, const E* w, const E* bias, const E* res, E* y, int64_t M, int32_t N,
                                   int32_t K, int epi, hipStream_t s, const LnFold* fold, float* split_scratch) {
  if (M <= 0) return hipSuccess;
  static LdsAttrOnce attr_small, attr_small_fold;  // per element type
  const LnFold lf = fold != nullptr ? *fold : LnFold{};
  const bool wants_fold = epi == EPI_LNFOLD || epi == EPI_LNFOLD_GELU;
  if (wants_fold && (lf.stats == nullptr || lf.colsum == nullptr || lf.bias == nullptr)) return hipErrorInvalidValue;
  if (lf.partial != nullptr && (epi != EPI_BIAS_RESIDUAL || !gemm_emits_row_partials(M, N, K, res == y)))
    return hipErrorInvalidValue;
  if (lf.partial == nullptr && gemm_skinny_takes(M, N, K, epi))
    return launch_gemm_skinny<E>(x, w, bias, res, y, M, N, K, epi, s, split_scratch);
  if (takes_sched_kernel(M, N, K, res == y)) {
    if (wants_fold) return launch_sched<E, kEpiFolded>(x, w, bias, res, y, M, N, K, epi, lf, s, nullptr);
    if (lf.partial != nullptr) return launch_sched<E, kEpiResidualStats>(x, w, bias, res, y, M, N, K, epi, lf, s, nullptr);
    return launch_sched<E, kEpiPlain>(x, w, bias, res, y, M, N, K, epi, lf, s, split_scratch);
  }
  // A batch of a generation step too large for the few-row kernel, with scratch from the caller: K cut
  // over workgroups until there are enough of them, the parts added by a second kernel.  (Not where only
  // the aliased residual kept the shape from the 256x256 kernel: the scratch was sized for that one.)
  if (split_scratch != nullptr && !wants_fold && lf.partial == nullptr && !takes_sched_kernel(M, N, K, false)) {
    int32_t tile, ks;
    gemm_split_plan(M, N, K, &tile, &ks);
    if (ks > 1) {
      LnFold sp;
      sp.partial = split_scratch;
      static LdsAttrOnce attr_s64, attr_s128;
      hipError_t e = tile == 64
          ? launch_tiles<E>(gemm_mfma_tile_kernel<E, 64, 64, 2, 2, 2>, attr_s64, 64, 64, 256,
                            2 * (size_t)(64 + 64) * kChunks * sizeof(uint4), x, w, bias, res, y, M, N, K, epi, sp, s, ks)
          : launch_tiles<E>(gemm_mfma_tile_kernel<E, 128, 128, 2, 2, 2>, attr_s128, 128, 128, 256,
                            2 * (size_t)(128 + 128) * kChunks * sizeof(uint4), x, w, bias, res, y, M, N, K, epi, sp, s, ks);
      if (e != hipSuccess) return e;
      return launch_partial_reduce<E>(split_scratch, ks, bias, res, y, M, N, epi, s);
    }
  }
  // Few 128x128 tiles leave most of the 256 CUs idle: 64x64 tiles give four times as many workgroups
  // (measured: 593 x 1024 x 4096 44 -> 33 us, 128 x 15360 x 5120 60 -> 44 us).
  const int64_t tiles128 = ((M + 127) / 128) * ((N + 127) / 128);
  if (tiles128 < 128 && !wants_fold) {
    static LdsAttrOnce attr_64;
    return launch_tiles<E>(gemm_mfma_tile_kernel<E, 64, 64, 2, 2, 0>, attr_64, 64, 64, 256,
                           2 * (size_t)(64 + 64) * kChunks * sizeof(uint4), x, w, bias, res, y, M, N, K, epi, lf, s);
  }
  if (wants_fold)
    return launch_tiles<E>(gemm_mfma_tile_kernel<E, 128, 128, 2, 2, 1>, attr_small_fold, 128, 128, 256,
                           2 * (size_t)(128 + 128) * kChunks * sizeof(uint4), x, w, bias, res, y, M, N, K, epi, lf, s);
  return launch_tiles<E>(gemm_mfma_tile_kernel<E, 128, 128, 2, 2, 0>, attr_small, 128, 128, 256,
                         2 * (size_t)(128 + 128) * kChunks * sizeof(uint4), x, w, bias, res, y, M, N, K, epi, lf, s);
}

hipError_t launch_gemm_bf16(const bf16_t* x, const bf16_t* w, const bf16_t* bias, const bf16_t* res, bf16_t* y,
                            int64_t M, int32_t N, int32_t K, int epi, hipStream_t s, const LnFold* fold,
                            float* split_scratch) {
  return launch_gemm_mfma<bf16_t>(x, w, bias, res, y, M, N, K, epi, s, fold, split_scratch);
}

hipError_t launch_gemm_f16(const f16_t* x, const f16_t* w, const f16_t* bias, const f16_t* res, f16_t* y, int64_t M,
                           int32_t N, int32_t K, int epi, hipStream_t s, const LnFold* fold, float* split_scratch) {
  return launch_gemm_mfma<f16_t>(x, w, bias, res, y, M, N, K, epi, s, fold, split_scratch);
}

}  // namespace energon
