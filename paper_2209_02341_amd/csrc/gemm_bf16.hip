// bf16 linear layer  y[M,N] = epilogue(x[M,K] W[N,K]^T + b)  on packed rows: the dense
// contractions that the paper (Sec. 3.1, Sec. 5.5) reports as >95 % of a large layer's time
// and that the padding removal (Sec. 4.3) shrinks from B*S rows to T rows.
//
// Design for gfx950:
//  * both operands are contiguous along K, so x rows feed the MFMA A operand and W rows the
//    B operand with the same 16-byte chunks; v_mfma_f32_32x32x16_bf16, fp32 accumulators;
//  * a BM x BN output tile per workgroup, K walked in slabs of 64 (128 bytes per row), two
//    slab buffers in LDS filled straight from global memory (global_load_lds_dwordx4: no
//    staging registers, no LDS store instructions);
//  * one such load writes 1 KiB of LDS = 8 rows x 8 chunks in lane order, so the swizzle is
//    applied on the global side: the lane that lands in slot s of row r fetches chunk
//    s ^ swz(r).  The 32 rows a wavefront reads for one MFMA operand then fall in distinct
//    banks (measured: zero bank conflicts);
//  * workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2, so the id is
//    remapped to give every XCD a contiguous run of tiles, ordered in bands of 8 row tiles:
//    the 32 tiles resident on an XCD form an 8 x 4 block that shares x and W slabs in that L2;
//  * ragged M (T is arbitrary) and ragged N: loads clamp the row index, stores are predicated;
//  * epilogue in fp32 on the accumulators: + bias, GeLU(erf) or + residual, one rounding.
// Two kernels: a hand-scheduled 256x256 tile (4 wavefronts x 128x128, accumulators in AGPRs)
// for the large layer shapes, and a compiler-scheduled template used with 128x128 tiles when
// the problem has too few 256x256 tiles to fill the 256 CUs.
#include "common.h"

namespace energon {

constexpr int BK = 64;            // K elements per slab
constexpr int kChunks = BK / 8;   // 16-byte chunks per LDS row
constexpr int kXcds = 8;
constexpr int kGroupM = 8;        // row tiles per band

typedef __attribute__((address_space(1))) const void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

__device__ __forceinline__ int swz(int row) { return (row & 7) ^ ((row >> 3) & 1); }

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
template <int TM, int TN>
__device__ __forceinline__ void store_tile(const f32x16 (&acc)[TM][TN], const bf16_t* __restrict__ bias,
                                           const bf16_t* res, bf16_t* y, int64_t M, int32_t N, int epi, int64_t mw,
                                           int32_t nw, int lane) {
  const int lrow = lane & 31, lhalf = lane >> 5;
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int32_t n = nw + j * 32 + lrow;
    const bool n_ok = n < N;
    const float bv = (bias != nullptr && n_ok) ? static_cast<float>(bias[n]) : 0.f;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int64_t m = mw + i * 32 + (e >> 2) * 8 + lhalf * 4 + (e & 3);
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

// ---- compiler-scheduled tile kernel ---------------------------------------------------------
template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(WM* WN * 64) void gemm_bf16_tile_kernel(const bf16_t* __restrict__ x,
                                                                     const bf16_t* __restrict__ w,
                                                                     const bf16_t* __restrict__ bias,
                                                                     const bf16_t* res, bf16_t* y, int64_t M,
                                                                     int32_t N, int32_t K, int epi, int32_t tiles_m,
                                                                     int32_t tiles_n) {
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
  const char* xbase = reinterpret_cast<const char*>(x + (size_t)m0 * K);
  const char* wbase = reinterpret_cast<const char*>(w + (size_t)n0 * K);
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
  const int KT = K / BK;

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
    bf16x8 af[2][TM], bfr[2][TN];
#pragma unroll
    for (int t = 0; t < TM; ++t) af[0][t] = *reinterpret_cast<const bf16x8*>(&cur[fa[t] + (lhalf ^ fsa[t])]);
#pragma unroll
    for (int t = 0; t < TN; ++t) bfr[0][t] = *reinterpret_cast<const bf16x8*>(&cur[fb[t] + (lhalf ^ fsb[t])]);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      const int p = ks & 1;
      if (ks + 1 < BK / 16) {
        const int c = (ks + 1) * 2 + lhalf;
#pragma unroll
        for (int t = 0; t < TM; ++t) af[p ^ 1][t] = *reinterpret_cast<const bf16x8*>(&cur[fa[t] + (c ^ fsa[t])]);
#pragma unroll
        for (int t = 0; t < TN; ++t) bfr[p ^ 1][t] = *reinterpret_cast<const bf16x8*>(&cur[fb[t] + (c ^ fsb[t])]);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[p][i], bfr[p][j], acc[i][j], 0, 0, 0);
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

  store_tile<TM, TN>(acc, bias, res, y, M, N, epi, m0 + wm0, n0 + wn0, lane);
}

// ---- hand-scheduled 256x256 kernel ----------------------------------------------------------
// Same tiling and LDS layout, but the slab loop is written as ordered inline-asm
// statements so that the issue order is exactly the one below (the compiler otherwise re-serialises
// LDS reads and MFMAs).  One wavefront per SIMD (4 per workgroup), 128x128 per wavefront,
// accumulators in AGPRs.  Per slab of 64 along K, four steps of 16:
//   step s   : 16 MFMAs on operand set s, with the 8 LDS reads of step s+1 slotted between them
//   before step 3: wait for this wavefront's LDS reads and its direct-to-LDS loads of the NEXT
//              slab, barrier; now the current buffer is free, so the loads of slab kt+2 are issued
//              into it, and step 3's MFMAs overlap the reads of the next slab's step 0.
// The barrier thus sits in the shadow of queued MFMAs and the loads have a whole slab to land.
#define ENERGON_DS_READ(dst, addr, off) \
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(off) : "memory")
#define ENERGON_MFMA(acc, a, b) \
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b))

template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(WM* WN * 64) void gemm_bf16_sched_kernel(const bf16_t* __restrict__ x,
                                                                    const bf16_t* __restrict__ w,
                                                                    const bf16_t* __restrict__ bias,
                                                                    const bf16_t* res, bf16_t* y, int64_t M,
                                                                    int32_t N, int32_t K, int epi, int32_t tiles_m,
                                                                    int32_t tiles_n) {
  constexpr int NW = WM * WN;
  constexpr int WTM = BM / WM, WTN = BN / WN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int GA = BM / 8 / NW, GB = BN / 8 / NW;
  static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "row groups must divide evenly");
  static_assert((BM + BN) * 128 == 65536, "stage stride is assumed to be 64 KiB");
  extern __shared__ uint4 smem[];  // [2][BM + BN][kChunks]

  int64_t m0;
  int32_t n0;
  if (!tile_origin<BM, BN>(tiles_m, tiles_n, m0, n0)) return;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, kept in an SGPR
  const int wm0 = (wave / WN) * WTM, wn0 = (wave % WN) * WTN;

  const char* xbase = reinterpret_cast<const char*>(x + (size_t)m0 * K);
  const char* wbase = reinterpret_cast<const char*>(w + (size_t)n0 * K);
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

  // LDS byte address of this lane's operand chunk for step ks; tile t adds t*4096 (32 rows).
  // swz depends on row % 16 only and all tile rows are congruent to lrow mod 32.
  const int lrow = lane & 31, lhalf = lane >> 5;
  uint32_t aaddr[4], baddr[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const uint32_t chunk = (uint32_t)((ks * 2 + lhalf) ^ swz(lrow)) * 16u;
    aaddr[ks] = (uint32_t)(wm0 + lrow) * 128u + chunk;
    baddr[ks] = (uint32_t)(BM + wn0 + lrow) * 128u + chunk;
  }

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  constexpr int kStage = (BM + BN) * kChunks;
  const int KT = K / BK;

  // direct-to-LDS load number i of a slab (i < GA: x rows, else W rows) into `stage`
  auto issue_one = [&](int i, int kt, int stage) {
    uint4* base = smem + stage * kStage;
    if (i < GA)
      __builtin_amdgcn_global_load_lds((gptr_t)(xbase + (size_t)kt * (BK * 2) + oa[i]),
                                       (lptr_t)(base + (wave + i * NW) * 64), 16, 0, 0);
    else
      __builtin_amdgcn_global_load_lds((gptr_t)(wbase + (size_t)kt * (BK * 2) + ob[i - GA]),
                                       (lptr_t)(base + BM * kChunks + (wave + (i - GA) * NW) * 64), 16, 0, 0);
  };
  auto issue = [&](int kt, int stage) {
#pragma unroll
    for (int i = 0; i < GA + GB; ++i) issue_one(i, kt, stage);
  };

  bf16x8 fa0[TM], fb0[TN], fa1[TM], fb1[TN];  // operand sets for even / odd steps

#define ENERGON_READ_SET(FA, FB, ks)                                      \
  do {                                                                    \
    ENERGON_DS_READ(FA[0], aaddr[ks], 0);                                 \
    ENERGON_DS_READ(FB[0], baddr[ks], 0);                                 \
    ENERGON_DS_READ(FB[1], baddr[ks], 4096);                              \
    ENERGON_DS_READ(FB[2], baddr[ks], 8192);                              \
    ENERGON_DS_READ(FB[3], baddr[ks], 12288);                             \
    ENERGON_DS_READ(FA[1], aaddr[ks], 4096);                              \
    ENERGON_DS_READ(FA[2], aaddr[ks], 8192);                              \
    ENERGON_DS_READ(FA[3], aaddr[ks], 12288);                             \
  } while (0)

// 16 MFMAs on (CA, CB); the 8 reads of (NA, NB) for step nks go after MFMAs 1..8
#define ENERGON_STEP(CA_, CB_, NA, NB, nks)                               \
  do {                                                                    \
    ENERGON_MFMA(acc[0][0], CA_[0], CB_[0]); ENERGON_DS_READ(NA[0], aaddr[nks], 0);      \
    ENERGON_MFMA(acc[0][1], CA_[0], CB_[1]); ENERGON_DS_READ(NB[0], baddr[nks], 0);      \
    ENERGON_MFMA(acc[0][2], CA_[0], CB_[2]); ENERGON_DS_READ(NB[1], baddr[nks], 4096);   \
    ENERGON_MFMA(acc[0][3], CA_[0], CB_[3]); ENERGON_DS_READ(NB[2], baddr[nks], 8192);   \
    ENERGON_MFMA(acc[1][0], CA_[1], CB_[0]); ENERGON_DS_READ(NB[3], baddr[nks], 12288);  \
    ENERGON_MFMA(acc[1][1], CA_[1], CB_[1]); ENERGON_DS_READ(NA[1], aaddr[nks], 4096);   \
    ENERGON_MFMA(acc[1][2], CA_[1], CB_[2]); ENERGON_DS_READ(NA[2], aaddr[nks], 8192);   \
    ENERGON_MFMA(acc[1][3], CA_[1], CB_[3]); ENERGON_DS_READ(NA[3], aaddr[nks], 12288);  \
    ENERGON_MFMA(acc[2][0], CA_[2], CB_[0]); ENERGON_MFMA(acc[2][1], CA_[2], CB_[1]);    \
    ENERGON_MFMA(acc[2][2], CA_[2], CB_[2]); ENERGON_MFMA(acc[2][3], CA_[2], CB_[3]);    \
    ENERGON_MFMA(acc[3][0], CA_[3], CB_[0]); ENERGON_MFMA(acc[3][1], CA_[3], CB_[1]);    \
    ENERGON_MFMA(acc[3][2], CA_[3], CB_[2]); ENERGON_MFMA(acc[3][3], CA_[3], CB_[3]);    \
  } while (0)

// step 3: the reads go after MFMAs 1..8 as above, the 16 direct-to-LDS loads of the slab after
// next go two at a time after MFMAs 9..16
#define ENERGON_STEP_LOAD(CA_, CB_, NA, NB, nks, kt_, st_)                              \
  do {                                                                                  \
    ENERGON_MFMA(acc[0][0], CA_[0], CB_[0]); ENERGON_DS_READ(NA[0], aaddr[nks], 0);      \
    ENERGON_MFMA(acc[0][1], CA_[0], CB_[1]); ENERGON_DS_READ(NB[0], baddr[nks], 0);      \
    ENERGON_MFMA(acc[0][2], CA_[0], CB_[2]); ENERGON_DS_READ(NB[1], baddr[nks], 4096);   \
    ENERGON_MFMA(acc[0][3], CA_[0], CB_[3]); ENERGON_DS_READ(NB[2], baddr[nks], 8192);   \
    ENERGON_MFMA(acc[1][0], CA_[1], CB_[0]); ENERGON_DS_READ(NB[3], baddr[nks], 12288);  \
    ENERGON_MFMA(acc[1][1], CA_[1], CB_[1]); ENERGON_DS_READ(NA[1], aaddr[nks], 4096);   \
    ENERGON_MFMA(acc[1][2], CA_[1], CB_[2]); ENERGON_DS_READ(NA[2], aaddr[nks], 8192);   \
    ENERGON_MFMA(acc[1][3], CA_[1], CB_[3]); ENERGON_DS_READ(NA[3], aaddr[nks], 12288);  \
    ENERGON_MFMA(acc[2][0], CA_[2], CB_[0]); issue_one(0, kt_, st_); issue_one(1, kt_, st_);   \
    ENERGON_MFMA(acc[2][1], CA_[2], CB_[1]); issue_one(2, kt_, st_); issue_one(3, kt_, st_);   \
    ENERGON_MFMA(acc[2][2], CA_[2], CB_[2]); issue_one(4, kt_, st_); issue_one(5, kt_, st_);   \
    ENERGON_MFMA(acc[2][3], CA_[2], CB_[3]); issue_one(6, kt_, st_); issue_one(7, kt_, st_);   \
    ENERGON_MFMA(acc[3][0], CA_[3], CB_[0]); issue_one(8, kt_, st_); issue_one(9, kt_, st_);   \
    ENERGON_MFMA(acc[3][1], CA_[3], CB_[1]); issue_one(10, kt_, st_); issue_one(11, kt_, st_); \
    ENERGON_MFMA(acc[3][2], CA_[3], CB_[2]); issue_one(12, kt_, st_); issue_one(13, kt_, st_); \
    ENERGON_MFMA(acc[3][3], CA_[3], CB_[3]); issue_one(14, kt_, st_); issue_one(15, kt_, st_); \
  } while (0)

  static_assert(TM == 4 && TN == 4 && GA + GB == 16, "the hand schedule is written for 4 x (128x128)");

  issue(0, 0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  issue(KT > 1 ? 1 : 0, 1);
  ENERGON_READ_SET(fa0, fb0, 0);
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");

  for (int kt = 0; kt < KT; ++kt) {
    ENERGON_STEP(fa0, fb0, fa1, fb1, 1);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    ENERGON_STEP(fa1, fb1, fa0, fb0, 2);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    ENERGON_STEP(fa0, fb0, fa1, fb1, 3);
    // all reads of the current buffer are done, the next slab has landed
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    // Step 3 overlaps the reads of the next slab's step 0 (other buffer) and the loads of slab
    // kt+2 into the buffer just freed.  Past the end the last slab is fetched again: it lands in
    // a buffer nobody reads any more, and the final wait below drains it.
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) { aaddr[ks] ^= 0x10000u; baddr[ks] ^= 0x10000u; }
    const int kload = kt + 2 < KT ? kt + 2 : KT - 1;
    ENERGON_STEP_LOAD(fa1, fb1, fa0, fb0, 0, kload, kt & 1);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  }
  // Drain: outstanding direct-to-LDS loads, and the MFMA pipeline before any accumulator is read
  // (the accumulators are operands so that no read of them can be placed above this statement).
  asm volatile("s_waitcnt vmcnt(0)\n\ts_nop 15\n\ts_nop 15"
               : "+a"(acc[0][0]), "+a"(acc[0][1]), "+a"(acc[0][2]), "+a"(acc[0][3]), "+a"(acc[1][0]), "+a"(acc[1][1]),
                 "+a"(acc[1][2]), "+a"(acc[1][3]), "+a"(acc[2][0]), "+a"(acc[2][1]), "+a"(acc[2][2]), "+a"(acc[2][3]),
                 "+a"(acc[3][0]), "+a"(acc[3][1]), "+a"(acc[3][2]), "+a"(acc[3][3])
               :
               : "memory");
#undef ENERGON_STEP_LOAD
#undef ENERGON_STEP
#undef ENERGON_READ_SET

  store_tile<TM, TN>(acc, bias, res, y, M, N, epi, m0 + wm0, n0 + wn0, lane);
}

template <typename Kern>
static hipError_t launch_tiles(Kern kern, bool& attr_set, int BM, int BN, int threads, const bf16_t* x,
                               const bf16_t* w, const bf16_t* bias, const bf16_t* res, bf16_t* y, int64_t M, int32_t N,
                               int32_t K, int epi, hipStream_t s) {
  const size_t lds = 2 * (size_t)(BM + BN) * kChunks * sizeof(uint4);
  if (!attr_set) {  // idempotent; a race between host threads only repeats the call
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int32_t tiles_m = (int32_t)((M + BM - 1) / BM), tiles_n = (N + BN - 1) / BN;
  const int64_t total = (int64_t)tiles_m * tiles_n;
  const int64_t grid = (total + kXcds - 1) / kXcds * kXcds;
  kern<<<dim3((unsigned)grid), dim3(threads), lds, s>>>(x, w, bias, res, y, M, N, K, epi, tiles_m, tiles_n);
  return hipGetLastError();
}

hipError_t launch_gemm_bf16(const bf16_t* x, const bf16_t* w, const bf16_t* bias, const bf16_t* res, bf16_t* y,
                            int64_t M, int32_t N, int32_t K, int epi, hipStream_t s) {
  if (M <= 0) return hipSuccess;
  static bool attr_big = false, attr_small = false;
  const int64_t big_tiles = ((M + 255) / 256) * ((N + 255) / 256);
  if (big_tiles >= 192)  // enough 256x256 tiles for most of the 256 CUs
    return launch_tiles(gemm_bf16_sched_kernel<256, 256, 2, 2>, attr_big, 256, 256, 256, x, w, bias, res, y, M, N, K,
                        epi, s);
  return launch_tiles(gemm_bf16_tile_kernel<128, 128, 2, 2>, attr_small, 128, 128, 256, x, w, bias, res, y, M, N, K,
                      epi, s);
}

}  // namespace energon
