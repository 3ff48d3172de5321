// bf16 linear layer  y[M,N] = epilogue(x[M,K] W[N,K]^T + b)  on packed rows: the dense
// contractions that the paper (Sec. 3.1, Sec. 5.5) reports as >95 % of a large layer's time
// and that the padding removal (Sec. 4.3) shrinks from B*S rows to T rows.
//
// Design for gfx950:
//  * both operands are contiguous along K, so x rows feed the MFMA A operand and W rows the
//    B operand with the same 16-byte chunks; v_mfma_f32_32x32x16_bf16, fp32 accumulators;
//  * a BM x BN output tile per workgroup, K walked in slabs of 64 (128 bytes per row), two
//    slab buffers in LDS;
//  * an LDS row is 8 chunks of 16 bytes; chunk c of row r is stored in slot c ^ swz(r), so the
//    32 rows a wavefront reads for one MFMA operand fall in distinct banks (measured: zero bank
//    conflicts).  Slabs are moved in 1 KiB groups = 8 rows x 8 slots in lane order, the lane that
//    lands in slot s of row r fetching chunk s ^ swz(r): full 128-byte lines on the global side;
//  * workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2, so the id is
//    remapped to give every XCD a contiguous run of tiles, ordered in bands of 8 row tiles:
//    the 32 tiles resident on an XCD form an 8 x 4 block that shares x and W slabs in that L2;
//  * epilogue in fp32: + bias, GeLU(erf) or + residual, one rounding to bf16.
// Two kernels:
//  * gemm_bf16_sched_kernel, 256x256 tile, 4 wavefronts x 128x128 with the 256 accumulators in
//    AGPRs, slab loop hand-scheduled; slab chunks are fetched into registers four slabs ahead and
//    written to LDS two slabs ahead (a two-slab load window); edge tiles are shifted inwards, so
//    nothing is clamped or predicated; the epilogue goes through LDS and leaves as 16-byte stores;
//  * gemm_bf16_tile_kernel, compiler-scheduled, direct-to-LDS loads (global_load_lds_dwordx4),
//    clamped loads and predicated stores: used with 128x128 tiles for everything the first
//    kernel does not take (small or ragged-below-one-tile problems, odd slab counts).
#include "common.h"

namespace energon {

constexpr int BK = 64;            // K elements per slab
constexpr int kChunks = BK / 8;   // 16-byte chunks per LDS row
constexpr int kXcds = 8;
constexpr int kGroupM = 8;        // row tiles per band

#ifdef ENERGON_GEMM_TIMING  // development aid, never defined in the library build
__device__ long long* g_gemm_timing;
#define ENERGON_STAMP(i) do { if (threadIdx.x == 0) g_gemm_timing[blockIdx.x * 4 + (i)] = wall_clock64(); } while (0)
#else
#define ENERGON_STAMP(i) do { } while (0)
#endif

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

// Epilogue of one wavefront's 128x128 tile through LDS, for tiles that lie wholly inside the
// matrix.  The accumulators go to LDS as fp32 (64 rows at a time, rows padded to 136 floats so
// the two half-wavefronts of a store hit different banks); each lane then owns 8 consecutive
// columns of a row: bias, GeLU / residual are applied there in fp32 and the row segment leaves as
// one 16-byte store, 16 lanes per 256-byte row segment.  One rounding, full-line writes.
constexpr int kEpiLd = 136;
constexpr int kEpiWaveFloats = 64 * kEpiLd;
__device__ __forceinline__ void store_tile_coalesced(const f32x16 (&acc)[4][4], const bf16_t* __restrict__ bias,
                                                     const bf16_t* res, bf16_t* y, int32_t N, int epi, int64_t mw,
                                                     int32_t nw, int lane, float* stage) {
  const int lrow = lane & 31, lhalf = lane >> 5;
  const int rr = lane >> 4, c8 = (lane & 15) * 8;
  float bv[8];
  if (bias != nullptr) {
    const bf16x8 b8 = *reinterpret_cast<const bf16x8*>(bias + nw + c8);
#pragma unroll
    for (int q = 0; q < 8; ++q) bv[q] = static_cast<float>(b8[q]);
  } else {
#pragma unroll
    for (int q = 0; q < 8; ++q) bv[q] = 0.f;
  }
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    __syncthreads();  // the slab buffers (first pass) / the previous pass's rows are no longer read
#pragma unroll
    for (int ii = 0; ii < 2; ++ii)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e)
          stage[(ii * 32 + (e >> 2) * 8 + lhalf * 4 + (e & 3)) * kEpiLd + j * 32 + lrow] = acc[pass * 2 + ii][j][e];
    __syncthreads();
#pragma unroll 4
    for (int it = 0; it < 16; ++it) {
      const int r = it * 4 + rr;
      const float4 lo = *reinterpret_cast<const float4*>(&stage[r * kEpiLd + c8]);
      const float4 hi = *reinterpret_cast<const float4*>(&stage[r * kEpiLd + c8 + 4]);
      float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
      const size_t off = (size_t)(mw + pass * 64 + r) * N + nw + c8;
#pragma unroll
      for (int q = 0; q < 8; ++q) v[q] += bv[q];
      if (epi == EPI_BIAS_GELU) {
#pragma unroll
        for (int q = 0; q < 8; ++q) v[q] = gelu_erf(v[q]);
      }
      if (epi == EPI_BIAS_RESIDUAL) {
        const bf16x8 r8 = *reinterpret_cast<const bf16x8*>(res + off);
#pragma unroll
        for (int q = 0; q < 8; ++q) v[q] += static_cast<float>(r8[q]);
      }
      bf16x8 o;
#pragma unroll
      for (int q = 0; q < 8; ++q) o[q] = static_cast<bf16_t>(v[q]);
      *reinterpret_cast<bf16x8*>(y + off) = o;
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
// The slab loop is written as ordered inline-asm statements so that the issue order is exactly
// the one below (the compiler otherwise re-serialises LDS reads and MFMAs, and it must not copy
// or spill a register whose load is still in flight).  One wavefront per SIMD, 128x128 per
// wavefront.  Per slab of 64 along K, four steps of 16; every step issues 16 MFMAs and, slotted
// between them, the 8 LDS reads of the next step's operands, 4 global loads and 4 LDS writes
// (see ENERGON_STEP and ENERGON_SLAB).  One barrier per slab, in the shadow of queued MFMAs; a
// fetched chunk has two slab times to arrive.
// What the compiler cannot see inside asm statements it cannot guard: this code itself keeps
// the wait states between an MFMA and the first read of its result (end of the slab loop) and
// between a register write and an MFMA reading it (accumulator zeroing).
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
  // Ragged edges: the last tile of a row / column of tiles is shifted back so that it ends at
  // M / N (needs M >= BM, N >= BN).  It overlaps its neighbour; both compute bit-identical values
  // for the shared elements, so no load is clamped and no store is predicated.
  if (m0 > M - BM) m0 = M - BM;
  if (n0 > N - BN) n0 = N - BN;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, kept in an SGPR
  const int wm0 = (wave / WN) * WTM, wn0 = (wave % WN) * WTN;

  // Row group g (8 rows, 1 KiB of LDS) of a slab is fetched by wavefront g % 4; lane l fetches
  // the chunk that the swizzle puts in slot l % 8 of row l / 8.  swz(row) depends on row % 16,
  // i.e. on (l / 8) and the parity of the group = parity of the wavefront: the lane's byte offset
  // inside its group is the same for every group, and the group bases are scalar.
  const uint32_t voff = ((uint32_t)(lane >> 3) * (uint32_t)K + (uint32_t)(((lane & 7) ^ swz((wave & 1) * 8 + (lane >> 3))) * 8)) * 2u;
  const char* xbase = reinterpret_cast<const char*>(x + ((size_t)m0 + 8 * wave) * K);
  const char* wbase = reinterpret_cast<const char*>(w + ((size_t)n0 + 8 * wave) * K);
  const size_t gstride = (size_t)(8 * NW) * K * 2;  // bytes between consecutive groups of one wavefront

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
  // The compiler sees no MFMA (they are inside asm statements) and so adds no wait states between
  // a register write and an MFMA that reads it: have the zeros written here, before the prologue.
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) asm volatile("" : "+a"(acc[i][j]));

  const int KT = K / BK;

  // Register-staged slab loads with a two-slab window.  Load i of a slab (i < GA: x rows, else
  // W rows) fetches this lane's 16-byte chunk of row group (wave + i*NW) into rs[slab & 1][i]; two
  // slabs later it is written to the LDS buffer that has just been freed.
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  u32x4 rs0[GA + GB], rs1[GA + GB];
  const uint32_t wa0 = (uint32_t)wave * 1024u + (uint32_t)lane * 16u;  // LDS byte address of group `wave`, buffer 0
  const uint32_t wa1 = wa0 + 0x10000u;                                    // ... buffer 1
#define ENERGON_GLOAD(dst, i, kt_)                                                                      \
  asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(dst) : "v"(voff),                                \
               "s"(((i) < GA ? xbase + (i) * gstride : wbase + ((i) - GA) * gstride) + (size_t)(kt_) * (BK * 2)) \
               : "memory")
#define ENERGON_LWRITE(src, i, WA)                                                                      \
  asm volatile("ds_write_b128 %0, %1 offset:%2" : : "v"(WA), "v"(src),                                   \
               "n"(((i) < GA ? (i) * NW * 1024 : BM * 128 + ((i) - GA) * NW * 1024)) : "memory")

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

// One step: 16 MFMAs on (CA_, CB_) with, slotted between them,
//  * the 8 LDS reads of (NA, NB) for step nks (after MFMAs 1..8);
//  * after MFMAs 5..8, the reload of the four staged registers RL[il..il+3] with slab kl_.  Their
//    previous contents were written to LDS in the step before; an LDS write reads its data
//    registers only when it executes, so they may be overwritten only once that write has
//    completed: LDS operations complete in order, hence the lgkmcnt(4) after the first 4 reads;
//  * after MFMAs 9..12, the write of RW[iw..iw+3] (fetched 32 loads ago: loads return in order,
//    so all but the newest 28 have landed) to the LDS buffer addressed by WA.
#define ENERGON_STEP(CA_, CB_, NA, NB, nks, RL, il, kl_, RW, iw, WA)                                    \
  do {                                                                                                  \
    ENERGON_MFMA(acc[0][0], CA_[0], CB_[0]); ENERGON_DS_READ(NA[0], aaddr[nks], 0);                      \
    ENERGON_MFMA(acc[0][1], CA_[0], CB_[1]); ENERGON_DS_READ(NB[0], baddr[nks], 0);                      \
    ENERGON_MFMA(acc[0][2], CA_[0], CB_[2]); ENERGON_DS_READ(NB[1], baddr[nks], 4096);                   \
    ENERGON_MFMA(acc[0][3], CA_[0], CB_[3]); ENERGON_DS_READ(NB[2], baddr[nks], 8192);                   \
    asm volatile("s_waitcnt lgkmcnt(4)" ::: "memory");                                                  \
    ENERGON_MFMA(acc[1][0], CA_[1], CB_[0]); ENERGON_DS_READ(NB[3], baddr[nks], 12288);                  \
    ENERGON_GLOAD(RL[(il) + 0], (il) + 0, kl_);                                                          \
    ENERGON_MFMA(acc[1][1], CA_[1], CB_[1]); ENERGON_DS_READ(NA[1], aaddr[nks], 4096);                   \
    ENERGON_GLOAD(RL[(il) + 1], (il) + 1, kl_);                                                          \
    ENERGON_MFMA(acc[1][2], CA_[1], CB_[2]); ENERGON_DS_READ(NA[2], aaddr[nks], 8192);                   \
    ENERGON_GLOAD(RL[(il) + 2], (il) + 2, kl_);                                                          \
    ENERGON_MFMA(acc[1][3], CA_[1], CB_[3]); ENERGON_DS_READ(NA[3], aaddr[nks], 12288);                  \
    ENERGON_GLOAD(RL[(il) + 3], (il) + 3, kl_);                                                          \
    asm volatile("s_waitcnt vmcnt(28)" ::: "memory");                                                   \
    ENERGON_MFMA(acc[2][0], CA_[2], CB_[0]); ENERGON_LWRITE(RW[(iw) + 0], (iw) + 0, WA);                 \
    ENERGON_MFMA(acc[2][1], CA_[2], CB_[1]); ENERGON_LWRITE(RW[(iw) + 1], (iw) + 1, WA);                 \
    ENERGON_MFMA(acc[2][2], CA_[2], CB_[2]); ENERGON_LWRITE(RW[(iw) + 2], (iw) + 2, WA);                 \
    ENERGON_MFMA(acc[2][3], CA_[2], CB_[3]); ENERGON_LWRITE(RW[(iw) + 3], (iw) + 3, WA);                 \
    ENERGON_MFMA(acc[3][0], CA_[3], CB_[0]); ENERGON_MFMA(acc[3][1], CA_[3], CB_[1]);                    \
    ENERGON_MFMA(acc[3][2], CA_[3], CB_[2]); ENERGON_MFMA(acc[3][3], CA_[3], CB_[3]);                    \
  } while (0)

  static_assert(TM == 4 && TN == 4 && GA + GB == 16, "the hand schedule is written for 4 x (128x128)");

  const int klast = KT - 1;
  // Prologue.  Afterwards: slab 0 complete in buffer 0, chunks 0..3 of slab 1 in buffer 1,
  // rs1[4..15] = rest of slab 1 (landed), rs0 = slab 2 in flight, rs1[0..3] free (their LDS
  // writes have completed).
#pragma unroll
  for (int i = 0; i < 16; ++i) ENERGON_GLOAD(rs0[i], i, 0);
#pragma unroll
  for (int i = 0; i < 16; ++i) ENERGON_GLOAD(rs1[i], i, (1 < klast ? 1 : klast));
  asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
#pragma unroll
  for (int i = 0; i < 16; ++i) ENERGON_LWRITE(rs0[i], i, wa0);
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");  // slab 1 landed; rs0 has been read
#pragma unroll
  for (int i = 0; i < 16; ++i) ENERGON_GLOAD(rs0[i], i, (2 < klast ? 2 : klast));
#pragma unroll
  for (int i = 0; i < 4; ++i) ENERGON_LWRITE(rs1[i], i, wa1);
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  ENERGON_READ_SET(fa0, fb0, 0);
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");

  // Slab kt is consumed from buffer kt&1.  RN = rs[(kt+1)&1] holds slab kt+1: its chunks 0..3
  // reached the other buffer in the previous slab's step 3, chunks 4..15 follow in steps 0..2,
  // four per step, and each group of four registers is refilled with slab kt+3 one step after
  // it was written out.  After the barrier this buffer is free, and step 3 moves chunks 0..3 of
  // slab kt+2 from RC = rs[kt&1] into it.  LDS traffic is thereby even over the steps: 8 reads
  // + 4 writes per wavefront in each.  Two slabs per trip so that register sets and buffer
  // addresses are static.
#define ENERGON_SLAB(RC, RN, WC, WN_, kt_)                                                              \
  {                                                                                                     \
    const int kl3 = (kt_) + 3 < KT ? (kt_) + 3 : klast;                                                 \
    ENERGON_STEP(fa0, fb0, fa1, fb1, 1, RN, 0, kl3, RN, 4, WN_);                                        \
    asm volatile("s_waitcnt lgkmcnt(4)" ::: "memory"); /* LDS returns in order: the reads are back */  \
    ENERGON_STEP(fa1, fb1, fa0, fb0, 2, RN, 4, kl3, RN, 8, WN_);                                        \
    asm volatile("s_waitcnt lgkmcnt(4)" ::: "memory");                                                  \
    ENERGON_STEP(fa0, fb0, fa1, fb1, 3, RN, 8, kl3, RN, 12, WN_);                                       \
    /* this wavefront has read all of the current buffer and written all of slab kt+1 */                \
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");                                                  \
    __builtin_amdgcn_s_barrier();                                                                       \
    _Pragma("unroll") for (int ks = 0; ks < 4; ++ks) { aaddr[ks] ^= 0x10000u; baddr[ks] ^= 0x10000u; }  \
    ENERGON_STEP(fa1, fb1, fa0, fb0, 0, RN, 12, kl3, RC, 0, WC);                                        \
    asm volatile("s_waitcnt lgkmcnt(4)" ::: "memory");                                                  \
  }
  for (int kt = 0; kt < KT; kt += 2) {  // KT is even (K % 128 == 0, checked by the launcher)
    ENERGON_SLAB(rs0, rs1, wa0, wa1, kt)
    ENERGON_SLAB(rs1, rs0, wa1, wa0, kt + 1)
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
  // Outstanding loads (the clamped refetches of the last slabs) and LDS writes.
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
#undef ENERGON_GLOAD
#undef ENERGON_LWRITE
#undef ENERGON_STEP
#undef ENERGON_READ_SET

  // The epilogue's per-lane addresses must not be computed (and kept live) above the slab loop,
  // where every VGPR is spoken for: route the lane id through an ordered asm statement.
  ENERGON_STAMP(2);
  int lane_e = lane;
  asm volatile("" : "+v"(lane_e));
  store_tile_coalesced(acc, bias, res, y, N, epi, m0 + wm0, n0 + wn0, lane_e,
                       reinterpret_cast<float*>(smem) + wave * kEpiWaveFloats);
  ENERGON_STAMP(3);
}

template <typename Kern>
static hipError_t launch_tiles(Kern kern, bool& attr_set, int BM, int BN, int threads, size_t lds, const bf16_t* x,
                               const bf16_t* w, const bf16_t* bias, const bf16_t* res, bf16_t* y, int64_t M, int32_t N,
                               int32_t K, int epi, hipStream_t s) {
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
  // the 256x256 kernel needs whole tiles to shift at the edges, an even number of slabs, and
  // enough tiles for most of the 256 CUs
  // (shifted edge tiles overlap their neighbours: with the residual aliasing y, an overlapped
  // element could be read after the neighbour's write, so that case needs whole tiles)
  const bool overlap_safe = res != y || (M % 256 == 0 && N % 256 == 0);
  if (M >= 256 && N >= 256 && K % 128 == 0 && big_tiles >= 192 && overlap_safe) {
    constexpr size_t slabs = 2 * (size_t)(256 + 256) * kChunks * sizeof(uint4);
    constexpr size_t epi_stage = 4 * (size_t)kEpiWaveFloats * sizeof(float);
    return launch_tiles(gemm_bf16_sched_kernel<256, 256, 2, 2>, attr_big, 256, 256, 256,
                        slabs > epi_stage ? slabs : epi_stage, x, w, bias, res, y, M, N, K, epi, s);
  }
  return launch_tiles(gemm_bf16_tile_kernel<128, 128, 2, 2>, attr_small, 128, 128, 256,
                      2 * (size_t)(128 + 128) * kChunks * sizeof(uint4), x, w, bias, res, y, M, N, K, epi, s);
}

}  // namespace energon
