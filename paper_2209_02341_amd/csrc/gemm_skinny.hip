// 16-bit linear layer for few rows (M <= 64): y[M,N] = epilogue(x[M,K] W[N,K]^T + b).
// This is the shape of a generation step, one token per sequence: every weight is used M times
// only, so the contraction is bound by streaming W from HBM once (N*K*e bytes), not by the
// matrix cores.  Design for gfx950:
//  * a workgroup owns 32 or 64 output columns (rows of W) and all of K, or 1/KS of it; its 4
//    wavefronts split that in interleaved slabs of 64 (wavefront w takes slabs w, w + 4, ...) and
//    add their partial sums through LDS at the end, in a fixed order.  With K cut over KS
//    workgroups (only where the caller provides room for KS fp32 partial results) a second small
//    kernel adds the parts in a fixed order and applies the epilogue.  Deterministic, no atomics;
//  * a slab of W (32 or 64 rows x 128 bytes) and the same slab of x (16 MT rows x 128 bytes) go
//    from global memory straight to LDS (global_load_lds_dwordx4, whole 128-byte lines) into a
//    ring that is private to the wavefront, 2 or 4 slabs deep (the depth made no measurable
//    difference): no barrier and no staging register in the streaming loop.  x is read again by every workgroup, from the L2; fetched as whole lines it
//    costs the W stream 20 % (measured in a probe: 24.7 -> 29.6 us for a 157 MB matrix), as 64-byte
//    operand gathers into registers 60 %.  The XOR swizzle of the 256x256 kernel keeps the operand
//    reads free of bank conflicts;
//  * v_mfma_f32_16x16x32: x rows are the A operand (row tiles of 16, MT of them), W rows the B
//    operand; at these sizes the matrix cores are idle most of the time by design.
#include "common.h"

namespace energon {

namespace {

typedef __attribute__((address_space(1))) const void* sk_gptr_t;
typedef __attribute__((address_space(3))) void* sk_lptr_t;

constexpr int kSkWaves = 4;     // a workgroup's share of K is split over this many wavefronts

__device__ __forceinline__ int sk_swz(int row) {
  return ((row >> 1) & 1) | (((row >> 2) & 1) << 2) | (((row >> 3) & 1) << 1);
}

// MT row tiles of x (16 rows each), NT row tiles of W (= 16 NT output columns per workgroup)
template <int MT, int NT> struct SkCfg {
  static constexpr int kBN = 16 * NT;
  static constexpr int kSlotVecs = (16 * NT + 16 * MT) * 8;      // uint4 per ring slot: W rows, then x rows
  static constexpr int kDepth = kSlotVecs * 16 <= 6144 ? 4 : 2;  // slabs in flight per wavefront
  static constexpr int kRedLd = kBN + 4;                         // floats per row of the reduction buffer:
                                                                 // rows 4 apart land 16 banks apart
  static constexpr size_t kRing = (size_t)kSkWaves * kDepth * kSlotVecs * 16;
  static constexpr size_t kRed = (size_t)kSkWaves * MT * 16 * kRedLd * sizeof(float);
  static constexpr size_t kLds = kRing > kRed ? kRing : kRed;
};

// grid = (N / BN, KS).  Workgroup (nb, kz) contracts slabs [kz * KT / KS, (kz + 1) * KT / KS) of K for
// columns 16 NT nb ..; with partial == nullptr (KS = 1) it applies the epilogue and writes y, otherwise
// it writes its fp32 sums to partial[kz][M][N] and skinny_reduce_kernel finishes the job.
template <typename E, int MT, int NT>
__global__ __launch_bounds__(kSkWaves * 64) void gemm_skinny_kernel(const E* __restrict__ x, const E* __restrict__ w,
                                                                   const E* __restrict__ bias, const E* res, E* y,
                                                                   float* __restrict__ partial, int32_t M, int32_t N,
                                                                   int32_t K, int epi) {
  static_assert(MT == 1 || MT == 2 || MT == 4, "row tiles of x");
  static_assert(NT == 2 || NT == 4, "row tiles of W");
  using Cfg = SkCfg<MT, NT>;
  constexpr int D = Cfg::kDepth, SV = Cfg::kSlotVecs, BN = Cfg::kBN, RLD = Cfg::kRedLd;
  constexpr int GW = 2 * NT, GX = 2 * MT;   // 8-row groups of W and x per slab
  constexpr int G = GW + GX;                // direct-to-LDS instructions per slab
  extern __shared__ uint4 lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int32_t n0 = blockIdx.x * BN;
  const int32_t KTs = K / 64 / (int32_t)gridDim.y;            // slabs of this workgroup
  const int32_t s0 = (int32_t)blockIdx.y * KTs;               // its first slab
  const int32_t ns = (KTs - wave + kSkWaves - 1) / kSkWaves;  // slabs of this wavefront (>= 0)

  uint4* ring = lds + wave * (D * SV);
  const int lrow = lane & 15, lq = lane >> 4;

  // A row group = 8 rows x 128 bytes in lane order, lane l landing in slot l % 8 of row l / 8 and
  // fetching the chunk the swizzle puts there (even groups are rows 0..7 of a 16-row tile, odd
  // groups rows 8..15).  Addresses are a wavefront-uniform base (first row of the group, this
  // workgroup's first slab) plus a 32-bit per-lane offset, so that advancing along K is scalar
  // arithmetic.  x rows are clamped to M - 1: rows past M are computed and dropped.
  const uint32_t row_b = (uint32_t)K * (uint32_t)sizeof(E);
  const uint32_t ch_even = (uint32_t)(((lane & 7) ^ sk_swz(lane >> 3)) * 16);
  const uint32_t ch_odd = (uint32_t)(((lane & 7) ^ sk_swz((lane >> 3) | 8)) * 16);
  const uint32_t woff_even = (uint32_t)(lane >> 3) * row_b + ch_even, woff_odd = (uint32_t)(lane >> 3) * row_b + ch_odd;
  const char* wbase = reinterpret_cast<const char*>(w + (size_t)n0 * K) + (size_t)s0 * 128;   // uniform
  const char* xbase = reinterpret_cast<const char*>(x) + (size_t)s0 * 128;                    // uniform
  uint32_t xoff[GX];
#pragma unroll
  for (int j = 0; j < GX; ++j) xoff[j] = (uint32_t)min(8 * j + (lane >> 3), M - 1) * row_b + ((j & 1) ? ch_odd : ch_even);
  // operand reads from a ring slot: row l % 16 of a 16-row tile, chunk (4 ks + l / 16) ^ swizzle
  uint32_t foff[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) foff[ks] = (uint32_t)(lrow * 8 + ((ks * 4 + lq) ^ sk_swz(lrow)));

  f32x4 acc[MT][NT];
#pragma unroll
  for (int t = 0; t < MT; ++t)
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[t][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  // slab i of this wavefront -> ring slot i % D
  auto issue = [&](int32_t slot, int32_t i) {
    const size_t kb = (size_t)(wave + i * kSkWaves) * 128;
    uint4* dst = ring + slot * SV;
#pragma unroll
    for (int j = 0; j < GW; ++j)
      __builtin_amdgcn_global_load_lds((sk_gptr_t)(wbase + (size_t)(8 * j) * row_b + kb + ((j & 1) ? woff_odd : woff_even)),
                                       (sk_lptr_t)(dst + j * 64), 16, 0, 0);
#pragma unroll
    for (int j = 0; j < GX; ++j)
      __builtin_amdgcn_global_load_lds((sk_gptr_t)(xbase + kb + xoff[j]), (sk_lptr_t)(dst + (GW + j) * 64), 16, 0, 0);
  };

  for (int32_t u = 0; u < D && u < ns; ++u) issue(u, u);
  int32_t slot = 0;
  for (int32_t i = 0; i < ns; ++i) {
    // Loads return in order.  Behind slab i's loads are those of the next D - 1 slabs while they
    // all exist; on the last D - 1 trips fewer are outstanding and the wait is for everything.
    if (i + D <= ns) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((D - 1) * G) : "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    const uint4* slab = ring + slot * SV;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      vec8<E> wb[NT], xa[MT];
#pragma unroll
      for (int j = 0; j < NT; ++j) wb[j] = *reinterpret_cast<const vec8<E>*>(&slab[j * 128 + foff[ks]]);
#pragma unroll
      for (int t = 0; t < MT; ++t) xa[t] = *reinterpret_cast<const vec8<E>*>(&slab[(NT + t) * 128 + foff[ks]]);
#pragma unroll
      for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int j = 0; j < NT; ++j) acc[t][j] = Mfma<E>::m16x16x32(xa[t], wb[j], acc[t][j]);
    }
    if (i + D < ns) {
      // the slot is refilled by the load unit, which is not ordered with this wavefront's LDS
      // reads: they must have returned first
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      issue(slot, i + D);
    }
    slot = slot + 1 == D ? 0 : slot + 1;
  }

  // Sum over the wavefronts through LDS (the rings are free once every wavefront is here; each
  // has waited for its own last load), then the epilogue: thread -> row, 4 columns.
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  __syncthreads();
  float* red = reinterpret_cast<float*>(lds);
  constexpr int kRedWave = MT * 16 * RLD;
#pragma unroll
  for (int t = 0; t < MT; ++t)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e)
        red[wave * kRedWave + (16 * t + 4 * lq + e) * RLD + 16 * j + lrow] = acc[t][j][e];
  __syncthreads();
  constexpr int TPR = BN / 4;   // threads per output row
  const int32_t c4 = (tid % TPR) * 4;
  for (int32_t m = tid / TPR; m < MT * 16 && m < M; m += kSkWaves * 64 / TPR) {
    float v[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int wv = 0; wv < kSkWaves; ++wv) {
      const float4 p = *reinterpret_cast<const float4*>(&red[wv * kRedWave + m * RLD + c4]);
      v[0] += p.x; v[1] += p.y; v[2] += p.z; v[3] += p.w;
    }
    const size_t off = (size_t)m * N + n0 + c4;
    if (partial != nullptr) {
      *reinterpret_cast<float4*>(partial + (size_t)blockIdx.y * M * N + off) = make_float4(v[0], v[1], v[2], v[3]);
      continue;
    }
    if (bias != nullptr) {
      const vec4<E> b4 = *reinterpret_cast<const vec4<E>*>(bias + n0 + c4);
#pragma unroll
      for (int q = 0; q < 4; ++q) v[q] += static_cast<float>(b4[q]);
    }
    if (epi == EPI_BIAS_GELU) {
#pragma unroll
      for (int q = 0; q < 4; ++q) v[q] = gelu_erf(v[q]);
    }
    if (epi == EPI_BIAS_RESIDUAL) {
      const vec4<E> r4 = *reinterpret_cast<const vec4<E>*>(res + off);
#pragma unroll
      for (int q = 0; q < 4; ++q) v[q] += static_cast<float>(r4[q]);
    }
    vec4<E> o;
#pragma unroll
    for (int q = 0; q < 4; ++q) o[q] = static_cast<E>(v[q]);
    *reinterpret_cast<vec4<E>*>(y + off) = o;
  }
}

// y = epilogue(sum over kz of partial[kz] + b): the partial sums are added in the order of kz.
template <typename E>
__global__ __launch_bounds__(256) void skinny_reduce_kernel(const float* __restrict__ partial, int32_t KS,
                                                            const E* __restrict__ bias, const E* res, E* y, int32_t M,
                                                            int32_t N, int epi) {
  const size_t i4 = (size_t)blockIdx.x * 256 + threadIdx.x;   // group of 4 columns
  const size_t total4 = (size_t)M * N / 4;
  if (i4 >= total4) return;
  const size_t off = i4 * 4;
  const int32_t n = (int32_t)(off % N);
  float v[4] = {0.f, 0.f, 0.f, 0.f};
  for (int32_t kz = 0; kz < KS; ++kz) {
    const float4 p = *reinterpret_cast<const float4*>(partial + (size_t)kz * M * N + off);
    v[0] += p.x; v[1] += p.y; v[2] += p.z; v[3] += p.w;
  }
  if (bias != nullptr) {
    const vec4<E> b4 = *reinterpret_cast<const vec4<E>*>(bias + n);
#pragma unroll
    for (int q = 0; q < 4; ++q) v[q] += static_cast<float>(b4[q]);
  }
  if (epi == EPI_BIAS_GELU) {
#pragma unroll
    for (int q = 0; q < 4; ++q) v[q] = gelu_erf(v[q]);
  }
  if (epi == EPI_BIAS_RESIDUAL) {
    const vec4<E> r4 = *reinterpret_cast<const vec4<E>*>(res + off);
#pragma unroll
    for (int q = 0; q < 4; ++q) v[q] += static_cast<float>(r4[q]);
  }
  vec4<E> o;
#pragma unroll
  for (int q = 0; q < 4; ++q) o[q] = static_cast<E>(v[q]);
  *reinterpret_cast<vec4<E>*>(y + off) = o;
}

template <typename E, int MT, int NT>
hipError_t launch_cfg(const E* x, const E* w, const E* bias, const E* res, E* y, float* partial, int32_t KS, int32_t M,
                      int32_t N, int32_t K, int epi, hipStream_t s) {
  auto kern = gemm_skinny_kernel<E, MT, NT>;
  constexpr size_t lds = SkCfg<MT, NT>::kLds;
  static LdsAttrOnce once;
  {
    hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), lds, once);
    if (e != hipSuccess) return e;
  }
  kern<<<dim3((unsigned)(N / (16 * NT)), (unsigned)KS), dim3(kSkWaves * 64), lds, s>>>(x, w, bias, res, y, partial, M, N,
                                                                                      K, epi);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || partial == nullptr) return e;
  return launch_partial_reduce<E>(partial, KS, bias, res, y, M, N, epi, s);
}

template <typename E, int NT>
hipError_t launch_nt(const E* x, const E* w, const E* bias, const E* res, E* y, float* partial, int32_t KS, int32_t M,
                     int32_t N, int32_t K, int epi, hipStream_t s) {
  if (M <= 16) return launch_cfg<E, 1, NT>(x, w, bias, res, y, partial, KS, M, N, K, epi, s);
  if (M <= 32) return launch_cfg<E, 2, NT>(x, w, bias, res, y, partial, KS, M, N, K, epi, s);
  return launch_cfg<E, 4, NT>(x, w, bias, res, y, partial, KS, M, N, K, epi, s);
}

}  // namespace

template <typename E>
hipError_t launch_partial_reduce(const float* partial, int32_t KS, const E* bias, const E* res, E* y, int64_t M,
                                 int32_t N, int epi, hipStream_t s) {
  const size_t total4 = (size_t)M * N / 4;   // N % 4 == 0 for every caller (N % 8 == 0 is an ABI rule)
  if (total4 == 0) return hipSuccess;
  skinny_reduce_kernel<E><<<dim3((unsigned)((total4 + 255) / 256)), dim3(256), 0, s>>>(partial, KS, bias, res, y,
                                                                                       (int32_t)M, N, epi);
  return hipGetLastError();
}
template hipError_t launch_partial_reduce<bf16_t>(const float*, int32_t, const bf16_t*, const bf16_t*, bf16_t*, int64_t,
                                                  int32_t, int, hipStream_t);
template hipError_t launch_partial_reduce<f16_t>(const float*, int32_t, const f16_t*, const f16_t*, f16_t*, int64_t,
                                                 int32_t, int, hipStream_t);

bool gemm_skinny_takes(int64_t M, int32_t N, int32_t K, int epi) {
  return M >= 1 && M <= 64 && N % 32 == 0 && K % 64 == 0 && epi >= EPI_BIAS && epi <= EPI_BIAS_RESIDUAL;
}

// Shape of the launch, from measurements on the 13B-shape matrices with M = 32 (W streamed at
// 5.2-5.7 TB/s when x is not fetched at all; fetching x, which every workgroup reads again from
// the L2, costs about x-bytes-fetched / 15 TB/s on top, and x-bytes-fetched = W bytes * M / BN):
//  * 64 columns per workgroup when that gives one full round of workgroups (200..256), else 32;
//  * K cut over 4 or 8 workgroups only where there are few column blocks and K is long (each part
//    >= 40 slabs) and the caller has room for the fp32 partial sums: FC2's shape gains 14 %, shorter
//    K loses to the second kernel and the partial traffic.
void gemm_skinny_plan(int64_t M, int32_t N, int32_t K, bool can_split, int32_t* bn, int32_t* ks) {
  (void)M;
  const int32_t KT = K / 64;
  const int32_t b = (N % 64 == 0 && N / 64 >= 200 && N / 64 <= 256) ? 64 : 32;
  int32_t k = 1;
  if (can_split && N / b <= 256) {
    while (k < 8 && KT % (2 * k) == 0 && KT / (2 * k) >= 40) k *= 2;
    if (k < 4) k = 1;
  }
  *bn = b;
  *ks = k;
}

size_t gemm_skinny_partial_bytes(int64_t M, int32_t N, int32_t K) {
  int32_t bn, ks;
  gemm_skinny_plan(M, N, K, true, &bn, &ks);
  return ks > 1 ? (size_t)ks * (size_t)M * N * sizeof(float) : 0;
}

// partial == nullptr: one launch, K not split.  Otherwise `partial` must hold
// gemm_skinny_partial_bytes(M, N, K) bytes and the plan above decides.
template <typename E>
hipError_t launch_gemm_skinny(const E* x, const E* w, const E* bias, const E* res, E* y, int64_t M, int32_t N,
                              int32_t K, int epi, hipStream_t s, float* partial) {
  if (!gemm_skinny_takes(M, N, K, epi)) return hipErrorInvalidValue;
  int32_t bn, ks;
  gemm_skinny_plan(M, N, K, partial != nullptr, &bn, &ks);
  float* p = ks > 1 ? partial : nullptr;
  if (bn == 64) return launch_nt<E, 4>(x, w, bias, res, y, p, ks, (int32_t)M, N, K, epi, s);
  return launch_nt<E, 2>(x, w, bias, res, y, p, ks, (int32_t)M, N, K, epi, s);
}

template hipError_t launch_gemm_skinny<bf16_t>(const bf16_t*, const bf16_t*, const bf16_t*, const bf16_t*, bf16_t*,
                                               int64_t, int32_t, int32_t, int, hipStream_t, float*);
template hipError_t launch_gemm_skinny<f16_t>(const f16_t*, const f16_t*, const f16_t*, const f16_t*, f16_t*, int64_t,
                                              int32_t, int32_t, int, hipStream_t, float*);

}  // namespace energon
