// 16-bit linear layer for few rows (M <= 64): y[M,N] = epilogue(x[M,K] W[N,K]^T + b).
// This is the shape of a generation step, one token per sequence: every weight is used M times
// only, so the contraction is bound by streaming W from HBM once (N*K*e bytes), not by the
// matrix cores.  Design for gfx950:
//  * a workgroup owns 32 output columns (32 rows of W) and all of K; its 8 wavefronts split K in
//    interleaved slabs of 64 (wavefront w takes slabs w, w + 8, ...) and add their partial sums
//    through LDS at the end, in a fixed order: one launch, deterministic, no atomics, no workspace;
//  * W slabs (32 rows x 128 bytes) go from global memory straight to LDS
//    (global_load_lds_dwordx4, whole 128-byte lines per row) into a ring that is private to the
//    wavefront, four slabs deep: 16 KiB in flight per wavefront, 128 KiB per CU, with no barrier
//    and no staging register in the streaming loop.  The XOR swizzle of the 256x256 kernel keeps
//    the operand reads free of bank conflicts;
//  * the few x rows come from the L2 (x is read again by every workgroup) straight into MFMA
//    operand registers, also four slabs ahead;
//  * v_mfma_f32_16x16x32: x rows are the A operand (row tiles of 16, MT of them), W rows the B
//    operand; at these sizes the matrix cores are idle most of the time by design.
#include "common.h"

namespace energon {

namespace {

typedef __attribute__((address_space(1))) const void* sk_gptr_t;
typedef __attribute__((address_space(3))) void* sk_lptr_t;

constexpr int kSkBN = 32;       // output columns per workgroup
constexpr int kSkWaves = 8;     // K is split over this many wavefronts
constexpr int kSkDepth = 4;     // slabs in flight per wavefront
constexpr int kSkRedLd = 36;    // floats per row of the reduction buffer (4 rows apart -> 16 banks apart)

__device__ __forceinline__ int sk_swz(int row) {
  return ((row >> 1) & 1) | (((row >> 2) & 1) << 2) | (((row >> 3) & 1) << 1);
}

template <typename E, int MT>
__global__ __launch_bounds__(kSkWaves * 64) void gemm_skinny_kernel(const E* __restrict__ x, const E* __restrict__ w,
                                                                   const E* __restrict__ bias, const E* res, E* y,
                                                                   int32_t M, int32_t N, int32_t K, int epi) {
  static_assert(MT == 1 || MT == 2 || MT == 4, "row tiles per workgroup");
  constexpr int G = 2 * MT + 4;  // vector-memory instructions per slab: x fragments, then W row groups
  extern __shared__ uint4 lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int32_t n0 = blockIdx.x * kSkBN;
  const int32_t KT = K / 64;
  const int32_t ns = (KT - wave + kSkWaves - 1) / kSkWaves;   // slabs of this wavefront (>= 0)

  uint4* ring = lds + wave * (kSkDepth * 256);                // 4 KiB per slot
  const int lrow = lane & 15, lq = lane >> 4;

  // W row group j of a slab: 8 rows x 128 bytes in lane order, lane l landing in slot l % 8 of row
  // 8 j + l / 8 and fetching the chunk the swizzle puts there.
  const char* wsrc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int r = 8 * j + (lane >> 3);
    wsrc[j] = reinterpret_cast<const char*>(w + (size_t)(n0 + r) * K) + (((lane & 7) ^ sk_swz(r & 15)) * 16);
  }
  // x fragment of row tile t: lane l holds row 16 t + l % 16 (clamped: rows past M are computed
  // and dropped), 16-byte chunk 4 ks + l / 16 of the slab.
  const char* xsrc[MT];
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    const int32_t r = min(16 * t + lrow, M - 1);
    xsrc[t] = reinterpret_cast<const char*>(x + (size_t)r * K) + lq * 16;
  }
  // operand reads of W from the ring: row 16 j + l % 16, chunk (4 ks + l / 16) ^ swizzle
  uint32_t woff[2][2];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) woff[j][ks] = (uint32_t)((16 * j + lrow) * 8 + ((ks * 4 + lq) ^ sk_swz(lrow)));

  f32x4 acc[MT][2];
#pragma unroll
  for (int t = 0; t < MT; ++t)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[t][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  vec8<E> xa[kSkDepth][MT][2];

  // Every step of the loop below issues the same number of vector-memory instructions, so that
  // "the loads of slab i have landed" is a fixed count of younger loads (they return in order).
  // Past the wavefront's last slab the step still issues them, all lanes on one address (one
  // cache line, an L2 hit) into a ring slot that is never read again.
  // The x fragments are loaded by asm statements: the compiler's own wait insertion loses count
  // of loads carried around the loop and would drain the queue once per trip.  It therefore does
  // not know that these registers are pending: SK_WAIT both waits and takes them as in/out
  // operands, so every later use is ordered behind the wait.
#define SK_ISSUE(slot, i)                                                                              \
  do {                                                                                                 \
    const bool real = (i) < ns;                                                                        \
    const size_t kb = (size_t)(wave + (i) * kSkWaves) * 128;                                           \
    _Pragma("unroll") for (int t = 0; t < MT; ++t) {                                                   \
      const char* px = real ? xsrc[t] + kb : reinterpret_cast<const char*>(x);                         \
      asm volatile("global_load_dwordx4 %0, %1, off" : "=&v"(xa[slot][t][0]) : "v"(px) : "memory");    \
      asm volatile("global_load_dwordx4 %0, %1, off offset:64" : "=&v"(xa[slot][t][1]) : "v"(px) : "memory"); \
    }                                                                                                  \
    _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                                    \
      const char* pw = real ? wsrc[j] + kb : reinterpret_cast<const char*>(w);                         \
      __builtin_amdgcn_global_load_lds((sk_gptr_t)pw, (sk_lptr_t)(ring + (slot) * 256 + j * 64), 16, 0, 0); \
    }                                                                                                  \
  } while (0)
#define SK_WAIT(slot)                                                                                  \
  do {                                                                                                 \
    if constexpr (MT == 1)                                                                             \
      asm volatile("s_waitcnt vmcnt(%2)" : "+v"(xa[slot][0][0]), "+v"(xa[slot][0][1]) : "n"((kSkDepth - 1) * G) : "memory"); \
    else if constexpr (MT == 2)                                                                        \
      asm volatile("s_waitcnt vmcnt(%4)" : "+v"(xa[slot][0][0]), "+v"(xa[slot][0][1]), "+v"(xa[slot][1][0]), "+v"(xa[slot][1][1]) \
                   : "n"((kSkDepth - 1) * G) : "memory");                                              \
    else                                                                                               \
      asm volatile("s_waitcnt vmcnt(%8)" : "+v"(xa[slot][0][0]), "+v"(xa[slot][0][1]), "+v"(xa[slot][1][0]), "+v"(xa[slot][1][1]), \
                     "+v"(xa[slot][2][0]), "+v"(xa[slot][2][1]), "+v"(xa[slot][3][0]), "+v"(xa[slot][3][1]) \
                   : "n"((kSkDepth - 1) * G) : "memory");                                              \
  } while (0)

#pragma unroll
  for (int u = 0; u < kSkDepth; ++u) SK_ISSUE(u, u);

  for (int32_t i0 = 0; i0 < ns; i0 += kSkDepth) {
#pragma unroll
    for (int u = 0; u < kSkDepth; ++u) {
      const int32_t i = i0 + u;
      SK_WAIT(u);   // behind slab i's loads are exactly those of the next Depth - 1 steps
      if (i < ns) {   // wavefront-uniform
        const uint4* slab = ring + u * 256;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
          vec8<E> wb[2];
#pragma unroll
          for (int j = 0; j < 2; ++j) wb[j] = *reinterpret_cast<const vec8<E>*>(&slab[woff[j][ks]]);
#pragma unroll
          for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[t][j] = Mfma<E>::m16x16x32(xa[u][t][ks], wb[j], acc[t][j]);
        }
      }
      // the slot is refilled by the load unit, which is not ordered with this wavefront's LDS
      // reads: they must have returned first
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      SK_ISSUE(u, i + kSkDepth);
    }
  }
#undef SK_ISSUE
#undef SK_WAIT

  // Sum over the 8 wavefronts through LDS (the rings are free once every wavefront is here; each
  // has waited for its own last load), then the epilogue: thread -> row tid / 8, 4 columns.
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  __syncthreads();
  float* red = reinterpret_cast<float*>(lds);
  constexpr int kRedWave = MT * 16 * kSkRedLd;
#pragma unroll
  for (int t = 0; t < MT; ++t)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e)
        red[wave * kRedWave + (16 * t + 4 * lq + e) * kSkRedLd + 16 * j + lrow] = acc[t][j][e];
  __syncthreads();
  const int32_t m = tid >> 3, c4 = (tid & 7) * 4;
  if (m < MT * 16 && m < M) {
    float v[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int wv = 0; wv < kSkWaves; ++wv) {
      const float4 p = *reinterpret_cast<const float4*>(&red[wv * kRedWave + m * kSkRedLd + c4]);
      v[0] += p.x; v[1] += p.y; v[2] += p.z; v[3] += p.w;
    }
    const size_t off = (size_t)m * N + n0 + c4;
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

template <typename E, int MT>
hipError_t launch_mt(const E* x, const E* w, const E* bias, const E* res, E* y, int32_t M, int32_t N, int32_t K,
                     int epi, hipStream_t s) {
  auto kern = gemm_skinny_kernel<E, MT>;
  constexpr size_t ring = (size_t)kSkWaves * kSkDepth * 4096;
  constexpr size_t red = (size_t)kSkWaves * MT * 16 * kSkRedLd * sizeof(float);
  constexpr size_t lds = ring > red ? ring : red;
  static bool attr_set = false;  // idempotent; a race between host threads only repeats the call
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  kern<<<dim3((unsigned)(N / kSkBN)), dim3(kSkWaves * 64), lds, s>>>(x, w, bias, res, y, M, N, K, epi);
  return hipGetLastError();
}

}  // namespace

bool gemm_skinny_takes(int64_t M, int32_t N, int32_t K, int epi) {
  return M >= 1 && M <= 64 && N % kSkBN == 0 && K % 64 == 0 && epi >= EPI_BIAS && epi <= EPI_BIAS_RESIDUAL;
}

template <typename E>
hipError_t launch_gemm_skinny(const E* x, const E* w, const E* bias, const E* res, E* y, int64_t M, int32_t N,
                              int32_t K, int epi, hipStream_t s) {
  if (!gemm_skinny_takes(M, N, K, epi)) return hipErrorInvalidValue;
  const int32_t m = (int32_t)M;
  if (m <= 16) return launch_mt<E, 1>(x, w, bias, res, y, m, N, K, epi, s);
  if (m <= 32) return launch_mt<E, 2>(x, w, bias, res, y, m, N, K, epi, s);
  return launch_mt<E, 4>(x, w, bias, res, y, m, N, K, epi, s);
}

template hipError_t launch_gemm_skinny<bf16_t>(const bf16_t*, const bf16_t*, const bf16_t*, const bf16_t*, bf16_t*,
                                               int64_t, int32_t, int32_t, int, hipStream_t);
template hipError_t launch_gemm_skinny<f16_t>(const f16_t*, const f16_t*, const f16_t*, const f16_t*, f16_t*, int64_t,
                                              int32_t, int32_t, int, hipStream_t);

}  // namespace energon
