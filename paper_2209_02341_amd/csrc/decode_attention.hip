// Attention of one generation step: one new token per sequence attends the keys / values cached
// for its sequence's earlier tokens plus its own.  The paper (Sec. 2.2) defines the decoder block
// with a causal mask; under that mask earlier tokens' K and V rows never change, so a step needs
// only the cache and the new token's q, k, v.  Every sequence has its own cached length: as in the
// paper's padding elimination (Sec. 4.3), no position beyond a sequence's real length is touched.
//
// The work is one pass over the cached rows (2 * d * e bytes per key and head, each used once):
// bound by HBM, so there is no MFMA here.  One workgroup (4 wavefronts) per (sequence, head); a
// key's head slice (d elements) is spread over d / 8 lanes, 16 bytes each, so a wavefront takes
// 64 / (d / 8) keys per step with fully coalesced loads and the workgroup four times that; each
// lane group runs its own online softmax over the keys it sees, and the 4 * 64 / (d / 8) partial
// states are merged through LDS at the end.  The new token's k and v are read from the qkv row and
// written to the cache row at the sequence's length by the same workgroup.
#include "common.h"

namespace energon {

namespace {

constexpr int kDecWaves = 4;
constexpr int kDecUnroll = 4;   // key steps whose loads are in flight together
constexpr float kDecLog2e = 1.4426950408889634f;

// sum over the LPK consecutive lanes that hold one key (LPK = 8 or 16, inside one DPP row)
template <int LPK> __device__ __forceinline__ float key_sum(float v) {
  v += __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
  v += __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
  v += __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), 0x141, 0xF, 0xF, true));  // row_half_mirror
  if constexpr (LPK == 16) v += __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), 0x140, 0xF, 0xF, true));  // row_mirror
  return v;
}

template <typename E, int D>
__global__ __launch_bounds__(kDecWaves * 64) void decode_attention_kernel(const E* __restrict__ qkv, E* k_cache,
                                                                         E* v_cache, const int32_t* __restrict__ lens,
                                                                         int32_t nh, int32_t S_cap,
                                                                         E* __restrict__ out) {
  constexpr int LPK = D / 8;          // lanes per key
  constexpr int KPW = 64 / LPK;       // keys per wavefront step
  constexpr int KPB = KPW * kDecWaves;
  constexpr int NSTREAM = KPB;        // independent online-softmax states in the workgroup
  __shared__ float st_m[NSTREAM], st_l[NSTREAM];
  __shared__ float st_o[NSTREAM][D + 4];

  const int32_t b = blockIdx.x / nh, h = blockIdx.x % nh;
  const int32_t A = nh * D;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int sub = lane % LPK, slot = wave * KPW + lane / LPK;   // which 8 elements of d; which key of a step
  int32_t p = lens[b];
  p = p < 0 ? 0 : (p > S_cap ? S_cap : p);     // cached keys; the new token is key p
  const int32_t n_keys = p + 1;

  const E* qrow = qkv + (size_t)b * 3 * A + (size_t)h * D + sub * 8;
  const vec8<E> q8 = *reinterpret_cast<const vec8<E>*>(qrow);
  const E* knew = qrow + A;
  const E* vnew = qrow + 2 * A;
  const float sc = rsqrtf((float)D) * kDecLog2e;
  float q[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) q[e] = static_cast<float>(q8[e]) * sc;

  const size_t head_off = (size_t)b * S_cap * A + (size_t)h * D + sub * 8;
  const E* kc = k_cache + head_off;
  const E* vc = v_cache + head_off;

  // append: the new token's k and v become cache row p (one wavefront's first LPK lanes)
  if (wave == 0 && lane < LPK && p < S_cap) {
    *reinterpret_cast<vec8<E>*>(k_cache + head_off + (size_t)p * A) = *reinterpret_cast<const vec8<E>*>(knew);
    *reinterpret_cast<vec8<E>*>(v_cache + head_off + (size_t)p * A) = *reinterpret_cast<const vec8<E>*>(vnew);
  }

  float m_run = -INFINITY, l_run = 0.f, o[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = 0.f;

  for (int32_t j0 = 0; j0 < n_keys; j0 += KPB * kDecUnroll) {
    vec8<E> k8[kDecUnroll], v8[kDecUnroll];
#pragma unroll
    for (int u = 0; u < kDecUnroll; ++u) {
      const int32_t j = j0 + u * KPB + slot;
      // key p is the new token (read from the qkv row, never from the cache row written above);
      // keys past it are clamped to it and masked below
      const bool cached = j < p;
      const E* kp = cached ? kc + (size_t)j * A : knew;
      const E* vp = cached ? vc + (size_t)j * A : vnew;
      k8[u] = *reinterpret_cast<const vec8<E>*>(kp);
      v8[u] = *reinterpret_cast<const vec8<E>*>(vp);
    }
#pragma unroll
    for (int u = 0; u < kDecUnroll; ++u) {
      const int32_t j = j0 + u * KPB + slot;
      float s = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) s = fmaf(q[e], static_cast<float>(k8[u][e]), s);
      s = key_sum<LPK>(s);                       // the key's score in log2 units, in all its lanes
      if (j < n_keys) {
        const float m_new = fmaxf(m_run, s);
        const float corr = __builtin_amdgcn_exp2f(m_run - m_new);   // first key: exp2(-inf) = 0
        const float pw = __builtin_amdgcn_exp2f(s - m_new);
        l_run = fmaf(l_run, corr, pw);
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = fmaf(o[e], corr, pw * static_cast<float>(v8[u][e]));
        m_run = m_new;
      }
    }
  }

  // merge the NSTREAM partial states: weights 2^(m_i - M); a stream that saw no key has m = -inf, l = 0
  if (sub == 0) { st_m[slot] = m_run; st_l[slot] = l_run; }
#pragma unroll
  for (int e = 0; e < 8; ++e) st_o[slot][sub * 8 + e] = o[e];
  __syncthreads();
  if (tid < D) {
    float M = st_m[0];
#pragma unroll
    for (int i = 1; i < NSTREAM; ++i) M = fmaxf(M, st_m[i]);   // finite: key 0 exists
    float L = 0.f, acc = 0.f;
#pragma unroll
    for (int i = 0; i < NSTREAM; ++i) {
      const float wgt = __builtin_amdgcn_exp2f(st_m[i] - M);
      L = fmaf(st_l[i], wgt, L);
      acc = fmaf(st_o[i][tid], wgt, acc);
    }
    out[(size_t)b * A + (size_t)h * D + tid] = static_cast<E>(acc / L);
  }
}

template <typename E>
hipError_t launch_dec(const E* qkv, E* kc, E* vc, const int32_t* lens, int32_t B, int32_t S_cap, int32_t nh, int32_t d,
                      E* out, hipStream_t s) {
  const dim3 grid((unsigned)((int64_t)B * nh)), block(kDecWaves * 64);
  if (d == 128) decode_attention_kernel<E, 128><<<grid, block, 0, s>>>(qkv, kc, vc, lens, nh, S_cap, out);
  else decode_attention_kernel<E, 64><<<grid, block, 0, s>>>(qkv, kc, vc, lens, nh, S_cap, out);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_decode_attention(const void* qkv, void* k_cache, void* v_cache, const int32_t* lens, int32_t B,
                                   int32_t S_cap, int32_t nh, int32_t d, int dtype, void* out, hipStream_t s) {
  if (B <= 0) return hipSuccess;
  return dtype == 1 ? launch_dec<bf16_t>((const bf16_t*)qkv, (bf16_t*)k_cache, (bf16_t*)v_cache, lens, B, S_cap, nh, d,
                                         (bf16_t*)out, s)
                    : launch_dec<f16_t>((const f16_t*)qkv, (f16_t*)k_cache, (f16_t*)v_cache, lens, B, S_cap, nh, d,
                                        (f16_t*)out, s);
}

}  // namespace energon
