// bf16 causal attention over each sequence's real length, on packed rows.  The paper
// (Sec. 4.3) rebuilds the padding around the attention core; here the core itself is
// variable-length, so nothing is rebuilt inside a layer and no score is computed for a pad.
//
// One workgroup (4 wavefronts) = one (sequence, head, block of 128 queries); each wavefront
// owns 32 queries.  Keys/values are walked in tiles of 64 keys staged in LDS (double-buffered)
// and shared by the four wavefronts; tiles above the causal diagonal are never visited.
//
// Everything is computed transposed so that a query is a *column* of every MFMA result:
//   S^T[key, query] = K[key, :] . Q[query, :]      A operand = K rows, B operand = Q rows
//   O^T[dd,  query] += V^T[dd, key] . P^T[key, query]
// In the 32x32 accumulator layout a lane holds one query column, so the online-softmax state
// (running max, running sum, rescale factor) is one scalar per lane, and the exponentiated
// scores are already laid out as the B operand of the second product: no cross-lane movement
// of P.  The contraction index (key) may be enumerated in any order as long as both operands
// agree, so V^T is read from LDS in the order the accumulator layout dictates.
// V is transposed on its way into LDS (key-contiguous rows), two keys per 32-bit store.
#include "common.h"

namespace energon {

constexpr int kBQ = 128, kBKV = 64;
constexpr float kLog2e = 1.4426950408889634f;

template <int D> __device__ __forceinline__ int kswz(int row) {
  return D == 128 ? (row & 15) : ((row & 7) ^ ((row >> 3) & 1));
}
__device__ __forceinline__ int vswz(int dd) { return (dd >> 1) & 7; }

template <int D>
__global__ __launch_bounds__(256) void attention_bf16_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ out,
                                                             const int32_t* __restrict__ cu, int32_t nh,
                                                             int32_t n_qblocks) {
  constexpr int DC = D / 16;        // 16-wide chunks of the head dimension (S^T contraction steps)
  constexpr int DT = D / 32;        // 32-row tiles of O^T
  constexpr int KC = D / 8;         // 16-byte chunks per K row
  constexpr int KLOADS = kBKV * KC / 256;   // 16-byte K chunks staged per thread
  constexpr int VLOADS = KC / 4;            // 16-byte V chunks staged per thread
  constexpr int kStage = (kBKV * D * 2 + D * kBKV * 2) / 16;  // uint4 per stage: K tile + V^T tile
  extern __shared__ uint4 lds[];

  const int32_t b = blockIdx.z, h = blockIdx.y;
  const int32_t qb = n_qblocks - 1 - (int32_t)blockIdx.x;  // longest (most keys) first
  const int32_t c0 = cu[b], len = cu[b + 1] - c0;
  const int32_t q0 = qb * kBQ;
  if (q0 >= len) return;  // whole workgroup leaves before any barrier

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lq = lane & 31, g = lane >> 5;
  const int32_t A = nh * D;
  const size_t ld = (size_t)3 * A;
  const bf16_t* qbase = qkv + (size_t)c0 * ld + (size_t)h * D;
  const bf16_t* kbase = qbase + A;
  const bf16_t* vbase = qbase + 2 * (size_t)A;

  const int32_t wq_first = q0 + 32 * wave, wq_last = wq_first + 31;
  const int32_t qi = wq_first + lq;
  const int32_t qc = qi < len ? qi : len - 1;

  bf16x8 qf[DC];
#pragma unroll
  for (int dc = 0; dc < DC; ++dc) qf[dc] = *reinterpret_cast<const bf16x8*>(qbase + (size_t)qc * ld + dc * 16 + 8 * g);

  const int32_t kv_end = min(q0 + kBQ, len);           // keys 0 .. kv_end-1 are needed
  const int32_t n_tiles = (kv_end + kBKV - 1) / kBKV;

  f32x16 oacc[DT];
#pragma unroll
  for (int i = 0; i < DT; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[i][e] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float sc = rsqrtf((float)D) * kLog2e;  // scores are kept in log2 units

  // Tile t+1 is fetched from global memory into registers while tile t is consumed from LDS,
  // and written to the other LDS buffer afterwards.  The loop starts at t = -1 (fetch tile 0,
  // nothing to consume); past the end the last tile is fetched again and never used.
  for (int32_t t = -1; t < n_tiles; ++t) {
    const int32_t tn = t + 1 < n_tiles ? t + 1 : n_tiles - 1;
    uint4 kreg[KLOADS], vreg[VLOADS];
#pragma unroll
    for (int i = 0; i < KLOADS; ++i) {
      const int q = tid + i * 256, row = q / KC, c = q % KC;
      int32_t key = tn * kBKV + row; key = key < len ? key : len - 1;
      kreg[i] = *reinterpret_cast<const uint4*>(kbase + (size_t)key * ld + c * 8);
    }
    {
      int32_t vkey = tn * kBKV + lane; vkey = vkey < len ? vkey : len - 1;
#pragma unroll
      for (int j = 0; j < VLOADS; ++j)
        vreg[j] = *reinterpret_cast<const uint4*>(vbase + (size_t)vkey * ld + (wave + 4 * j) * 8);
    }
    const int32_t k0 = t * kBKV;
    if (t >= 0 && k0 <= wq_last) {  // wavefront-uniform: the tile is not wholly above this wavefront's diagonal
      const uint4* ks = lds + (t & 1) * kStage;
      const char* vt = reinterpret_cast<const char*>(ks + kBKV * KC);
      f32x16 sacc[2];
#pragma unroll
      for (int j = 0; j < 2; ++j) {
#pragma unroll
        for (int e = 0; e < 16; ++e) sacc[j][e] = 0.f;
        const int row = j * 32 + lq;
#pragma unroll
        for (int dc = 0; dc < DC; ++dc) {
          const bf16x8 kf = *reinterpret_cast<const bf16x8*>(&ks[row * KC + ((dc * 2 + g) ^ kswz<D>(row))]);
          sacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[dc], sacc[j], 0, 0, 0);
        }
      }
      // scale, causal mask (also hides keys >= len: they are > every valid query), tile max
      const bool diag = k0 + kBKV - 1 > wq_first;
      float mx = -INFINITY;
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          float s = sacc[j][e] * sc;
          if (diag) {
            const int32_t key = k0 + j * 32 + (e >> 2) * 8 + g * 4 + (e & 3);
            s = key > qi ? -INFINITY : s;
          }
          sacc[j][e] = s;
          mx = fmaxf(mx, s);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m_run, mx);   // finite from tile 0 on: key 0 <= every query
      const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
      float psum = 0.f;
      bf16x8 pf[4];
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float p = __builtin_amdgcn_exp2f(sacc[j][e] - m_new);
          psum += p;
          pf[j * 2 + (e >> 3)][e & 7] = static_cast<bf16_t>(p);
        }
      l_run = l_run * corr + psum;
      m_run = m_new;
#pragma unroll
      for (int i = 0; i < DT; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[i][e] *= corr;
      // O^T += V^T P^T ; step tp covers keys 16tp + {4g..4g+3, 8+4g..8+4g+3}
#pragma unroll
      for (int tp = 0; tp < 4; ++tp) {
#pragma unroll
        for (int i = 0; i < DT; ++i) {
          const int dd = i * 32 + lq;
          const char* rowp = vt + dd * 128 + 8 * g;
          const uint2 lo = *reinterpret_cast<const uint2*>(rowp + (((2 * tp) ^ vswz(dd)) * 16));
          const uint2 hi = *reinterpret_cast<const uint2*>(rowp + (((2 * tp + 1) ^ vswz(dd)) * 16));
          union { uint4 u; bf16x8 v; } vf;
          vf.u = make_uint4(lo.x, lo.y, hi.x, hi.y);
          oacc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.v, pf[tp], oacc[i], 0, 0, 0);
        }
      }
    }
    {
      uint4* ks = lds + ((t + 1) & 1) * kStage;
      uint32_t* vt = reinterpret_cast<uint32_t*>(ks + kBKV * KC);
#pragma unroll
      for (int i = 0; i < KLOADS; ++i) {
        const int q = tid + i * 256, row = q / KC, c = q % KC;
        ks[row * KC + (c ^ kswz<D>(row))] = kreg[i];
      }
      // transpose: this lane holds 8 consecutive dd of one key; with its neighbour (key ^ 1) it
      // forms, per dd, the 32-bit word (even key, odd key).  Even lanes write dd 0,2,4,6 of the
      // chunk, odd lanes dd 1,3,5,7.
      const int kp = lane >> 1, odd = lane & 1;
#pragma unroll
      for (int j = 0; j < VLOADS; ++j) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const uint32_t we = e == 0 ? vreg[j].x : e == 1 ? vreg[j].y : e == 2 ? vreg[j].z : vreg[j].w;
          const uint32_t p = (uint32_t)__shfl_xor((int)we, 1, 64);
          const uint32_t word = odd ? ((p >> 16) | (we & 0xFFFF0000u)) : ((we & 0xFFFFu) | (p << 16));
          const int dd = (wave + 4 * j) * 8 + 2 * e + odd;
          vt[dd * 32 + (((kp >> 2) ^ vswz(dd)) * 4) + (kp & 3)] = word;
        }
      }
    }
    __syncthreads();
  }

  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (qi < len) {
    const float inv = 1.0f / l_tot;
    bf16_t* orow = out + (size_t)(c0 + qi) * A + (size_t)h * D;
#pragma unroll
    for (int i = 0; i < DT; ++i)
#pragma unroll
      for (int eg = 0; eg < 4; ++eg) {
        bf16x4 o4;
#pragma unroll
        for (int e = 0; e < 4; ++e) o4[e] = static_cast<bf16_t>(oacc[i][eg * 4 + e] * inv);
        *reinterpret_cast<bf16x4*>(orow + i * 32 + eg * 8 + g * 4) = o4;
      }
  }
}

template <int D>
static hipError_t launch_d(const bf16_t* qkv, bf16_t* out, const int32_t* cu, int32_t B, int32_t max_len, int32_t nh,
                           hipStream_t s) {
  auto kern = attention_bf16_kernel<D>;
  constexpr size_t lds = 2 * (size_t)(kBKV * D * 2 + D * kBKV * 2);
  static bool attr_set = false;  // idempotent; a race between host threads only repeats the call
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int32_t n_qblocks = (max_len + kBQ - 1) / kBQ;
  kern<<<dim3((unsigned)n_qblocks, (unsigned)nh, (unsigned)B), dim3(256), lds, s>>>(qkv, out, cu, nh, n_qblocks);
  return hipGetLastError();
}

hipError_t launch_attention_bf16(const bf16_t* qkv, bf16_t* out, const int32_t* cu, int32_t B, int32_t max_len,
                                 int32_t nh, int32_t d, hipStream_t s) {
  if (B <= 0 || max_len <= 0) return hipSuccess;
  return d == 128 ? launch_d<128>(qkv, out, cu, B, max_len, nh, s) : launch_d<64>(qkv, out, cu, B, max_len, nh, s);
}

}  // namespace energon
