// Causal attention (bf16 or fp16 storage) over each sequence's real length, on packed rows.  The paper
// (Sec. 4.3) rebuilds the padding around the attention core; here the core itself is
// variable-length, so nothing is rebuilt inside a layer and no score is computed for a pad.
//
// One workgroup (8 wavefronts; registers are capped so that two workgroups share a CU and one's
// memory waits hide behind the other's arithmetic) = one (sequence, head, block of 128 queries);
// each wavefront owns 16 queries.
// Keys/values are walked in tiles of 64 keys held in LDS (double-buffered) and shared by the
// eight wavefronts; tiles above the causal diagonal are never visited.
//
// Everything is computed transposed so that a query is a *column* of every MFMA result
// (v_mfma_f32_16x16x32_bf16 / _f16: the lane holds column lane % 16, rows 4 * (lane / 16) + e):
//   S^T[key, query] = K[key, :] . Q[query, :]      A operand = K rows, B operand = Q rows
//   O^T[dd,  query] += V^T[dd, key] . P^T[key, query]
// so the online-softmax state (running max, running sum) is one scalar per lane, and the
// exponentiated scores are already laid out as the B operand of the second product: no
// cross-lane movement of P.  The contraction index (key) may be enumerated in any order as long
// as both operands agree, so V^T is kept in LDS in the order the accumulator layout dictates:
// position 8 g + i of a 32-key step holds key 4 g + i (i < 4) or 16 + 4 g + i - 4 of that step,
// which makes a lane's 8 keys (g = lane / 16) one 16-byte read.
// K and V tiles go from global memory straight to LDS (global_load_lds_dwordx4, whole 128- or
// 256-byte row pieces, the swizzle applied on the global side).  Every wavefront then reads back the
// eight V rows it fetched itself (no barrier needed for that), 16 bytes per lane, and writes them
// transposed (key-contiguous rows), two keys per 32-bit store, into the V^T tile.  (Fetching V
// with one key per lane, so that it arrives in the registers ready for that transposition, made
// every load instruction touch 64 different cache lines for 16 bytes each; the kernel then ran at
// under 3 TB/s of useful bytes on short sequences, where it is a plain streaming read.)
#include "common.h"

namespace energon {

constexpr int kBQ = 128, kBKV = 64, kAttnWaves = 8;
constexpr float kLog2e = 1.4426950408889634f;

typedef __attribute__((address_space(1))) const void* attn_gptr_t;
typedef __attribute__((address_space(3))) void* attn_lptr_t;

template <int D> __device__ __forceinline__ int kswz(int row) {
  return D == 128 ? (row & 15) : ((row & 7) ^ ((row >> 3) & 1));
}
// V^T rows are 128 bytes (64 keys); a lane reads row dd % 16 of a 16-row block, chunk 4 s + lane / 16:
// the access shape of the GEMM's 16-row operand tiles, and the same conflict-free swizzle.
__device__ __forceinline__ int vswz(int dd) {
  return ((dd >> 1) & 1) | (((dd >> 2) & 1) << 2) | (((dd >> 3) & 1) << 1);
}

// PADDED = false: Q, K, V are thirds of the packed [T, 3A] rows, the output is packed [T, A], and
// only the len[b] real queries of a sequence are computed.  PADDED = true (the paper's own path,
// Sec. 4.3): q, k, v, out are [B, nh, S, d] with zeros at the pads, all S queries are computed,
// and a key is allowed iff it is <= the query and < len[b].
template <typename E, int D, bool PADDED>
__global__ __launch_bounds__(kAttnWaves * 64, 4) void attention_mfma_kernel(const E* __restrict__ qptr,
                                                                          const E* __restrict__ kptr,
                                                                          const E* __restrict__ vptr,
                                                                          E* __restrict__ out,
                                                                          const int32_t* __restrict__ cu, int32_t nh,
                                                                          int32_t n_qblocks, int32_t n_pairs,
                                                                          int32_t S) {
  constexpr int KS = D / 32;        // 32-wide steps of the head dimension (S^T contraction)
  constexpr int DB = D / 16;        // 16-row blocks of O^T
  constexpr int KC = D / 8;         // 16-byte chunks per K row
  constexpr int KROWS = 64 / KC;    // K rows moved by one direct-to-LDS instruction (1 KiB)
  constexpr int KDMA = kBKV / KROWS / kAttnWaves;   // such instructions per wavefront and tile
  constexpr int VLOADS = KC / kAttnWaves;           // 16-byte V chunks transposed per thread
  constexpr int kTile = kBKV * D * 2 / 16;          // uint4 per K, V or V^T tile
  // LDS: K tile of the even trips, K tile of the odd trips, the V tile as fetched, the V^T tile
  static_assert(KDMA >= 1 && VLOADS >= 1, "head dimension too small for eight wavefronts");
  extern __shared__ uint4 lds[];

  // Workgroups are handed out in id order: all pairs' last query block first (the one with the
  // most keys), then the block before it, and so on, so that the long workgroups start early
  // and the short ones fill the end (measured: 10 % faster than keeping a pair's blocks
  // together, also when those share an L2).
  const int32_t pair = blockIdx.x % n_pairs;
  const int32_t b = pair / nh, h = pair % nh;
  const int32_t qb = n_qblocks - 1 - blockIdx.x / n_pairs;
  const int32_t c0 = cu[b], len = cu[b + 1] - c0;
  const int32_t q0 = qb * kBQ;
  const int32_t n_queries = PADDED ? S : len;   // queries of this sequence that are computed
  if (q0 >= n_queries) return;  // whole workgroup leaves before any barrier

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lq = lane & 15, g4 = lane >> 4;
  const int32_t A = nh * D;
  // row stride and first row of this (sequence, head) in each operand
  const size_t ld = PADDED ? (size_t)D : (size_t)3 * A;
  const size_t first = PADDED ? (size_t)pair * S * D : (size_t)c0 * ld + (size_t)h * D;
  const E* qbase = qptr + first;
  const E* kbase = kptr + first;
  const E* vbase = vptr + first;

  const int32_t wq_first = q0 + 16 * wave, wq_last = wq_first + 15;
  const int32_t qi = wq_first + lq;
  const int32_t qc = qi < n_queries ? qi : n_queries - 1;

  vec8<E> qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const vec8<E>*>(qbase + (size_t)qc * ld + ks * 32 + 8 * g4);

  const int32_t kv_end = min(q0 + kBQ, len);           // keys 0 .. kv_end-1 are needed
  const int32_t n_tiles = (kv_end + kBKV - 1) / kBKV;

  f32x4 oacc[DB];
#pragma unroll
  for (int i = 0; i < DB; ++i) oacc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;        // running max in log2 units (already scaled), running sum
  const float sc = rsqrtf((float)D) * kLog2e;  // raw score -> log2 units

  // Addresses inside this (sequence, head): a wavefront-uniform base plus a 32-bit byte offset
  // (the launcher checks that S rows fit in 32 bits).
  const char* kbytes = reinterpret_cast<const char*>(kbase);
  const char* vbytes = reinterpret_cast<const char*>(vbase);
  const uint32_t ld_b = (uint32_t)(ld * sizeof(E));
  // this lane's part of a K tile transfer: row kr of the instruction's KROWS rows, LDS slot ksl
  const int kr = lane / KC, ksl = lane % KC;
  uint32_t kcol[KDMA];   // byte offset of the chunk this lane fetches, inside its row
#pragma unroll
  for (int i = 0; i < KDMA; ++i) kcol[i] = (uint32_t)((ksl ^ kswz<D>((wave * KDMA + i) * KROWS + kr)) * 16);
  // V: the wavefront fetches rows 8 w .. 8 w + 7 of the tile (the same row groups as for K, swizzled by
  // the row's low three bits) and later reads them back itself: the lane takes key 8 w + lane % 8 and,
  // per read, the chunk c of 8 consecutive dd chosen so that 16 neighbouring lanes cover all 64 banks
  // (D = 128: the two halves of a row alternate every 8 lanes).  With its neighbour (key ^ 1, same
  // chunk) it forms, per dd, the 32-bit word (even key, odd key): even lanes write dd 0, 2, 4, 6 of the
  // chunk, odd lanes dd 1, 3, 5, 7; one byte permute builds the word.
  uint32_t vcol[KDMA];   // byte offset of the chunk this lane fetches, inside its row
#pragma unroll
  for (int i = 0; i < KDMA; ++i) vcol[i] = (uint32_t)((ksl ^ (((wave * KDMA + i) * KROWS + kr) & 7)) * 16);
  const int vkey = wave * 8 + (lane & 7), odd = lane & 1;
  const int kp = vkey >> 1;
  const uint32_t vsel = odd ? 0x03020706u : 0x05040100u;   // v_perm_b32 selector, bytes of {partner, own}
  uint32_t vsrc[VLOADS];     // uint4 index of the read inside the fetched V tile
  uint32_t vdst[VLOADS][4];  // word index of the store inside the V^T tile
#pragma unroll
  for (int j = 0; j < VLOADS; ++j) {
    const int c = KC == 16 ? 8 * ((lane >> 3) & 1) + (lane >> 4) + 4 * j : (lane >> 3);
    vsrc[j] = (uint32_t)(vkey * KC + (c ^ (vkey & 7)));
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int dd = c * 8 + 2 * e + odd;
      // key pair kp = 16 s + 8 h + 2 g + i (keys 32 s + 16 h + 4 g + 2 i, + 1) goes to 16-byte chunk
      // 4 s + g of the row, word 2 h + i of the chunk
      const int chunk = 4 * (kp >> 4) + ((kp >> 1) & 3), word = 2 * ((kp >> 3) & 1) + (kp & 1);
      vdst[j][e] = (uint32_t)(dd * 32 + ((chunk ^ vswz(dd)) * 4) + word);
    }
  }

  // Tile t+1 is fetched while tile t is consumed: K into the other K buffer (free since the barrier
  // that ended the previous trip), V into the one buffer for fetched V tiles (its previous content
  // was transposed out before that barrier).  After the arithmetic and a barrier (V^T(t) is no longer
  // read) every wavefront waits for its own loads, transposes its eight V rows into the V^T tile,
  // and a second barrier publishes K(t+1) and V^T(t+1).  The loop starts at t = -1 (fetch tile 0,
  // nothing to consume) and ends after the arithmetic of the last tile.
  uint4* const vraw = lds + 2 * kTile;
  uint32_t* const vt_words = reinterpret_cast<uint32_t*>(lds + 3 * kTile);
  for (int32_t t = n_tiles > 0 ? -1 : 0; t < n_tiles; ++t) {  // no tile at all: an empty sequence on the padded path
    const bool more = t + 1 < n_tiles;   // workgroup-uniform: there is a tile to fetch
    if (more) {
      uint4* ks_next = lds + ((t + 1) & 1) * kTile;
#pragma unroll
      for (int i = 0; i < KDMA; ++i) {
        int32_t key = (t + 1) * kBKV + (wave * KDMA + i) * KROWS + kr; key = key < len ? key : len - 1;
        __builtin_amdgcn_global_load_lds((attn_gptr_t)(kbytes + ((uint32_t)key * ld_b + kcol[i])),
                                         (attn_lptr_t)(ks_next + (wave * KDMA + i) * 64), 16, 0, 0);
        __builtin_amdgcn_global_load_lds((attn_gptr_t)(vbytes + ((uint32_t)key * ld_b + vcol[i])),
                                         (attn_lptr_t)(vraw + (wave * KDMA + i) * 64), 16, 0, 0);
      }
    }
    const int32_t k0 = t * kBKV;
    if (t >= 0 && k0 <= wq_last) {  // wavefront-uniform: the tile is not wholly above this wavefront's diagonal
      const uint4* ks = lds + (t & 1) * kTile;
      const char* vt = reinterpret_cast<const char*>(vt_words);
      f32x4 sacc[4];
#pragma unroll
      for (int kb = 0; kb < 4; ++kb) {
        sacc[kb] = f32x4{0.f, 0.f, 0.f, 0.f};
        const int row = kb * 16 + lq;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
          const vec8<E> kf = *reinterpret_cast<const vec8<E>*>(&ks[row * KC + ((s * 4 + g4) ^ kswz<D>(row))]);
          sacc[kb] = Mfma<E>::m16x16x32(kf, qf[s], sacc[kb]);
        }
      }
      // Mask (only on tiles that touch the diagonal or, on the padded path, the end of the
      // sequence: wavefront-uniform), then the tile max of the raw scores.  Packed: the causal
      // mask also hides keys >= len (they are > every real query).  Padded: pad queries lie beyond
      // len, so keys >= len are masked explicitly.
      if (k0 + kBKV - 1 > wq_first || (PADDED && k0 + kBKV > len)) {
#pragma unroll
        for (int kb = 0; kb < 4; ++kb)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int32_t key = k0 + kb * 16 + g4 * 4 + e;
            if (key > qi || (PADDED && key >= len)) sacc[kb][e] = -INFINITY;
          }
      }
      float mx = fmaxf(fmaxf(sacc[0][0], sacc[0][1]), fmaxf(sacc[0][2], sacc[0][3]));
#pragma unroll
      for (int kb = 1; kb < 4; ++kb)
#pragma unroll
        for (int e = 0; e < 4; ++e) mx = fmaxf(mx, sacc[kb][e]);
      // the query's max over the four lane groups that hold its keys: exchange with lane ^ 16, then
      // lane ^ 32 (v_permlane16_swap / v_permlane32_swap of a value with itself leave own and
      // partner's value in the two results)
      {
        const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
        mx = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
        const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
        mx = fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
      }
      const float m_new = fmaxf(m_run, mx * sc);   // finite from tile 0 on: key 0 <= every query (sc > 0)
      const bool rescale = __any(m_new != m_run);  // wavefront-uniform
      const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
      float psum = 0.f;
      vec8<E> pf[2];
#pragma unroll
      for (int kb = 0; kb < 4; ++kb)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float p = __builtin_amdgcn_exp2f(fmaf(sacc[kb][e], sc, -m_new));
          psum += p;
          pf[kb >> 1][(kb & 1) * 4 + e] = static_cast<E>(p);
        }
      l_run = l_run * corr + psum;
      m_run = m_new;
      if (rescale) {
#pragma unroll
        for (int i = 0; i < DB; ++i)
#pragma unroll
          for (int e = 0; e < 4; ++e) oacc[i][e] *= corr;
      }
      // O^T += V^T P^T ; step s, lane group g4: keys 32 s + {4 g4 .. 4 g4 + 3, 16 + 4 g4 .. 16 + 4 g4 + 3},
      // adjacent in the V^T row by construction
#pragma unroll
      for (int s = 0; s < 2; ++s) {
#pragma unroll
        for (int i = 0; i < DB; ++i) {
          const int dd = i * 16 + lq;
          union { uint4 u; vec8<E> v; } vf;
          vf.u = *reinterpret_cast<const uint4*>(vt + dd * 128 + (((4 * s + g4) ^ vswz(dd)) * 16));
          oacc[i] = Mfma<E>::m16x16x32(vf.v, pf[s], oacc[i]);
        }
      }
    }
    if (!more) break;                    // the last tile: nothing was fetched, nothing to publish
    if (t >= 0) __syncthreads();         // V^T(t) is no longer read
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wavefront's K and V rows have landed in LDS
    asm volatile("" ::: "memory");       // the reads below must stay behind that wait
#pragma unroll
    for (int j = 0; j < VLOADS; ++j) {
      const uint4 v = vraw[vsrc[j]];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t we = e == 0 ? v.x : e == 1 ? v.y : e == 2 ? v.z : v.w;
        // the neighbour lane's word (lane ^ 1 inside each quad: quad_perm [1, 0, 3, 2])
        const uint32_t p = (uint32_t)__builtin_amdgcn_mov_dpp((int)we, 0xB1, 0xF, 0xF, true);
        vt_words[vdst[j][e]] = __builtin_amdgcn_perm(p, we, vsel);
      }
    }
    __syncthreads();                     // K(t+1) and V^T(t+1) are complete
  }

  float l_tot = l_run + __shfl_xor(l_run, 16, 64);
  l_tot += __shfl_xor(l_tot, 32, 64);
  if (qi < n_queries) {
    const float inv = n_tiles > 0 ? 1.0f / l_tot : 0.f;   // no allowed key at all (len = 0): a zero row
    E* orow = PADDED ? out + first + (size_t)qi * D : out + (size_t)(c0 + qi) * A + (size_t)h * D;
#pragma unroll
    for (int i = 0; i < DB; ++i) {
      vec4<E> o4;
#pragma unroll
      for (int e = 0; e < 4; ++e) o4[e] = static_cast<E>(oacc[i][e] * inv);
      *reinterpret_cast<vec4<E>*>(orow + i * 16 + g4 * 4) = o4;
    }
  }
}

template <typename E, int D, bool PADDED>
static hipError_t launch_d(const E* q, const E* k, const E* v, E* out, const int32_t* cu, int32_t B, int32_t max_len,
                           int32_t nh, hipStream_t s) {
  auto kern = attention_mfma_kernel<E, D, PADDED>;
  constexpr size_t lds = 4 * (size_t)(kBKV * D * 2);   // two K tiles, the fetched V tile, the V^T tile
  static LdsAttrOnce once;
  {
    hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), lds, once);
    if (e != hipSuccess) return e;
  }
  const int32_t n_qblocks = (max_len + kBQ - 1) / kBQ;
  const int32_t n_pairs = B * nh;
  const int64_t grid = (int64_t)n_pairs * n_qblocks;
  kern<<<dim3((unsigned)grid), dim3(kAttnWaves * 64), lds, s>>>(q, k, v, out, cu, nh, n_qblocks, n_pairs, max_len);
  return hipGetLastError();
}

template <typename E>
static hipError_t launch_packed(const E* qkv, E* out, const int32_t* cu, int32_t B, int32_t max_len, int32_t nh,
                                int32_t d, hipStream_t s) {
  if (B <= 0 || max_len <= 0) return hipSuccess;
  const size_t A = (size_t)nh * d;
  return d == 128 ? launch_d<E, 128, false>(qkv, qkv + A, qkv + 2 * A, out, cu, B, max_len, nh, s)
                  : launch_d<E, 64, false>(qkv, qkv + A, qkv + 2 * A, out, cu, B, max_len, nh, s);
}

template <typename E>
static hipError_t launch_padded(const E* q, const E* k, const E* v, E* out, const int32_t* cu, int32_t B, int32_t S,
                                int32_t nh, int32_t d, hipStream_t s) {
  if (B <= 0 || S <= 0) return hipSuccess;
  return d == 128 ? launch_d<E, 128, true>(q, k, v, out, cu, B, S, nh, s)
                  : launch_d<E, 64, true>(q, k, v, out, cu, B, S, nh, s);
}

hipError_t launch_attention_bf16(const bf16_t* qkv, bf16_t* out, const int32_t* cu, int32_t B, int32_t max_len,
                                 int32_t nh, int32_t d, hipStream_t s) {
  return launch_packed<bf16_t>(qkv, out, cu, B, max_len, nh, d, s);
}
hipError_t launch_attention_f16(const f16_t* qkv, f16_t* out, const int32_t* cu, int32_t B, int32_t max_len, int32_t nh,
                                int32_t d, hipStream_t s) {
  return launch_packed<f16_t>(qkv, out, cu, B, max_len, nh, d, s);
}
hipError_t launch_attention_padded_bf16(const bf16_t* q, const bf16_t* k, const bf16_t* v, bf16_t* out,
                                        const int32_t* cu, int32_t B, int32_t S, int32_t nh, int32_t d, hipStream_t s) {
  return launch_padded<bf16_t>(q, k, v, out, cu, B, S, nh, d, s);
}
hipError_t launch_attention_padded_f16(const f16_t* q, const f16_t* k, const f16_t* v, f16_t* out, const int32_t* cu,
                                       int32_t B, int32_t S, int32_t nh, int32_t d, hipStream_t s) {
  return launch_padded<f16_t>(q, k, v, out, cu, B, S, nh, d, s);
}

}  // namespace energon
