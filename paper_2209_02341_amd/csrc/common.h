// Shared device helpers and the launch functions each kernel file exports.
// gfx950 only: 64-lane wavefronts, bf16 MFMA, hardware bf16 conversion.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace energon {

typedef __bf16 bf16_t;
typedef _Float16 f16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
template <typename E> using vec8 = E __attribute__((ext_vector_type(8)));   // one MFMA operand fragment
template <typename E> using vec4 = E __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;

// Element traits: VEC elements make one 16-byte vector.
template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int VEC = 4;
  __device__ static inline float to_f32(float v) { return v; }
  __device__ static inline float from_f32(float v) { return v; }
};
template <> struct Elem<bf16_t> {
  static constexpr int VEC = 8;
  __device__ static inline float to_f32(bf16_t v) { return static_cast<float>(v); }
  __device__ static inline bf16_t from_f32(float v) { return static_cast<bf16_t>(v); }  // RNE
};

template <> struct Elem<f16_t> {
  static constexpr int VEC = 8;
  __device__ static inline float to_f32(f16_t v) { return static_cast<float>(v); }
  __device__ static inline f16_t from_f32(float v) { return static_cast<f16_t>(v); }  // RNE
};

// The two 16-bit MFMA forms of gfx950 for an element type (bf16 or fp16), fp32 accumulation.
template <typename E> struct Mfma;
template <> struct Mfma<bf16_t> {
  __device__ static inline f32x16 m32x32x16(vec8<bf16_t> a, vec8<bf16_t> b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
  __device__ static inline f32x4 m16x16x32(vec8<bf16_t> a, vec8<bf16_t> b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
  }
};
template <> struct Mfma<f16_t> {
  __device__ static inline f32x16 m32x32x16(vec8<f16_t> a, vec8<f16_t> b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
  }
  __device__ static inline f32x4 m16x16x32(vec8<f16_t> a, vec8<f16_t> b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
  }
};

template <typename T> struct alignas(16) Vec16 { T v[Elem<T>::VEC]; };

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// GeLU in its erf form, z * Phi(z) = 0.5 z (1 + erf(z / sqrt 2)), in fp32, written without the
// cancellation of 1 + erf for negative z:
//   GeLU(z) = max(z, 0) - 0.5 |z| erfc(|z| / sqrt 2),
// with erfc(|z| / sqrt 2) = 2^P(|z|), P a degree-7 polynomial without constant term.  Its
// coefficients are a weighted least-squares fit (reweighted towards the minimax solution) of
// log2 erfc on 0 <= |z| <= 7.35, weighted by the error the term leaves on GeLU, with the leading
// coefficient held negative so that P -> -inf and 2^P -> 0 beyond the fitted range.  Absolute
// error on GeLU <= 1.3e-7 before the final fp32 rounding (a host-side test re-evaluates these
// constants against a library erf); one transcendental instruction and ten multiply-adds per
// element, branch-free, |z| taken as an operand modifier.
constexpr float kGeluErfcPoly[7] = {-1.1511532068252563f,    -0.4588780403137207f,   -0.05332031473517418f,
                                    0.008061456494033337f,   -0.0007832530536688864f, 4.081824226886965e-05f,
                                    -1.0515688018131186e-06f};
__device__ inline float gelu_erf(float z) {
  const float a = fabsf(z);
  float p = fmaf(kGeluErfcPoly[6], a, kGeluErfcPoly[5]);
  p = fmaf(p, a, kGeluErfcPoly[4]);
  p = fmaf(p, a, kGeluErfcPoly[3]);
  p = fmaf(p, a, kGeluErfcPoly[2]);
  p = fmaf(p, a, kGeluErfcPoly[1]);
  p = fmaf(p, a, kGeluErfcPoly[0]);
  const float e = __builtin_amdgcn_exp2f(p * a);   // erfc(|z| / sqrt 2)
  return fmaf(-0.5f * a, e, fmaxf(z, 0.f));
}

// Kernels that use more dynamic LDS than the default limit must be told so once per device (the
// attribute belongs to the kernel on a device).  One flag per device; a race between host threads
// only repeats the call.
struct LdsAttrOnce { bool done[32] = {}; };
inline hipError_t ensure_dynamic_lds(const void* kern, size_t bytes, LdsAttrOnce& once) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const bool tracked = dev >= 0 && dev < 32;
  if (tracked && once.done[dev]) return hipSuccess;
  e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e == hipSuccess && tracked) once.done[dev] = true;
  return e;
}

enum Epilogue { EPI_BIAS = 0, EPI_BIAS_GELU = 1, EPI_BIAS_RESIDUAL = 2, EPI_LNFOLD = 3, EPI_LNFOLD_GELU = 4 };

// LayerNorm folded into a 16-bit linear (the fusion of Sec. 5.5's comparison system, in algebraic
// form): with mean mu and r = 1/sqrt(var + eps) of an x row,
//   LayerNorm(x) W^T + b = r (x Wf^T - mu c) + bf,   Wf = W gamma,  c = row sums of Wf,  bf = b + W beta.
// EPI_LNFOLD / EPI_LNFOLD_GELU read stats, colsum and bias (fp32); the E-typed bias is unused.
// With EPI_BIAS_RESIDUAL, a non-null `partial` receives, per output row and 128-column segment,
// (sum, sum of squared deviations from the segment mean) of the ROUNDED outputs: the next
// LayerNorm's statistics without another pass over the row.  Null members = feature unused.
constexpr int kStatSeg = 128;  // columns per partial
struct LnFold {
  const float* stats = nullptr;   // [M][2] mu, r
  const float* colsum = nullptr;  // [N]
  const float* bias = nullptr;    // [N]
  float* partial = nullptr;       // [M][N / kStatSeg][2]
};

// ---- launchers (each returns the hipError_t of its launch) --------------------------------
// pack.hip
// Up to kLensArgMax sequence lengths travel by value in the gather kernel's argument block (the
// block is limited to 4 KiB), which then builds cu_seqlens itself: one launch, no copy.
constexpr int kLensArgMax = 896;
struct LensArg { int32_t v[kLensArgMax]; };
hipError_t launch_pack_scan_rows(const void* x_padded, void* x_packed, const int32_t* lengths_host, int32_t* cu,
                                 int32_t* token_idx, int32_t B, int32_t S, int64_t row_bytes, int64_t T,
                                 hipStream_t s);
// cu_seqlens[0..B] from lengths on the host, any B, in launches that carry 896 lengths each in their argument block
hipError_t launch_scan_lengths_host(const int32_t* lengths_host, int32_t* cu_seqlens, int32_t B, hipStream_t s);
hipError_t launch_pack_rows(const void* x_padded, void* x_packed, const int32_t* cu, int32_t* token_idx,
                            int32_t B, int32_t S, int64_t row_bytes, int64_t T, hipStream_t s);
hipError_t launch_unpack_rows(const void* y_packed, void* y_padded, const int32_t* cu, int32_t B, int32_t S,
                              int64_t row_bytes, hipStream_t s);
// layernorm.hip
// dtype: 0 fp32, 1 bf16, 2 fp16 (the values of energon_dtype)
hipError_t launch_layernorm(const void* x, const void* gamma, const void* beta, void* y, int64_t T, int32_t H,
                            float eps, int dtype, hipStream_t s);
// gemm_f32.hip / gemm_mfma.hip (16-bit element types on the matrix cores)
hipError_t launch_gemm_f32(const float* x, const float* w, const float* bias, const float* res, float* y,
                           int64_t M, int32_t N, int32_t K, int epi, hipStream_t s);
// true if the launch for this shape can fill LnFold::partial (else the caller takes the statistics itself)
bool gemm_emits_row_partials(int64_t M, int32_t N, int32_t K, bool res_aliases_y);
// split_scratch (optional, gemm_scratch_bytes(M, N, K) bytes): lets problems with few rows cut K over
// several workgroups (partial sums in fp32, added in a fixed order by a second kernel).
size_t gemm_split_scratch_bytes(int64_t M, int32_t N, int32_t K);
// the part of the above that belongs to the persistent 256x256 kernel (0 if it does not take the shape
// or would not cut tiles along K): room for two pieces of 256x256 fp32 accumulators per workgroup
size_t gemm_sched_scratch_bytes(int64_t M, int32_t N, int32_t K);
// host-side replay of that kernel's work decomposition for one shape: 0 = every tile and slab covered once
int gemm_sched_selfcheck(int64_t M, int32_t N, int32_t K, int32_t wgs, int32_t can_split, int32_t* pieces_out);
hipError_t launch_gemm_bf16(const bf16_t* x, const bf16_t* w, const bf16_t* bias, const bf16_t* res, bf16_t* y,
                            int64_t M, int32_t N, int32_t K, int epi, hipStream_t s, const LnFold* fold = nullptr,
                            float* split_scratch = nullptr);
hipError_t launch_gemm_f16(const f16_t* x, const f16_t* w, const f16_t* bias, const f16_t* res, f16_t* y,
                           int64_t M, int32_t N, int32_t K, int epi, hipStream_t s, const LnFold* fold = nullptr,
                           float* split_scratch = nullptr);
// gemm_skinny.hip: M <= 64 rows (a generation step), bound by streaming W once.  With `partial`
// (gemm_skinny_partial_bytes bytes of scratch) K may be cut over several workgroups.
bool gemm_skinny_takes(int64_t M, int32_t N, int32_t K, int epi);
size_t gemm_skinny_partial_bytes(int64_t M, int32_t N, int32_t K);
template <typename E>
hipError_t launch_gemm_skinny(const E* x, const E* w, const E* bias, const E* res, E* y, int64_t M, int32_t N,
                              int32_t K, int epi, hipStream_t s, float* partial = nullptr);
// y = epilogue(sum over kz < KS of partial[kz][M][N] + b), the parts added in the order of kz
template <typename E>
hipError_t launch_partial_reduce(const float* partial, int32_t KS, const E* bias, const E* res, E* y, int64_t M,
                                 int32_t N, int epi, hipStream_t s);
// decode_attention.hip, model_ends.hip (dtype 1 or 2 only)
hipError_t launch_decode_attention(const void* qkv, void* k_cache, void* v_cache, const int32_t* lens, int32_t B,
                                   int32_t S_cap, int32_t nh, int32_t d, int dtype, void* out, hipStream_t s);
hipError_t launch_embed_packed(const int32_t* ids, const int32_t* cu, const int32_t* positions, int32_t B, int64_t T,
                               const void* wte, int32_t V, const void* wpe, int32_t P, int32_t H, int dtype, void* x,
                               hipStream_t s);
hipError_t launch_cache_fill(const void* qkv, const int32_t* cu, int32_t B, int64_t T, int64_t a_bytes, int32_t S_cap,
                             void* kc, void* vc, hipStream_t s);
hipError_t launch_last_rows(const void* x, const int32_t* cu, int32_t B, int64_t row_bytes, void* out, hipStream_t s);
// ln_fold.hip (dtype 1 or 2 only)
hipError_t launch_fold_weights(const void* w, const void* b, const void* gamma, const void* beta, int32_t N, int32_t K,
                               int dtype, void* wf, float* colsum, float* bias_f, hipStream_t s);
hipError_t launch_row_stats(const void* x, int64_t M, int32_t K, float eps, int dtype, float* stats, hipStream_t s);
hipError_t launch_merge_partials(const float* partial, int64_t M, int32_t P, float eps, float* stats, hipStream_t s);
// attention_f32.hip / attention_mfma.hip
hipError_t launch_attention_f32(const float* qkv, float* out, const int32_t* cu, int32_t B, int32_t max_len,
                                int32_t nh, int32_t d, hipStream_t s);
hipError_t launch_attention_bf16(const bf16_t* qkv, bf16_t* out, const int32_t* cu, int32_t B, int32_t max_len,
                                 int32_t nh, int32_t d, hipStream_t s);

hipError_t launch_attention_f16(const f16_t* qkv, f16_t* out, const int32_t* cu, int32_t B, int32_t max_len,
                                int32_t nh, int32_t d, hipStream_t s);
hipError_t launch_attention_padded_bf16(const bf16_t* q, const bf16_t* k, const bf16_t* v, bf16_t* out,
                                        const int32_t* cu, int32_t B, int32_t S, int32_t nh, int32_t d, hipStream_t s);
hipError_t launch_attention_padded_f16(const f16_t* q, const f16_t* k, const f16_t* v, f16_t* out,
                                       const int32_t* cu, int32_t B, int32_t S, int32_t nh, int32_t d, hipStream_t s);
// drce.hip (head_bytes = bytes of one head's slice of a row: d * element size)
hipError_t launch_rebuild_qkv(const void* qkv, void* q, void* k, void* v, const int32_t* cu, int32_t B, int32_t S,
                              int32_t nh, int32_t head_bytes, hipStream_t s);
hipError_t launch_remove_padding_heads(const void* o, void* out, const int32_t* cu, int32_t B, int32_t S, int32_t nh,
                                       int32_t head_bytes, hipStream_t s);

}  // namespace energon
