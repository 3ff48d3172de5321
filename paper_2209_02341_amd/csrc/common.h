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

// GeLU in its erf form, z * Phi(z) = 0.5 z (1 + erf(z / sqrt 2)), in fp32.  erf is evaluated
// branch-free with the rational approximation 7.1.26 of Abramowitz & Stegun,
//   erf(x) = 1 - (a1 t + ... + a5 t^5) exp(-x^2),  t = 1 / (1 + p x),  x >= 0,  |error| <= 1.5e-7,
// i.e. an absolute error of at most 7.5e-8 |z| on GeLU: two transcendental instructions and a
// dozen FMAs instead of the library erff's two divergent code paths.
__device__ inline float gelu_erf(float z) {
  const float x = fabsf(z) * 0.70710678118654752f;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, x, 1.0f));
  float p = fmaf(1.061405429f, t, -1.453152027f);
  p = fmaf(p, t, 1.421413741f);
  p = fmaf(p, t, -0.284496736f);
  p = fmaf(p, t, 0.254829592f);
  const float e = __builtin_amdgcn_exp2f(-x * x * 1.4426950408889634f);
  const float erf_abs = fmaf(-p * t, e, 1.0f);           // erf(|z| / sqrt 2)
  return 0.5f * z * (1.0f + copysignf(erf_abs, z));
}

enum Epilogue { EPI_BIAS = 0, EPI_BIAS_GELU = 1, EPI_BIAS_RESIDUAL = 2 };

// ---- launchers (each returns the hipError_t of its launch) --------------------------------
// pack.hip
hipError_t launch_scan_lengths(int32_t* cu_seqlens, int32_t B, hipStream_t s);
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
hipError_t launch_gemm_bf16(const bf16_t* x, const bf16_t* w, const bf16_t* bias, const bf16_t* res, bf16_t* y,
                            int64_t M, int32_t N, int32_t K, int epi, hipStream_t s);
hipError_t launch_gemm_f16(const f16_t* x, const f16_t* w, const f16_t* bias, const f16_t* res, f16_t* y,
                           int64_t M, int32_t N, int32_t K, int epi, hipStream_t s);
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
