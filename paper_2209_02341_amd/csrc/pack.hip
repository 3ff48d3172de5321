// Removing and rebuilding padding (paper Sec. 4.3): length scan, row gather, row scatter.
//
// The valid-token mask of a right-padded batch is run-length coded by the lengths, so its
// prefix sum is the prefix sum of the lengths (cu).  For batches of up to kLensArgMax sequences the
// whole removal is ONE launch and no copy: the lengths travel in the kernel's argument block, the
// first wavefront of every workgroup scans them with lane shuffles into LDS (a few hundred cycles,
// hidden behind the other workgroups' row traffic), workgroup 0 also writes cu to global memory,
// and every wavefront then gathers two consecutive packed rows, finding the first one's sequence by
// bisection in the LDS copy of cu.  Larger batches scan the lengths in launches of their own (896 per
// launch, again from the argument block, each continuing from the previous one's last sum) and gather
// with cu in global memory.  The scatter walks the padded rows and either
// copies a packed row or writes zeros.  All row traffic is 16-byte vectors, a wavefront per row, so
// every access is a full contiguous line; a row moves in batches of eight vectors per lane, all
// loaded before the first is stored.
#include "common.h"

namespace energon {

// Prefix sums of up to kLensArgMax lengths that arrive in the argument block, by one wavefront
// (inclusive scan of 64 values by shuffles, carry between chunks): cu points at the sum in front of
// them (written by the launch before this one on the stream, or set to 0 here if these are the first
// lengths); cu[1..n] receive the sums.
__global__ __launch_bounds__(64) void scan_lengths_arg_kernel(const LensArg lens, int32_t n, int32_t* __restrict__ cu,
                                                              int32_t first) {
  const int lane = threadIdx.x;
  int32_t carry = first ? 0 : cu[0];
  for (int32_t base = 0; base < n; base += kWave) {
    const int32_t i = base + lane;
    int32_t v = (i < n) ? lens.v[i] : 0;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
      const int32_t up = __shfl_up(v, o, kWave);
      if (lane >= o) v += up;
    }
    v += carry;
    if (i < n) cu[1 + i] = v;
    carry = __shfl(v, kWave - 1, kWave);
  }
  if (first && lane == 0) cu[0] = 0;
}

constexpr int kPackWaves = 4;     // wavefronts per workgroup
constexpr int kRowsPerWave = 2;   // consecutive packed rows gathered by one wavefront
constexpr int kRowsPerBlock = 4;  // scatter: one wavefront per padded row
constexpr int kCopyBatch = 8;     // 16-byte vectors per lane in flight
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // a 16-byte vector the non-temporal builtin takes

// One row of row_vecs 16-byte vectors, by one wavefront.  NT: non-temporal stores (measured on the
// scatter, whose output nothing here reads again: 41 -> 48 us, so it is not used there).
template <bool NT>
__device__ __forceinline__ void copy_row(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int32_t row_vecs,
                                         int lane) {
  int32_t c = lane;
  for (; c + (kCopyBatch - 1) * kWave < row_vecs; c += kCopyBatch * kWave) {
    u32x4 r[kCopyBatch];
#pragma unroll
    for (int u = 0; u < kCopyBatch; ++u) r[u] = src[c + u * kWave];
#pragma unroll
    for (int u = 0; u < kCopyBatch; ++u) {
      if (NT) __builtin_nontemporal_store(r[u], dst + c + u * kWave);
      else dst[c + u * kWave] = r[u];
    }
  }
  for (; c < row_vecs; c += kWave) {
    const u32x4 r = src[c];
    if (NT) __builtin_nontemporal_store(r, dst + c); else dst[c] = r;
  }
}

// SCAN: the lengths are in the argument block and cu is built here (see the file comment);
// otherwise cu_global already holds the prefix sums.
template <bool SCAN>
__global__ __launch_bounds__(kPackWaves* kWave) void pack_rows_kernel(
    const u32x4* __restrict__ x_padded, u32x4* __restrict__ x_packed, const LensArg lens, int32_t* cu_global,
    int32_t* __restrict__ token_idx, int32_t B, int32_t S, int32_t row_vecs, int64_t T) {
  __shared__ int32_t cu_s[SCAN ? kLensArgMax + 1 : 1];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if constexpr (SCAN) {
    if (wave == 0) {
      int32_t carry = 0;
      for (int32_t base = 0; base < B; base += kWave) {
        const int32_t i = base + lane;
        int32_t v = (i < B) ? lens.v[i] : 0;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
          const int32_t up = __shfl_up(v, o, kWave);
          if (lane >= o) v += up;
        }
        v += carry;
        if (i < B) cu_s[1 + i] = v;
        carry = __shfl(v, kWave - 1, kWave);
      }
      if (lane == 0) cu_s[0] = 0;
    }
    __syncthreads();
    if (blockIdx.x == 0)
      for (int32_t i = threadIdx.x; i <= B; i += kPackWaves * kWave) cu_global[i] = cu_s[i];
  }
  const int32_t* cu = SCAN ? cu_s : cu_global;
  const int64_t t0 = ((int64_t)blockIdx.x * kPackWaves + wave) * kRowsPerWave;
  if (t0 >= T) return;
  // largest b with cu[b] <= t0; then cu[b] <= t0 < cu[b+1], so sequence b is not empty
  int32_t lo = 0, hi = B;
  while (hi - lo > 1) {
    const int32_t mid = (lo + hi) >> 1;
    if ((int64_t)cu[mid] <= t0) lo = mid; else hi = mid;
  }
  int32_t b = lo;
#pragma unroll
  for (int r = 0; r < kRowsPerWave; ++r) {
    const int64_t t = t0 + r;
    if (t >= T) break;
    while (t >= (int64_t)cu[b + 1]) ++b;   // skips empty sequences; ends because t < T = cu[B]
    const int32_t src_row = b * S + (int32_t)(t - cu[b]);
    if (lane == 0) token_idx[t] = src_row;
    copy_row<false>(x_padded + (size_t)src_row * row_vecs, x_packed + (size_t)t * row_vecs, row_vecs, lane);
  }
}

__global__ __launch_bounds__(kRowsPerBlock* kWave) void unpack_rows_kernel(
    const u32x4* __restrict__ y_packed, u32x4* __restrict__ y_padded, const int32_t* __restrict__ cu, int32_t B,
    int32_t S, int32_t row_vecs) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t rows = (int64_t)B * S;
  for (int64_t r = (int64_t)blockIdx.x * kRowsPerBlock + wave; r < rows; r += (int64_t)gridDim.x * kRowsPerBlock) {
    const int32_t b = (int32_t)(r / S), s = (int32_t)(r - (int64_t)b * S);
    const int32_t c0 = cu[b], len = cu[b + 1] - c0;
    u32x4* dst = y_padded + (size_t)r * row_vecs;
    if (s < len) {
      copy_row<false>(y_packed + (size_t)(c0 + s) * row_vecs, dst, row_vecs, lane);
    } else {
      const u32x4 z = {0u, 0u, 0u, 0u};
      for (int32_t c = lane; c < row_vecs; c += kWave) dst[c] = z;
    }
  }
}

static int row_grid(int64_t rows) {
  int64_t blocks = (rows + kRowsPerBlock - 1) / kRowsPerBlock;
  const int64_t cap = 256 * 64;  // 64 resident groups per CU is more than enough to cover HBM latency
  return (int)(blocks < cap ? (blocks > 0 ? blocks : 1) : cap);
}

// cu[0..B] from lengths on the host, any B: one small launch per kLensArgMax lengths, each carrying its
// lengths in its argument block and continuing from the sum the launch before it left (stream order).
// No copy, so the call never waits and reads lengths_host only before it returns.
hipError_t launch_scan_lengths_host(const int32_t* lengths_host, int32_t* cu, int32_t B, hipStream_t s) {
  for (int32_t b0 = 0; b0 < B; b0 += kLensArgMax) {
    const int32_t n = B - b0 < kLensArgMax ? B - b0 : kLensArgMax;
    LensArg arg;
    for (int32_t i = 0; i < n; ++i) arg.v[i] = lengths_host[b0 + i];
    for (int32_t i = n; i < kLensArgMax; ++i) arg.v[i] = 0;
    scan_lengths_arg_kernel<<<1, kWave, 0, s>>>(arg, n, cu + b0, b0 == 0 ? 1 : 0);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

static unsigned pack_grid(int64_t T) {
  const int64_t per_block = kPackWaves * kRowsPerWave;
  const int64_t blocks = (T + per_block - 1) / per_block;   // T < 2^31
  return (unsigned)(blocks > 0 ? blocks : 1);
}

hipError_t launch_pack_scan_rows(const void* x_padded, void* x_packed, const int32_t* lengths_host, int32_t* cu,
                                 int32_t* token_idx, int32_t B, int32_t S, int64_t row_bytes, int64_t T,
                                 hipStream_t s) {
  if (B > kLensArgMax) return hipErrorInvalidValue;
  LensArg arg;
  for (int32_t b = 0; b < B; ++b) arg.v[b] = lengths_host[b];
  for (int32_t b = B; b < kLensArgMax; ++b) arg.v[b] = 0;
  pack_rows_kernel<true><<<pack_grid(T), kPackWaves * kWave, 0, s>>>((const u32x4*)x_padded, (u32x4*)x_packed, arg, cu,
                                                                     token_idx, B, S, (int32_t)(row_bytes / 16), T);
  return hipGetLastError();
}

hipError_t launch_pack_rows(const void* x_padded, void* x_packed, const int32_t* cu, int32_t* token_idx, int32_t B,
                            int32_t S, int64_t row_bytes, int64_t T, hipStream_t s) {
  if (T <= 0) return hipSuccess;
  const LensArg none{};
  pack_rows_kernel<false><<<pack_grid(T), kPackWaves * kWave, 0, s>>>(
      (const u32x4*)x_padded, (u32x4*)x_packed, none, const_cast<int32_t*>(cu), token_idx, B, S,
      (int32_t)(row_bytes / 16), T);
  return hipGetLastError();
}

hipError_t launch_unpack_rows(const void* y_packed, void* y_padded, const int32_t* cu, int32_t B, int32_t S,
                              int64_t row_bytes, hipStream_t s) {
  unpack_rows_kernel<<<row_grid((int64_t)B * S), kRowsPerBlock * kWave, 0, s>>>(
      (const u32x4*)y_packed, (u32x4*)y_padded, cu, B, S, (int32_t)(row_bytes / 16));
  return hipGetLastError();
}

}  // namespace energon
