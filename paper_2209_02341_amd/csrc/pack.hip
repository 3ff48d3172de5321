// Removing and rebuilding padding (paper Sec. 4.3): length scan, row gather, row scatter.
//
// The valid-token mask of a right-padded batch is run-length coded by the lengths, so its
// prefix sum is the prefix sum of the lengths (cu).  One wavefront scans them with lane
// shuffles; the gather finds each packed row's sequence by bisection in cu; the scatter
// walks the padded rows and either copies a packed row or writes zeros.  All row traffic
// is 16-byte vectors, one wavefront per row, so every access is a full contiguous line.
#include "common.h"

namespace energon {

// cu[1..B] holds the lengths on entry; on exit cu[0] = 0 and cu[b+1] = len[0]+..+len[b].
// One wavefront: inclusive scan of 64 values by shuffles, carry between chunks.
__global__ __launch_bounds__(64) void scan_lengths_kernel(int32_t* __restrict__ cu, int32_t B) {
  const int lane = threadIdx.x;
  int32_t carry = 0;
  for (int32_t base = 0; base < B; base += kWave) {
    const int32_t i = base + lane;
    int32_t v = (i < B) ? cu[1 + i] : 0;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
      const int32_t up = __shfl_up(v, o, kWave);
      if (lane >= o) v += up;
    }
    v += carry;
    if (i < B) cu[1 + i] = v;
    carry = __shfl(v, kWave - 1, kWave);
  }
  if (lane == 0) cu[0] = 0;
}

constexpr int kRowsPerBlock = 4;  // one wavefront per row

__global__ __launch_bounds__(kRowsPerBlock* kWave) void pack_rows_kernel(
    const uint4* __restrict__ x_padded, uint4* __restrict__ x_packed, const int32_t* __restrict__ cu,
    int32_t* __restrict__ token_idx, int32_t B, int32_t S, int32_t row_vecs, int64_t T) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  for (int64_t t = (int64_t)blockIdx.x * kRowsPerBlock + wave; t < T; t += (int64_t)gridDim.x * kRowsPerBlock) {
    // largest b with cu[b] <= t; then cu[b] <= t < cu[b+1], so sequence b is not empty
    int32_t lo = 0, hi = B;
    while (hi - lo > 1) {
      const int32_t mid = (lo + hi) >> 1;
      if ((int64_t)cu[mid] <= t) lo = mid; else hi = mid;
    }
    const int32_t src_row = lo * S + (int32_t)(t - cu[lo]);
    if (lane == 0) token_idx[t] = src_row;
    const uint4* src = x_padded + (size_t)src_row * row_vecs;
    uint4* dst = x_packed + (size_t)t * row_vecs;
    for (int32_t c = lane; c < row_vecs; c += kWave) dst[c] = src[c];
  }
}

__global__ __launch_bounds__(kRowsPerBlock* kWave) void unpack_rows_kernel(
    const uint4* __restrict__ y_packed, uint4* __restrict__ y_padded, const int32_t* __restrict__ cu, int32_t B,
    int32_t S, int32_t row_vecs) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t rows = (int64_t)B * S;
  for (int64_t r = (int64_t)blockIdx.x * kRowsPerBlock + wave; r < rows; r += (int64_t)gridDim.x * kRowsPerBlock) {
    const int32_t b = (int32_t)(r / S), s = (int32_t)(r - (int64_t)b * S);
    const int32_t c0 = cu[b], len = cu[b + 1] - c0;
    uint4* dst = y_padded + (size_t)r * row_vecs;
    if (s < len) {
      const uint4* src = y_packed + (size_t)(c0 + s) * row_vecs;
      for (int32_t c = lane; c < row_vecs; c += kWave) dst[c] = src[c];
    } else {
      const uint4 z = make_uint4(0u, 0u, 0u, 0u);
      for (int32_t c = lane; c < row_vecs; c += kWave) dst[c] = z;
    }
  }
}

static int row_grid(int64_t rows) {
  int64_t blocks = (rows + kRowsPerBlock - 1) / kRowsPerBlock;
  const int64_t cap = 256 * 64;  // 64 resident groups per CU is more than enough to cover HBM latency
  return (int)(blocks < cap ? (blocks > 0 ? blocks : 1) : cap);
}

hipError_t launch_scan_lengths(int32_t* cu, int32_t B, hipStream_t s) {
  scan_lengths_kernel<<<1, kWave, 0, s>>>(cu, B);
  return hipGetLastError();
}

hipError_t launch_pack_rows(const void* x_padded, void* x_packed, const int32_t* cu, int32_t* token_idx, int32_t B,
                            int32_t S, int64_t row_bytes, int64_t T, hipStream_t s) {
  if (T <= 0) return hipSuccess;
  pack_rows_kernel<<<row_grid(T), kRowsPerBlock * kWave, 0, s>>>((const uint4*)x_padded, (uint4*)x_packed, cu,
                                                                 token_idx, B, S, (int32_t)(row_bytes / 16), T);
  return hipGetLastError();
}

hipError_t launch_unpack_rows(const void* y_packed, void* y_padded, const int32_t* cu, int32_t B, int32_t S,
                              int64_t row_bytes, hipStream_t s) {
  unpack_rows_kernel<<<row_grid((int64_t)B * S), kRowsPerBlock * kWave, 0, s>>>(
      (const uint4*)y_packed, (uint4*)y_padded, cu, B, S, (int32_t)(row_bytes / 16));
  return hipGetLastError();
}

}  // namespace energon
