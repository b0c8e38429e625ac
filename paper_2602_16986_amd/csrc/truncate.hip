// Attention truncation on a jagged batch (paper Section 4.3): the layers after the first group run on the
// most recent `keep` history tokens of every sequence (plus its candidates).  Three HBM-bound kernels: the
// offsets of the truncated batch, the row gather, and its backward (row scatter with zero fill).
#include "hstu_kernels.h"

namespace hstu {
namespace {

constexpr int kScanThreads = 1024;
constexpr int kCopyThreads = 256;            // 4 waves
constexpr int kRowsPerWave = 8;              // consecutive rows handled by one wave per step
typedef int i32x4_t __attribute__((ext_vector_type(4)));

// out[b + 1] = sum over b' <= b of the kept rows of sequence b'; one workgroup walks the batch in chunks.
__global__ __launch_bounds__(kScanThreads) void truncate_offsets_kernel(int B, int keep, const int32_t* __restrict__ offsets,
                                                                        const int32_t* __restrict__ num_targets,
                                                                        int32_t* __restrict__ out) {
  __shared__ int32_t wave_sum[kScanThreads / 64];
  __shared__ int32_t carry_s;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) { carry_s = 0; out[0] = 0; }
  __syncthreads();
  for (int base = 0; base < B; base += kScanThreads) {
    const int b = base + tid;
    int kept = 0;
    if (b < B) {
      const int len = max(offsets[b + 1] - offsets[b], 0);
      const int m = num_targets ? min(max(num_targets[b], 0), len) : 0;
      kept = min(len - m, keep) + m;
    }
    int incl = kept;                         // inclusive scan inside the wave
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int up = __shfl_up(incl, d, 64);
      if (lane >= d) incl += up;
    }
    if (lane == 63) wave_sum[wave] = incl;
    __syncthreads();
    int before = carry_s;
    for (int w = 0; w < wave; ++w) before += wave_sum[w];
    if (b < B) out[b + 1] = before + incl;
    __syncthreads();
    if (tid == kScanThreads - 1) carry_s = before + incl;
    __syncthreads();
  }
}

// largest s with off[s] <= r (off non-decreasing, off[0] = 0 <= r < off[B]); lands on a non-empty sequence
__device__ __forceinline__ int find_sequence(const int32_t* __restrict__ off, int B, int r) {
  int lo = 0, hi = B;                        // off[lo] <= r < off[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (off[mid] <= r) lo = mid; else hi = mid;
  }
  return lo;
}

__device__ __forceinline__ void copy_rows(const char* const src[kRowsPerWave], char* const dst[kRowsPerWave], int64_t row_bytes,
                                          int lane) {
  for (int64_t c = (int64_t)lane * 16; c < row_bytes; c += 64 * 16) {
    i32x4_t v[kRowsPerWave];
#pragma unroll
    for (int i = 0; i < kRowsPerWave; ++i)
      v[i] = src[i] ? __builtin_nontemporal_load((const i32x4_t*)(src[i] + c)) : i32x4_t{0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < kRowsPerWave; ++i)
      if (dst[i]) __builtin_nontemporal_store(v[i], (i32x4_t*)(dst[i] + c));
  }
}

// y row r of truncated sequence b is x row  offsets[b+1] - (out_offsets[b+1] - r).
__global__ __launch_bounds__(kCopyThreads) void truncate_gather_kernel(int B, const int32_t* __restrict__ offsets,
                                                                       const int32_t* __restrict__ out_offsets, int64_t row_bytes,
                                                                       const char* __restrict__ x, int64_t x_stride,
                                                                       char* __restrict__ y, int64_t y_stride, int64_t y_rows) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t)blockIdx.x * (kCopyThreads / 64) + (threadIdx.x >> 6);
  const int64_t waves = (int64_t)gridDim.x * (kCopyThreads / 64);
  const int64_t rows = min((int64_t)out_offsets[B], y_rows);
  for (int64_t r0 = wave * kRowsPerWave; r0 < rows; r0 += waves * kRowsPerWave) {
    int b = find_sequence(out_offsets, B, (int)r0);
    const char* src[kRowsPerWave];
    char* dst[kRowsPerWave];
#pragma unroll
    for (int i = 0; i < kRowsPerWave; ++i) {
      const int64_t r = r0 + i;
      src[i] = nullptr; dst[i] = nullptr;
      if (r < rows) {
        while (b + 1 < B && r >= out_offsets[b + 1]) ++b;
        const int from = offsets[b + 1] - (out_offsets[b + 1] - (int)r);
        if (from >= offsets[b] && from < offsets[b + 1]) src[i] = x + (int64_t)from * x_stride;   // else: offsets that do not belong together
        dst[i] = y + r * y_stride;
      }
    }
    copy_rows(src, dst, row_bytes, lane);
  }
}

// dx row t of sequence b (position i, `drop` = rows of b that were cut) is dy row out_offsets[b] + i - drop, or zero for i < drop.
__global__ __launch_bounds__(kCopyThreads) void truncate_scatter_kernel(int B, int64_t T, const int32_t* __restrict__ offsets,
                                                                        const int32_t* __restrict__ out_offsets, int64_t row_bytes,
                                                                        const char* __restrict__ dy, int64_t dy_stride,
                                                                        char* __restrict__ dx, int64_t dx_stride) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t)blockIdx.x * (kCopyThreads / 64) + (threadIdx.x >> 6);
  const int64_t waves = (int64_t)gridDim.x * (kCopyThreads / 64);
  const int64_t rows = min((int64_t)offsets[B], T);
  for (int64_t r0 = wave * kRowsPerWave; r0 < rows; r0 += waves * kRowsPerWave) {
    int b = find_sequence(offsets, B, (int)r0);
    const char* src[kRowsPerWave];
    char* dst[kRowsPerWave];
#pragma unroll
    for (int i = 0; i < kRowsPerWave; ++i) {
      const int64_t r = r0 + i;
      src[i] = nullptr; dst[i] = nullptr;
      if (r < rows) {
        while (b + 1 < B && r >= offsets[b + 1]) ++b;
        const int drop = (offsets[b + 1] - offsets[b]) - (out_offsets[b + 1] - out_offsets[b]);
        const int pos = (int)r - offsets[b];
        if (pos >= drop && drop >= 0) src[i] = dy + (int64_t)(out_offsets[b] + pos - drop) * dy_stride;
        dst[i] = dx + r * dx_stride;
      }
    }
    copy_rows(src, dst, row_bytes, lane);
  }
}

int copy_grid(int64_t rows) {
  const int64_t steps = (rows + kRowsPerWave - 1) / kRowsPerWave;
  const int64_t wgs = (steps + kCopyThreads / 64 - 1) / (kCopyThreads / 64);
  return (int)max((int64_t)1, min(wgs, (int64_t)256 * 32));
}

}  // namespace

hipError_t launch_truncate_offsets(int B, int keep, const int32_t* offsets, const int32_t* num_targets, int32_t* out,
                                   hipStream_t stream) {
  hipLaunchKernelGGL(truncate_offsets_kernel, dim3(1), dim3(kScanThreads), 0, stream, B, keep, offsets, num_targets, out);
  return hipGetLastError();
}

hipError_t launch_truncate_gather(int B, const int32_t* offsets, const int32_t* out_offsets, int64_t row_bytes, const void* x,
                                  int64_t x_stride, void* y, int64_t y_stride, int64_t y_rows, hipStream_t stream) {
  hipLaunchKernelGGL(truncate_gather_kernel, dim3(copy_grid(y_rows)), dim3(kCopyThreads), 0, stream, B, offsets, out_offsets,
                     row_bytes, (const char*)x, x_stride, (char*)y, y_stride, y_rows);
  return hipGetLastError();
}

hipError_t launch_truncate_scatter(int B, int64_t T, const int32_t* offsets, const int32_t* out_offsets, int64_t row_bytes,
                                   const void* dy, int64_t dy_stride, void* dx, int64_t dx_stride, hipStream_t stream) {
  hipLaunchKernelGGL(truncate_scatter_kernel, dim3(copy_grid(T)), dim3(kCopyThreads), 0, stream, B, T, offsets, out_offsets,
                     row_bytes, (const char*)dy, dy_stride, (char*)dx, dx_stride);
  return hipGetLastError();
}

}  // namespace hstu
