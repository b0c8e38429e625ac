// Weight gradients of the layer's two projections (layer pseudocode of the paper's appendix: d_linear_w = X^T dY):
//   C[n1, n2] = sum over token rows t of A[t, n1] * B[t, n2],   A [T, N1], B [T, N2] bf16 row-major, C fp32.
// The reduction runs over the jagged token axis (10^5 rows) and the output is small (512 x 512 .. 2048 x 512), so the
// work is cut along t: a workgroup owns a 128 x 128 output tile and one slab of token rows, accumulates in registers and
// writes an fp32 partial tile; a second kernel adds the slabs in a fixed order (deterministic, no atomics).
// Both operands have the reduction index as their slow axis, which is the wrong way round for the matrix cores (a lane
// wants 8 consecutive k of one output row): the 32-row tiles go to LDS as they are and both fragments come out through the
// LDS transpose loads (ds_read_b64_tr_b16).  Both operands use the same k assignment, which is all the product needs.
#include "hstu_common.h"
#include "hstu_kernels.h"

namespace hstu {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) short4v* lds_s4;

constexpr int kTile = 128;                 // output tile edge
constexpr int kBK = 64;                    // token rows per LDS tile
constexpr int kPitch = kTile * 2;          // bytes per LDS row; 16-byte chunk c of row r sits at chunk c ^ (4 (r % 4) + (r / 4) % 4): the
                                           // rows that one transpose load touches fall into different bank groups
constexpr int kOperand = kBK * kPitch;     // bytes of one operand tile

__global__ __launch_bounds__(256, 2) void gemm_tn_kernel(const __bf16* __restrict__ A, int64_t lda, const __bf16* __restrict__ B,
                                                         int64_t ldb, int N1, int N2, int64_t T, int64_t slab_rows,
                                                         float* __restrict__ partial) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];              // [stage][A, B][row][pitch]
  const int t = threadIdx.x, w = t >> 6, l = t & 63, l32 = l & 31, hf = l >> 5, i16 = l & 15, grp16 = (l >> 4) & 1;
  const int tiles2 = N2 / kTile;
  // Workgroups go to the 8 dies round-robin in launch order; the tiles of one slab read the same rows of A and B, so they
  // are renumbered to sit on one die (and its L2) together: die = id % 8 takes the ids' contiguous range [die * n/8, ...).
  int tile_id = blockIdx.x, slab = blockIdx.y;
  {
    const int total = gridDim.x * gridDim.y, lin = blockIdx.y * gridDim.x + blockIdx.x;
    if (total % 8 == 0) {
      const int logical = (lin % 8) * (total / 8) + lin / 8;
      tile_id = logical % gridDim.x;
      slab = logical / gridDim.x;
    }
  }
  const int n1_0 = (tile_id / tiles2) * kTile, n2_0 = (tile_id % tiles2) * kTile;
  const int64_t t_begin = (int64_t)slab * slab_rows, t_end = min(t_begin + slab_rows, T);
  const int wi = w >> 1, wj = w & 1;       // this wave's 64 x 64 quarter of the tile

  // staging: thread -> rows t/16 + 16 i of the tile, 16-byte chunk t%16
  constexpr int NP = kBK / 16;
  const int srow = t >> 4, schunk = t & 15;
  u32x4 pa[NP], pb[NP];
  auto gload = [&](int64_t r0) {
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const int64_t r = r0 + srow + 16 * i;
      pa[i] = (u32x4){0u, 0u, 0u, 0u};
      pb[i] = (u32x4){0u, 0u, 0u, 0u};
      if (r < t_end) {
        pa[i] = *(const u32x4*)(A + r * lda + n1_0 + 8 * schunk);
        pb[i] = *(const u32x4*)(B + r * ldb + n2_0 + 8 * schunk);
      }
    }
  };
  auto lstore = [&](int stage) {
    unsigned char* base = smem + stage * 2 * kOperand;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const int off = (srow + 16 * i) * kPitch + 16 * (schunk ^ (4 * (srow & 3) + ((srow >> 2) & 3)));
      *(u32x4*)(base + off) = pa[i];
      *(u32x4*)(base + kOperand + off) = pb[i];
    }
  };
  // transposed fragment: rows [k0, k0 + 16) of an operand tile, features [f0, f0 + 32): lane l32 gets feature f0 + l32,
  // 8 values of k that depend on hf only.  Within a group of 16 lanes, lane i16 addresses row 4 hf + i16 / 4 (and +8),
  // chunk 2 (grp16) + (i16 % 4) / 2 of the 32 features, half 8 (i16 % 2) of that chunk.
  const int vchunk = 2 * grp16 + ((i16 & 3) >> 1), vbyte = 8 * (i16 & 1);
  // the rows' swizzle: row % 4 = i16 / 4, (row / 4) % 4 = hf for the first load and hf + 2 for the second (8 rows further)
  const int lane_row = (4 * hf + (i16 >> 2)) * kPitch, lane_swz = 4 * (i16 >> 2);
  const int vlo = 16 * (vchunk ^ hf) + vbyte, vhi = 16 * (vchunk ^ (hf + 2)) + vbyte + 8 * kPitch;
  auto trfrag = [&](const unsigned char* tile, int k0, int f0) -> bf16x8 {
    const unsigned char* p = tile + k0 * kPitch + lane_row + 16 * ((f0 >> 3) ^ lane_swz);
    const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(p + vlo));
    const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(p + vhi));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;

  gload(t_begin);
  int stage = 0;
  for (int64_t r0 = t_begin; r0 < t_end; r0 += kBK) {
    lstore(stage);
    __syncthreads();                                  // tile visible; the other stage is free again (all waves passed its products)
    if (r0 + kBK < t_end) gload(r0 + kBK);
    const unsigned char* at = smem + stage * 2 * kOperand;
    const unsigned char* bt = at + kOperand;
#pragma unroll
    for (int k0 = 0; k0 < kBK; k0 += 16) {
      bf16x8 af[2], bf[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) af[i] = trfrag(at, k0, 64 * wi + 32 * i);
#pragma unroll
      for (int j = 0; j < 2; ++j) bf[j] = trfrag(bt, k0, 64 * wj + 32 * j);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
    stage ^= 1;
  }

  // partial tile: accumulator lane = n2, registers = n1
  float* out = partial + ((int64_t)slab * N1 + n1_0 + 64 * wi) * N2 + n2_0 + 64 * wj + l32;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) out[(int64_t)(32 * i + 8 * (q >> 2) + 4 * hf + (q & 3)) * N2 + 32 * j] = acc[i][j][q];
}

// C = sum over slabs of partial, in slab order
__global__ __launch_bounds__(256) void gemm_tn_reduce_kernel(int64_t elems4, int nslab, const f32x4* __restrict__ partial,
                                                             f32x4* __restrict__ C) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= elems4) return;
  f32x4 s = partial[i];
  for (int k = 1; k < nslab; ++k) s += partial[(int64_t)k * elems4 + i];
  C[i] = s;
}

}  // namespace

bool gemm_tn_supported(int N1, int N2) { return N1 >= kTile && N2 >= kTile && N1 % kTile == 0 && N2 % kTile == 0; }

// slabs so that the grid is about 1024 workgroups (two rounds of two per compute unit), each slab a multiple of the row tile
int gemm_tn_slabs(int64_t T, int N1, int N2) {
  const int tiles = (N1 / kTile) * (N2 / kTile);
  int64_t nslab = (1024 + tiles - 1) / tiles;
  const int64_t max_slabs = (T + 4 * kBK - 1) / (4 * kBK);           // at least four tiles per slab
  if (nslab > max_slabs) nslab = max_slabs;
  if (nslab < 1) nslab = 1;
  return (int)nslab;
}

size_t gemm_tn_workspace_bytes(int64_t T, int N1, int N2) {
  return (size_t)gemm_tn_slabs(T, N1, N2) * (size_t)N1 * (size_t)N2 * sizeof(float);
}

hipError_t launch_gemm_tn(int64_t T, int N1, int N2, const void* A, int64_t lda, const void* B, int64_t ldb, float* C, float* partial,
                          hipStream_t stream) {
  const int nslab = gemm_tn_slabs(T, N1, N2);
  int64_t slab_rows = (T + nslab - 1) / nslab;
  slab_rows = (slab_rows + kBK - 1) / kBK * kBK;
  const dim3 grid((N1 / kTile) * (N2 / kTile), nslab);
  constexpr int smem = 2 * 2 * kOperand;
  static bool attr_set[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (!attr_set[dev]) {
    const hipError_t ea = hipFuncSetAttribute((const void*)gemm_tn_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (ea != hipSuccess) return ea;
    attr_set[dev] = true;
  }
  hipLaunchKernelGGL(gemm_tn_kernel, grid, dim3(256), smem, stream, (const __bf16*)A, lda, (const __bf16*)B, ldb, N1, N2, T, slab_rows,
                     partial);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int64_t elems4 = (int64_t)N1 * N2 / 4;
  hipLaunchKernelGGL(gemm_tn_reduce_kernel, dim3((unsigned)((elems4 + 255) / 256)), dim3(256), 0, stream, elems4, nslab,
                     (const f32x4*)partial, (f32x4*)C);
  return hipGetLastError();
}

}  // namespace hstu
