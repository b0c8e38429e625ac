// SiLU of the U/V/Q/K projection (paper Eq. 2, phi_1) and its backward: HBM-bound elementwise kernels over
// contiguous bf16 [T, C] buffers, 8 elements (16 bytes) per lane and step.
#include "hstu_common.h"
#include "hstu_kernels.h"

namespace hstu {
namespace {

constexpr int kThreads = 256;
constexpr int kMaxBlocks = 256 * 16;

__device__ __forceinline__ void unpack8(const u32x4 raw, float (&v)[8]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    v[2 * i] = __uint_as_float(raw[i] << 16);
    v[2 * i + 1] = __uint_as_float(raw[i] & 0xFFFF0000u);
  }
}
__device__ __forceinline__ u32x4 pack8(const float (&v)[8]) {
  return (u32x4){pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7])};
}
__device__ __forceinline__ float sigmoidf_fast(float t) {
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * t));
}

// act = pre * sigmoid(pre); `act` may be `pre` itself.  Columns [0, u_cols) of every row also go to u_out [T, u_cols]
// (the gate is kept for the backward while the rest of the projection is dropped), when u_out is given.  Columns before
// skip8 (in 8-element groups) are neither read nor written (the backward rebuilds V, Q, K only: the gate was saved).
__global__ __launch_bounds__(kThreads) void silu_fwd_kernel(int64_t groups, int C8, int skip8, const u32x4* pre, u32x4* act,
                                                            u32x4* __restrict__ u_out, int u8) {
  const int W8 = C8 - skip8;
  for (int64_t gi = (int64_t)blockIdx.x * kThreads + threadIdx.x; gi < groups; gi += (int64_t)gridDim.x * kThreads) {
    const int64_t row = gi / W8;
    const int col = skip8 + (int)(gi - row * W8);
    const int64_t g = row * C8 + col;
    float v[8];
    unpack8(pre[g], v);
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] *= sigmoidf_fast(v[i]);
    const u32x4 o = pack8(v);
    act[g] = o;
    if (u_out && col < u8) u_out[row * u8 + col] = o;
  }
}

// dpre = dact * d/dt [t sigmoid(t)] at t = pre, written over dact.
__global__ __launch_bounds__(kThreads) void silu_bwd_kernel(int64_t groups, const u32x4* __restrict__ pre, u32x4* __restrict__ dact) {
  for (int64_t g = (int64_t)blockIdx.x * kThreads + threadIdx.x; g < groups; g += (int64_t)gridDim.x * kThreads) {
    float t[8], d[8];
    unpack8(pre[g], t);
    unpack8(dact[g], d);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float sg = sigmoidf_fast(t[i]);
      d[i] *= sg * (1.0f + t[i] * (1.0f - sg));
    }
    dact[g] = pack8(d);
  }
}

int blocks_for(int64_t groups) {
  const int64_t b = (groups + kThreads - 1) / kThreads;
  return (int)(b < 1 ? 1 : (b > kMaxBlocks ? kMaxBlocks : b));
}

}  // namespace

hipError_t launch_silu_fwd(int64_t T, int C, const void* pre, void* act, void* u_out, int u_cols, hipStream_t stream, int skip_cols) {
  const int64_t groups = T * ((C - skip_cols) / 8);
  if (groups <= 0) return hipSuccess;
  hipLaunchKernelGGL(silu_fwd_kernel, dim3(blocks_for(groups)), dim3(kThreads), 0, stream, groups, C / 8, skip_cols / 8, (const u32x4*)pre,
                     (u32x4*)act, (u32x4*)u_out, u_cols / 8);
  return hipGetLastError();
}

hipError_t launch_silu_bwd(int64_t T, int C, const void* pre, void* dact, hipStream_t stream) {
  const int64_t groups = T * (C / 8);
  hipLaunchKernelGGL(silu_bwd_kernel, dim3(blocks_for(groups)), dim3(kThreads), 0, stream, groups, (const u32x4*)pre, (u32x4*)dact);
  return hipGetLastError();
}

}  // namespace hstu
