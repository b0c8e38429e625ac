// FP8 projection with a two-dimensional additive operand (paper Section 4.2.2 and the FP8 GEMM benchmark of the
// appendix: D = A B + C with C in R^{m x n}, the post-attention projection whose output is accumulated with the residual):
//   D[m, n] = a_scale[m] * b_scale[n] * sum_k Aq[m, k] Bq[n, k]  +  C[m, n]
// Aq [M, K] and Bq [N, K] are E4M3 codes with one fp32 scale per row (activations per token, weights per output feature),
// C and D are bf16.  M is the jagged token count (10^5..10^6), K and N are model widths (<= 1024): per output row the
// kernel owes 2 K N FLOPs and moves K + 4 N bytes, 205 FLOP/B at K = N = 512, so it is HBM-bound far below the FP8 matrix
// peak; the design goal is to stream A, C and D once at full-line granularity and keep the matrix work out of the way.
//
// One workgroup (4 waves) owns 128 rows of A.  A wave keeps its 32 rows as matrix-core operands in registers for the whole
// tile (K / 8 registers per lane).  The weights go through LDS in chunks of 64 output features (XOR-swizzled 16-byte
// pieces, conflict-free fragment reads), shared by the four waves.  v_mfma_f32_32x32x64_f8f6f4 with the weight rows on the
// accumulator's register axis and the token rows on its lane axis: a lane then owns one token row, its a_scale is a
// scalar, and the 4 consecutive features of a register group go to LDS as one 16-byte write.  From there the chunk is
// read back row-contiguous (8 features = 16 bytes of bf16 per lane, 128 contiguous bytes per row), added to C, which was
// fetched in that same layout before the products were issued, rounded once to bf16 and stored: every global access of
// C and D is a full 128-byte row segment.
#include "hstu_common.h"
#include "hstu_kernels.h"

namespace hstu {
namespace {

typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kBM = 128;            // rows of A per workgroup

// K = 64 * KS; kBN output features per chunk (64: full 128-byte row segments of C and D).  At K = 1024 the resident rows
// of A take 128 registers per lane and one workgroup runs per compute unit; 32-feature chunks at two workgroups per compute
// unit spilled and measured 25 % slower.
// SILU: the epilogue applies x sigmoid(x) before the rounding (the first projection of the layer, Eq. 2), and output
// features [0, u_cols) go to u_out [M, u_cols] instead of D (the gate is kept apart from the rest of the projection).
template <int KS, int kBN, bool SILU>
__global__ __launch_bounds__(256, KS >= 16 ? 1 : 2) void fp8_gemm_bias2d_kernel(int64_t M, int N, const unsigned char* __restrict__ A,
                                                                  const float* __restrict__ a_scale,
                                                                  const unsigned char* __restrict__ B,
                                                                  const float* __restrict__ b_scale, const __bf16* __restrict__ C,
                                                                  __bf16* __restrict__ D, __bf16* __restrict__ u_out, int u_cols) {
  constexpr int K = 64 * KS;
  constexpr int CPR = K / 16;                         // 16-byte pieces per weight row
  constexpr int SWZ = CPR >= 16 ? 15 : CPR - 1;       // pieces are XORed with the low bits of the row
  constexpr int kEpiPitch = kBN + 4;                  // floats per row of the epilogue staging area: the 16-byte writes of 32 lanes hit all banks
  constexpr int NT = kBN / 32;                        // 32-feature accumulator tiles per chunk
  constexpr int BP = kBN * CPR / 256;                 // 16-byte weight pieces per thread and chunk
  constexpr int LPR = kBN / 8;                        // lanes per row in the row-contiguous layout of C and D
  constexpr int RPI = 64 / LPR;                       // rows per wave instruction there
  constexpr int NI = 32 / RPI;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* bl = smem;                           // [kBN][K] weight chunk
  float* epi = (float*)(smem + kBN * K);              // [4 waves][32][kEpiPitch]
  float* sbl = epi + 4 * 32 * kEpiPitch;              // [N] weight scales
  const int t = threadIdx.x, w = t >> 6, l = t & 63, r = l & 31, h = l >> 5;
  const int64_t m0 = (int64_t)blockIdx.x * kBM + 32 * w;
  const int64_t gm = m0 + r;                          // this lane's token row
  const bool row_ok = gm < M;

  // ---- this wave's rows of A as B operands: lane (r, h) holds bytes [64 s + 32 h, +32) of row r for every k-step s
  i32x8 af[KS];
  {
    const unsigned char* ap = A + gm * K + 32 * h;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      u32x4 lo = {0u, 0u, 0u, 0u}, hi = {0u, 0u, 0u, 0u};
      if (row_ok) { lo = *(const u32x4*)(ap + 64 * s); hi = *(const u32x4*)(ap + 64 * s + 16); }
      af[s] = (i32x8){(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
    }
  }
  const float sa = row_ok ? a_scale[gm] : 0.f;

  // ---- staging of a weight chunk: piece p = t + 256 i is piece p % CPR of row p / CPR
  u32x4 bpre[BP];
  auto bload = [&](int n0) {
#pragma unroll
    for (int i = 0; i < BP; ++i) {
      const int p = t + 256 * i;
      bpre[i] = *(const u32x4*)(B + (int64_t)(n0 + p / CPR) * K + 16 * (p % CPR));
    }
  };
  auto bstore = [&]() {
#pragma unroll
    for (int i = 0; i < BP; ++i) {
      const int p = t + 256 * i, n = p / CPR, c = p % CPR;
      *(u32x4*)(bl + n * K + 16 * (c ^ (n & SWZ))) = bpre[i];
    }
  };
  // C in the row-contiguous layout of the stores: LPR lanes cover the chunk's features of a row, RPI rows per instruction
  const int er = l / LPR, ec = l % LPR;
  u32x4 cpre[NI];
  auto cload = [&](int n0) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int64_t row = m0 + RPI * i + er;
      cpre[i] = (u32x4){0u, 0u, 0u, 0u};
      if (C && row < M) cpre[i] = *(const u32x4*)(C + row * N + n0 + 8 * ec);
    }
  };

  for (int i = t; i < N; i += 256) sbl[i] = b_scale[i];   // visible after the first barrier of the chunk loop
  bload(0);
  cload(0);
  float* my_epi = epi + w * 32 * kEpiPitch;
  const int swz = r & SWZ;
  for (int n0 = 0; n0 < N; n0 += kBN) {
    __syncthreads();                                  // every wave is done with the previous chunk's fragments
    bstore();
    __syncthreads();
    if (n0 + kBN < N) bload(n0 + kBN);                // the next chunk travels while this one is multiplied
    f32x16 acc[NT];
#pragma unroll
    for (int jt = 0; jt < NT; ++jt)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[jt][q] = 0.f;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
#pragma unroll
      for (int jt = 0; jt < NT; ++jt) {
        const unsigned char* brow = bl + (32 * jt + r) * K;
        const u32x4 lo = *(const u32x4*)(brow + 16 * ((4 * s + 2 * h) ^ swz));
        const u32x4 hi = *(const u32x4*)(brow + 16 * ((4 * s + 2 * h + 1) ^ swz));
        const i32x8 bf = (i32x8){(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
        // weight rows on the register axis (i), token rows on the lane axis (j)
        acc[jt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(bf, af[s], acc[jt], 0, 0, 0, 0, 0, 0);
      }
    }

    // ---- epilogue: scale, transpose through LDS (this wave's area only), add C, round once, store full row segments
#pragma unroll
    for (int jt = 0; jt < NT; ++jt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const f32x4 sb = *(const f32x4*)(sbl + n0 + 32 * jt + 8 * g + 4 * h);   // weight scales of this register group
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = acc[jt][4 * g + e] * sa * sb[e];
        *(f32x4*)(my_epi + r * kEpiPitch + 32 * jt + 8 * g + 4 * h) = v;
      }
    // (LDS operations of one wave complete in order: the reads below see the writes above without a barrier)
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int64_t row = m0 + RPI * i + er;
      const float* src = my_epi + (RPI * i + er) * kEpiPitch + 8 * ec;
      const f32x4 x0 = *(const f32x4*)src, x1 = *(const f32x4*)(src + 4);
      float o[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        o[2 * e] = __uint_as_float(cpre[i][e] << 16);
        o[2 * e + 1] = __uint_as_float(cpre[i][e] & 0xFFFF0000u);
      }
      o[0] += x0[0]; o[1] += x0[1]; o[2] += x0[2]; o[3] += x0[3];
      o[4] += x1[0]; o[5] += x1[1]; o[6] += x1[2]; o[7] += x1[3];
      if constexpr (SILU) {
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] *= __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * o[e]));
      }
      __bf16* dst = D + row * N + n0 + 8 * ec;
      if constexpr (SILU) { if (n0 < u_cols) dst = u_out + row * u_cols + n0 + 8 * ec; }    // a chunk never straddles the gate's block
      if (row < M)
        *(u32x4*)dst = (u32x4){pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]), pack_bf16x2(o[4], o[5]), pack_bf16x2(o[6], o[7])};
    }
    // C of the next chunk: a whole chunk period (barriers, products) ahead of its use, in the registers just consumed
    if (n0 + kBN < N) cload(n0 + kBN);
  }
}

// K = 1024: the resident rows of A would take 128 registers per lane and leave one wave per SIMD.  Here a workgroup has 8
// waves, two per 32-row block, each holding one half of K (64 registers) and accumulating its half of every dot product.
// Both waves of a pair leave their raw partial sums in LDS; after a workgroup barrier each reads back 16 of the pair's 32
// rows in the row-contiguous layout from both areas, adds them, applies the scales and C and stores.  KSW k-steps per wave.
template <int KSW, bool SILU>
__global__ __launch_bounds__(512, 1) void fp8_gemm_ksplit_kernel(int64_t M, int N, const unsigned char* __restrict__ A,
                                                                  const float* __restrict__ a_scale,
                                                                  const unsigned char* __restrict__ B,
                                                                  const float* __restrict__ b_scale, const __bf16* __restrict__ C,
                                                                  __bf16* __restrict__ D, __bf16* __restrict__ u_out, int u_cols) {
  constexpr int K = 128 * KSW, kBN = 64, CPR = K / 16, SWZ = 15, kEpiPitch = kBN + 4, BP = kBN * CPR / 512;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* bl = smem;                           // [kBN][K] weight chunk
  float* epi = (float*)(smem + kBN * K);              // [8 waves][32][kEpiPitch] raw partial sums
  float* sbl = epi + 8 * 32 * kEpiPitch;              // [N] weight scales
  const int t = threadIdx.x, w = t >> 6, l = t & 63, r = l & 31, h = l >> 5;
  const int rb = w & 3, kh = w >> 2;                  // row block of the workgroup's 128 rows, half of K
  const int64_t m0 = (int64_t)blockIdx.x * kBM + 32 * rb;
  const int64_t gm = m0 + r;
  const bool row_ok = gm < M;
  i32x8 af[KSW];
  {
    const unsigned char* ap = A + gm * K + 64 * KSW * kh + 32 * h;
#pragma unroll
    for (int s = 0; s < KSW; ++s) {
      u32x4 lo = {0u, 0u, 0u, 0u}, hi = {0u, 0u, 0u, 0u};
      if (row_ok) { lo = *(const u32x4*)(ap + 64 * s); hi = *(const u32x4*)(ap + 64 * s + 16); }
      af[s] = (i32x8){(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
    }
  }
  u32x4 bpre[BP];
  auto bload = [&](int n0) {
#pragma unroll
    for (int i = 0; i < BP; ++i) {
      const int p = t + 512 * i;
      bpre[i] = *(const u32x4*)(B + (int64_t)(n0 + p / CPR) * K + 16 * (p % CPR));
    }
  };
  auto bstore = [&]() {
#pragma unroll
    for (int i = 0; i < BP; ++i) {
      const int p = t + 512 * i, n = p / CPR, c = p % CPR;
      *(u32x4*)(bl + n * K + 16 * (c ^ (n & SWZ))) = bpre[i];
    }
  };
  // read-back: this wave finishes rows [16 kh, 16 kh + 16) of its pair's block; 8 lanes per row, 8 rows per instruction
  const int er = l >> 3, ec = l & 7;
  u32x4 cpre[2];
  float sa_row[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int64_t row = m0 + 16 * kh + 8 * i + er;
    sa_row[i] = row < M ? a_scale[row] : 0.f;
  }
  auto cload = [&](int n0) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int64_t row = m0 + 16 * kh + 8 * i + er;
      cpre[i] = (u32x4){0u, 0u, 0u, 0u};
      if (C && row < M) cpre[i] = *(const u32x4*)(C + row * N + n0 + 8 * ec);
    }
  };
  for (int i = t; i < N; i += 512) sbl[i] = b_scale[i];
  bload(0);
  cload(0);
  float* my_epi = epi + w * 32 * kEpiPitch;
  const float* pair0 = epi + rb * 32 * kEpiPitch;             // partial sums of the pair's K halves
  const float* pair1 = epi + (4 + rb) * 32 * kEpiPitch;
  const int swz = r & SWZ;
  for (int n0 = 0; n0 < N; n0 += kBN) {
    __syncthreads();                                  // fragments and partial sums of the previous chunk are consumed
    bstore();
    __syncthreads();
    if (n0 + kBN < N) bload(n0 + kBN);
    f32x16 acc[2];
#pragma unroll
    for (int jt = 0; jt < 2; ++jt)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[jt][q] = 0.f;
#pragma unroll
    for (int s = 0; s < KSW; ++s) {
#pragma unroll
      for (int jt = 0; jt < 2; ++jt) {
        const unsigned char* brow = bl + (32 * jt + r) * K;
        const int c0 = 4 * (KSW * kh + s) + 2 * h;
        const u32x4 lo = *(const u32x4*)(brow + 16 * (c0 ^ swz));
        const u32x4 hi = *(const u32x4*)(brow + 16 * ((c0 + 1) ^ swz));
        const i32x8 bf = (i32x8){(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
        acc[jt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(bf, af[s], acc[jt], 0, 0, 0, 0, 0, 0);
      }
    }
#pragma unroll
    for (int jt = 0; jt < 2; ++jt)
#pragma unroll
      for (int g = 0; g < 4; ++g)
        *(f32x4*)(my_epi + r * kEpiPitch + 32 * jt + 8 * g + 4 * h) =
            (f32x4){acc[jt][4 * g + 0], acc[jt][4 * g + 1], acc[jt][4 * g + 2], acc[jt][4 * g + 3]};
    __syncthreads();                                  // both halves of every pair are in LDS
    const f32x4 sb0 = *(const f32x4*)(sbl + n0 + 8 * ec), sb1 = *(const f32x4*)(sbl + n0 + 8 * ec + 4);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int lr = 16 * kh + 8 * i + er;
      const int64_t row = m0 + lr;
      const float* s0 = pair0 + lr * kEpiPitch + 8 * ec;
      const float* s1 = pair1 + lr * kEpiPitch + 8 * ec;
      const f32x4 x0 = *(const f32x4*)s0 + *(const f32x4*)s1, x1 = *(const f32x4*)(s0 + 4) + *(const f32x4*)(s1 + 4);
      float o[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        o[2 * e] = __uint_as_float(cpre[i][e] << 16);
        o[2 * e + 1] = __uint_as_float(cpre[i][e] & 0xFFFF0000u);
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        o[e] += x0[e] * sa_row[i] * sb0[e];
        o[4 + e] += x1[e] * sa_row[i] * sb1[e];
      }
      if constexpr (SILU) {
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] *= __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * o[e]));
      }
      __bf16* dst = D + row * N + n0 + 8 * ec;
      if constexpr (SILU) { if (n0 < u_cols) dst = u_out + row * u_cols + n0 + 8 * ec; }
      if (row < M)
        *(u32x4*)dst = (u32x4){pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]), pack_bf16x2(o[4], o[5]), pack_bf16x2(o[6], o[7])};
    }
    if (n0 + kBN < N) cload(n0 + kBN);
  }
}

template <int KSW, bool SILU>
hipError_t launch_ksplit(int64_t M, int N, const void* A, const float* a_scale, const void* B, const float* b_scale, const void* C,
                         void* D, void* u_out, int u_cols, hipStream_t stream) {
  auto kern = fp8_gemm_ksplit_kernel<KSW, SILU>;
  const size_t smem = (size_t)64 * 128 * KSW + (size_t)8 * 32 * (64 + 4) * sizeof(float) + (size_t)N * sizeof(float);
  static bool attr_set[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (!attr_set[dev]) {
    const hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    attr_set[dev] = true;
  }
  const unsigned grid = (unsigned)((M + kBM - 1) / kBM);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(512), smem, stream, M, N, (const unsigned char*)A, a_scale, (const unsigned char*)B,
                     b_scale, (const __bf16*)C, (__bf16*)D, (__bf16*)u_out, u_cols);
  return hipGetLastError();
}

template <int KS, int kBN, bool SILU>
hipError_t launch_one(int64_t M, int N, const void* A, const float* a_scale, const void* B, const float* b_scale, const void* C,
                      void* D, void* u_out, int u_cols, hipStream_t stream) {
  auto kern = fp8_gemm_bias2d_kernel<KS, kBN, SILU>;
  const size_t smem = (size_t)kBN * 64 * KS + (size_t)4 * 32 * (kBN + 4) * sizeof(float) + (size_t)N * sizeof(float);
  static bool attr_set[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (!attr_set[dev]) {
    const hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    attr_set[dev] = true;
  }
  const unsigned grid = (unsigned)((M + kBM - 1) / kBM);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(256), smem, stream, M, N, (const unsigned char*)A, a_scale, (const unsigned char*)B,
                     b_scale, (const __bf16*)C, (__bf16*)D, (__bf16*)u_out, u_cols);
  return hipGetLastError();
}

}  // namespace

// (the K = 1024 kernel keeps 138 KB + 4 N bytes in LDS)
bool fp8_gemm_supported(int N, int K) { return (K == 128 || K == 256 || K == 512 || K == 1024) && N >= 64 && N % 64 == 0 && N <= 4096; }

hipError_t launch_fp8_gemm_bias2d(int64_t M, int N, int K, const void* A, const float* a_scale, const void* B, const float* b_scale,
                                  const void* C, void* D, hipStream_t stream) {
  switch (K) {
    case 128: return launch_one<2, 64, false>(M, N, A, a_scale, B, b_scale, C, D, nullptr, 0, stream);
    case 256: return launch_one<4, 64, false>(M, N, A, a_scale, B, b_scale, C, D, nullptr, 0, stream);
    case 512: return launch_one<8, 64, false>(M, N, A, a_scale, B, b_scale, C, D, nullptr, 0, stream);
    case 1024: return launch_ksplit<8, false>(M, N, A, a_scale, B, b_scale, C, D, nullptr, 0, stream);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_fp8_gemm_silu(int64_t M, int N, int K, const void* A, const float* a_scale, const void* B, const float* b_scale,
                                void* D, void* u_out, int u_cols, hipStream_t stream) {
  if (u_cols % 64 != 0 || (u_cols > 0 && !u_out)) return hipErrorInvalidValue;
  switch (K) {
    case 128: return launch_one<2, 64, true>(M, N, A, a_scale, B, b_scale, nullptr, D, u_out, u_cols, stream);
    case 256: return launch_one<4, 64, true>(M, N, A, a_scale, B, b_scale, nullptr, D, u_out, u_cols, stream);
    case 512: return launch_one<8, 64, true>(M, N, A, a_scale, B, b_scale, nullptr, D, u_out, u_cols, stream);
    case 1024: return launch_ksplit<8, true>(M, N, A, a_scale, B, b_scale, nullptr, D, u_out, u_cols, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace hstu
