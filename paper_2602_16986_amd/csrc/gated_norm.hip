// U-gated layer normalisation after the attention (paper Eq. 4 without the f2 projection):
//   Y = (LayerNorm_D(A) * gamma + beta) * U          over the D = H*d features of each token
// and its backward (gated_norm_backward of the paper's appendix pseudocode, which recomputes the
// normalised activations instead of saving them).  Both passes are HBM-bound streaming kernels:
// one wavefront per token row, 16-byte loads per lane, wave-level reductions through DPP
// shuffles, everything between the load and the store in registers.
#include "hstu_common.h"
#include "hstu_kernels.h"

namespace hstu {

constexpr int kRowsPerBlock = 4;        // forward: one wave per row, 4 waves per workgroup
constexpr int kBwdWaves = 8;            // backward: 8 waves per workgroup, each walking over rows
constexpr int kMaxBwdBlocks = 512;      // two workgroups per CU; also the number of partial column-sum rows

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
  return v;
}

// 8 consecutive elements starting at element index e0 of a row, widened to fp32
template <typename E>
__device__ __forceinline__ void load8(const E* row, int e0, float (&v)[8]) {
  if constexpr (sizeof(E) == 2) {
    const u32x4 raw = *(const u32x4*)(row + e0);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = __uint_as_float(raw[i] << 16);
      v[2 * i + 1] = __uint_as_float(raw[i] & 0xFFFF0000u);
    }
  } else {
    const f32x4 a = *(const f32x4*)(row + e0), b = *(const f32x4*)(row + e0 + 4);
#pragma unroll
    for (int i = 0; i < 4; ++i) { v[i] = a[i]; v[4 + i] = b[i]; }
  }
}

template <typename E>
__device__ __forceinline__ void store8(E* row, int e0, const float (&v)[8]) {
  if constexpr (sizeof(E) == 2) {
    *(u32x4*)(row + e0) = (u32x4){pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]),
                                  pack_bf16x2(v[6], v[7])};
  } else {
    *(f32x4*)(row + e0) = (f32x4){v[0], v[1], v[2], v[3]};
    *(f32x4*)(row + e0 + 4) = (f32x4){v[4], v[5], v[6], v[7]};
  }
}
// v[i] *= d/dt [t sigmoid(t)] at t = pre[e0 + i]: the gradient passes back through a SiLU whose input is `pre`
// 8 consecutive elements as loaded (one 16-byte chunk of bf16, two of fp32), widened when they are used
template <typename E> struct Raw8;
template <> struct Raw8<__bf16> { u32x4 w; };
template <> struct Raw8<float> { f32x4 lo, hi; };
__device__ __forceinline__ Raw8<__bf16> load8raw(const __bf16* row, int e0) { return {*(const u32x4*)(row + e0)}; }
__device__ __forceinline__ Raw8<float> load8raw(const float* row, int e0) { return {*(const f32x4*)(row + e0), *(const f32x4*)(row + e0 + 4)}; }
__device__ __forceinline__ void widen8(const Raw8<__bf16>& r, float (&v)[8]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    v[2 * i] = __uint_as_float(r.w[i] << 16);
    v[2 * i + 1] = __uint_as_float(r.w[i] & 0xFFFF0000u);
  }
}
__device__ __forceinline__ void widen8(const Raw8<float>& r, float (&v)[8]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) { v[i] = r.lo[i]; v[4 + i] = r.hi[i]; }
}

template <typename E>
__device__ __forceinline__ void dsilu8(const E* pre, int e0, float (&v)[8]) {
  float t[8];
  load8(pre, e0, t);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const float sg = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * t[i]));
    v[i] *= sg * (1.0f + t[i] * (1.0f - sg));
  }
}

// mean and reciprocal standard deviation of one row held as NCH chunks of 8 per lane
template <int NCH>
__device__ __forceinline__ void row_stats(const float (&a)[NCH][8], int lane, int D, float eps, float& mu, float& rs) {
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < NCH; ++c)
    if ((lane + 64 * c) * 8 < D)
#pragma unroll
      for (int i = 0; i < 8; ++i) s += a[c][i];
  mu = wave_sum(s) / (float)D;
  float q = 0.f;
#pragma unroll
  for (int c = 0; c < NCH; ++c)
    if ((lane + 64 * c) * 8 < D)
#pragma unroll
      for (int i = 0; i < 8; ++i) { const float dlt = a[c][i] - mu; q += dlt * dlt; }
  const float var = wave_sum(q) / (float)D;
  rs = 1.0f / sqrtf(var + eps);
}

template <typename E, int NCH>
__global__ __launch_bounds__(64 * kRowsPerBlock) void gated_norm_fwd_kernel(const NormFwdArgs p) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row = (int64_t)blockIdx.x * kRowsPerBlock + wave;
  const int D = p.D;
  if (row >= p.T) return;
  const E* arow = (const E*)p.a + row * p.sa;
  const E* urow = p.u ? (const E*)p.u + row * p.su : nullptr;       // no gate: plain layer norm
  E* yrow = (E*)p.y + row * p.sy;
  float a[NCH][8];
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int e0 = (lane + 64 * c) * 8;
    if (e0 < D) load8(arow, e0, a[c]);
  }
  float mu, rs;
  if (p.stats_in) { mu = p.mean[row]; rs = p.rstd[row]; }           // statistics saved by an earlier pass
  else row_stats<NCH>(a, lane, D, p.eps, mu, rs);
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int e0 = (lane + 64 * c) * 8;
    if (e0 < D) {
      float uv[8], gv[8], bv[8], out[8];
      if (urow) load8(urow, e0, uv);
      load8(p.gamma, e0, gv);
      if (p.beta) load8(p.beta, e0, bv);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        out[i] = (a[c][i] - mu) * rs * gv[i] + (p.beta ? bv[i] : 0.f);
        if (urow) out[i] *= uv[i];
      }
      store8(yrow, e0, out);
    }
  }
  if (lane == 0 && !p.stats_in) {
    if (p.mean) p.mean[row] = mu;
    if (p.rstd) p.rstd[row] = rs;
  }
}

// Forward with row-wise FP8 output (paper Section 4.2.2: the scaling and quantisation that the FP8 projections need are
// fused into the norm kernel that precedes them, Eq. 1 and Eq. 4, so that the normalised rows never make a round trip
// through memory in 16 bits).  Per row: y as in the kernel above (or, without gamma, the input rows themselves, times the
// gate if there is one: plain row-wise quantisation, used for the weights), amax = max |y|, scale = amax / 448,
// code = E4M3(y * (448 / amax)), ties to even.  All of it in fp32, one division per row and one multiplication per element.
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, 64));
  return v;
}

template <typename E, int NCH>
__global__ __launch_bounds__(64 * kRowsPerBlock) void norm_quant_fwd_kernel(const NormFwdArgs p, unsigned char* __restrict__ q,
                                                                            int64_t sq, float* __restrict__ qscale) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row = (int64_t)blockIdx.x * kRowsPerBlock + wave;
  const int D = p.D;
  if (row >= p.T) return;
  const E* arow = (const E*)p.a + row * p.sa;
  const E* urow = p.u ? (const E*)p.u + row * p.su : nullptr;
  float a[NCH][8];
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int e0 = (lane + 64 * c) * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) a[c][i] = 0.f;
    if (e0 < D) load8(arow, e0, a[c]);
  }
  float mu = 0.f, rs = 1.f;
  if (p.gamma) row_stats<NCH>(a, lane, D, p.eps, mu, rs);
  float amax = 0.f;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int e0 = (lane + 64 * c) * 8;
    if (e0 < D) {
      float uv[8], gv[8], bv[8];
      if (urow) load8(urow, e0, uv);
      if (p.gamma) load8(p.gamma, e0, gv);
      if (p.beta) load8(p.beta, e0, bv);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        float y = a[c][i];
        if (p.gamma) y = (y - mu) * rs * gv[i] + (p.beta ? bv[i] : 0.f);
        if (urow) y *= uv[i];
        a[c][i] = y;
        amax = fmaxf(amax, fabsf(y));
      }
    }
  }
  amax = wave_max(amax);
  const float safe = amax > 0.f ? amax : 448.0f;
  const float scale = safe / 448.0f;
  const float inv = 448.0f / safe;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int e0 = (lane + 64 * c) * 8;
    if (e0 < D) {
      int w0 = 0, w1 = 0;
      w0 = __builtin_amdgcn_cvt_pk_fp8_f32(a[c][0] * inv, a[c][1] * inv, w0, false);
      w0 = __builtin_amdgcn_cvt_pk_fp8_f32(a[c][2] * inv, a[c][3] * inv, w0, true);
      w1 = __builtin_amdgcn_cvt_pk_fp8_f32(a[c][4] * inv, a[c][5] * inv, w1, false);
      w1 = __builtin_amdgcn_cvt_pk_fp8_f32(a[c][6] * inv, a[c][7] * inv, w1, true);
      *(int2*)(q + row * sq + e0) = make_int2(w0, w1);
    }
  }
  if (lane == 0) {
    qscale[row] = scale;
    if (p.gamma && p.mean) p.mean[row] = mu;
    if (p.gamma && p.rstd) p.rstd[row] = rs;
  }
}

// Backward.  Per row: ahat = (a - mu) rstd, dn = dy u, dU = dy (ahat gamma + beta), dahat = dn gamma,
// dA = rstd (dahat - mean(dahat) - ahat mean(dahat ahat)).  Column sums dgamma = sum dn ahat and
// dbeta = sum dn are kept per lane over the rows a wave visits, combined across the workgroup's
// waves in a fixed order through LDS and written as one partial row per workgroup.
template <typename E, int NCH>
__global__ __launch_bounds__(64 * kBwdWaves, 4) void gated_norm_bwd_kernel(const NormBwdArgs p, float* __restrict__ partial) {
  extern __shared__ float red[];                       // [2][D]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int D = p.D;
  const float* __restrict__ gamma = p.gamma;
  const float* __restrict__ beta = p.beta;
  float gsum[NCH][8], bsum[NCH][8], gv[NCH][8], bv[NCH][8];
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int e0 = (lane + 64 * c) * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) { gsum[c][i] = 0.f; bsum[c][i] = 0.f; gv[c][i] = 0.f; bv[c][i] = 0.f; }
    if (e0 < D) {
      load8(gamma, e0, gv[c]);
      if (beta) load8(beta, e0, bv[c]);
    }
  }
  const int64_t stride = (int64_t)gridDim.x * kBwdWaves;
  for (int64_t row = (int64_t)blockIdx.x * kBwdWaves + wave; row < p.T; row += stride) {
    const E* arow = (const E*)p.a + row * p.sa;
    const E* dyrow = (const E*)p.dy + row * p.sdy;
    const E* urow = p.u ? (const E*)p.u + row * p.su : nullptr;         // no gate: plain layer norm, no dU
    const E* rrow = p.residual ? (const E*)p.residual + row * p.sres : nullptr;
    float a[NCH][8];
    Raw8<E> rraw[NCH];                                 // the residual's rows travel with the first loads, not after the reductions
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int e0 = (lane + 64 * c) * 8;
      if (e0 < D) {
        load8(arow, e0, a[c]);
        if (rrow) rraw[c] = load8raw(rrow, e0);
      }
    }
    float mu, rs;
    row_stats<NCH>(a, lane, D, p.eps, mu, rs);
    float m1 = 0.f, m2 = 0.f;
    float dah[NCH][8];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int e0 = (lane + 64 * c) * 8;
      if (e0 < D) {
        float dyv[8], uv[8], duv[8], yv[8];
        load8(dyrow, e0, dyv);
        if (urow) load8(urow, e0, uv);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float ah = (a[c][i] - mu) * rs;
          const float dn = urow ? dyv[i] * uv[i] : dyv[i];
          const float nv = ah * gv[c][i] + bv[c][i];
          duv[i] = dyv[i] * nv;
          yv[i] = urow ? nv * uv[i] : nv;
          gsum[c][i] += dn * ah;
          bsum[c][i] += dn;
          dah[c][i] = dn * gv[c][i];
          m1 += dah[c][i];
          m2 += dah[c][i] * ah;
          a[c][i] = ah;
        }
        if (urow) {
          if (p.du_pre) dsilu8((const E*)p.du_pre + row * p.sdu_pre, e0, duv);
          store8((E*)p.du + row * p.sdu, e0, duv);
          if (p.y_out) store8((E*)p.y_out + row * p.sy_out, e0, yv);
        }
      }
    }
    m1 = wave_sum(m1) / (float)D;
    m2 = wave_sum(m2) / (float)D;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int e0 = (lane + 64 * c) * 8;
      if (e0 < D) {
        float dav[8], rv[8];
        if (rrow) widen8(rraw[c], rv);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          dav[i] = rs * (dah[c][i] - m1 - a[c][i] * m2);
          if (rrow) dav[i] += rv[i];                   // gradient that bypasses the norm (residual connection)
        }
        store8((E*)p.da + row * p.sda, e0, dav);
      }
    }
  }
  // fixed-order combination of the waves' column sums
  for (int w = 0; w < kBwdWaves; ++w) {
    if (wave == w) {
#pragma unroll
      for (int c = 0; c < NCH; ++c) {
        const int e0 = (lane + 64 * c) * 8;
        if (e0 < D)
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            red[e0 + i] = (w == 0 ? 0.f : red[e0 + i]) + gsum[c][i];
            red[D + e0 + i] = (w == 0 ? 0.f : red[D + e0 + i]) + bsum[c][i];
          }
      }
    }
    __syncthreads();
  }
  float* prow = partial + (int64_t)blockIdx.x * 2 * D;
  for (int i = threadIdx.x; i < 2 * D; i += blockDim.x) prow[i] = red[i];
}

// Backward for rows wider than 512 features: a workgroup of W waves shares one row, every thread owns one 16-byte chunk
// of it (and the column sums of those 8 features over all the rows its workgroup visits, so the waves need no combination
// at the end).  The row statistics cross the waves through LDS with two barriers per row: the sum of a first, then
// sum (a - mu)^2, sum dahat and sum dahat (a - mu) together (mean(dahat ahat) = rstd times the last one / D).  The slots
// alternate with the row parity, so a wave that runs ahead never overwrites what a slower one still reads.  One wave per
// row needed 48 registers per 512 features (and spilled from 2048 features on).
template <typename E, int W>
__global__ __launch_bounds__(64 * W) void gated_norm_bwd_wide_kernel(const NormBwdArgs p, float* __restrict__ partial) {
  __shared__ float red1[2][W];
  __shared__ float red2[2][3][W];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int D = p.D, e0 = threadIdx.x * 8;
  const bool on = e0 < D;
  float gv[8], bv[8], gsum[8], bsum[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) { gv[i] = 0.f; bv[i] = 0.f; gsum[i] = 0.f; bsum[i] = 0.f; }
  if (on) {
    load8(p.gamma, e0, gv);
    if (p.beta) load8(p.beta, e0, bv);
  }
  const float inv_d = 1.0f / (float)D;
  int par = 0;
  for (int64_t row = blockIdx.x; row < p.T; row += gridDim.x, par ^= 1) {
    const E* arow = (const E*)p.a + row * p.sa;
    const E* dyrow = (const E*)p.dy + row * p.sdy;
    const E* urow = p.u ? (const E*)p.u + row * p.su : nullptr;         // no gate: plain layer norm, no dU
    const E* rrow = p.residual ? (const E*)p.residual + row * p.sres : nullptr;
    float a[8], dn[8], dyv[8], rv[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) { a[i] = 0.f; dn[i] = 0.f; dyv[i] = 0.f; rv[i] = 0.f; }
    if (on) {
      load8(arow, e0, a);
      load8(dyrow, e0, dyv);
      if (urow) load8(urow, e0, dn);
      if (rrow) load8(rrow, e0, rv);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) s += a[i];
    s = wave_sum(s);
    if (lane == 0) red1[par][wave] = s;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < W; ++w) tot += red1[par][w];
    const float mu = tot * inv_d;
    float q = 0.f, s1 = 0.f, s2 = 0.f, dah[8], uk[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float c = on ? a[i] - mu : 0.f;
      uk[i] = dn[i];                                   // the gate, for the optional Y output
      dn[i] = urow ? dyv[i] * dn[i] : dyv[i];
      dah[i] = dn[i] * gv[i];
      q += c * c;
      s1 += dah[i];
      s2 += dah[i] * c;
      a[i] = c;
    }
    q = wave_sum(q); s1 = wave_sum(s1); s2 = wave_sum(s2);
    if (lane == 0) { red2[par][0][wave] = q; red2[par][1][wave] = s1; red2[par][2][wave] = s2; }
    __syncthreads();
    float tq = 0.f, t1 = 0.f, t2 = 0.f;
#pragma unroll
    for (int w = 0; w < W; ++w) { tq += red2[par][0][w]; t1 += red2[par][1][w]; t2 += red2[par][2][w]; }
    const float rs = 1.0f / sqrtf(tq * inv_d + p.eps);
    const float m1 = t1 * inv_d, m2 = rs * t2 * inv_d;
    if (on) {
      float duv[8], dav[8], yv[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float ah = a[i] * rs;
        const float nv = ah * gv[i] + bv[i];
        duv[i] = dyv[i] * nv;
        yv[i] = nv * uk[i];
        gsum[i] += dn[i] * ah;
        bsum[i] += dn[i];
        dav[i] = rs * (dah[i] - m1 - ah * m2) + rv[i];     // rv: gradient that bypasses the norm (residual connection), else 0
      }
      if (urow) {
        if (p.du_pre) dsilu8((const E*)p.du_pre + row * p.sdu_pre, e0, duv);
        store8((E*)p.du + row * p.sdu, e0, duv);
        if (p.y_out) store8((E*)p.y_out + row * p.sy_out, e0, yv);
      }
      store8((E*)p.da + row * p.sda, e0, dav);
    }
  }
  if (on) {
    float* prow = partial + (int64_t)blockIdx.x * 2 * D;
#pragma unroll
    for (int i = 0; i < 8; ++i) { prow[e0 + i] = gsum[i]; prow[D + e0 + i] = bsum[i]; }
  }
}

// dgamma[c] = sum over workgroups of partial[blk][0][c]; dbeta likewise from partial[blk][1][c].
// 64 columns x 16 row groups per workgroup; the 16 partial sums of a column are combined in a fixed order.
__global__ __launch_bounds__(1024) void gated_norm_colsum_kernel(int nblk, int D, const float* __restrict__ partial,
                                                                 float* __restrict__ dgamma, float* __restrict__ dbeta) {
  __shared__ float red[16][64];
  const int col = threadIdx.x & 63, rg = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + col;
  float s = 0.f;
  if (c < 2 * D)
    for (int b = rg; b < nblk; b += 16) s += partial[(int64_t)b * 2 * D + c];
  red[rg][col] = s;
  __syncthreads();
  if (rg == 0 && c < 2 * D) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) t += red[i][col];
    if (c < D) dgamma[c] = t;
    else if (dbeta) dbeta[c - D] = t;
  }
}

// waves that share a row in the backward: 1 up to 512 features, else the power of two that gives every thread one chunk
static int bwd_row_waves(int D) {
  int w = 1;
  while (w * 512 < D) w <<= 1;
  return w;                                               // 1, 2, 4, 8, 16 (D <= 8192)
}

// workgroups of the backward = rows of partial column sums
int gated_norm_bwd_blocks(int64_t T, int D) {
  const int w = bwd_row_waves(D);
  if (w == 1) {
    const int64_t need = (T + kBwdWaves - 1) / kBwdWaves;
    return (int)(need < kMaxBwdBlocks ? need : kMaxBwdBlocks);
  }
  const int64_t cap = 256 * (16 / w);                     // 16 waves per compute unit
  return (int)(T < cap ? T : cap);
}

template <typename E, int NCH>
static hipError_t fwd_one(const NormFwdArgs& p, hipStream_t stream) {
  const unsigned grid = (unsigned)((p.T + kRowsPerBlock - 1) / kRowsPerBlock);
  hipLaunchKernelGGL((gated_norm_fwd_kernel<E, NCH>), dim3(grid), dim3(64 * kRowsPerBlock), 0, stream, p);
  return hipGetLastError();
}

template <typename E, int W>
static hipError_t bwd_wide(const NormBwdArgs& p, float* partial, hipStream_t stream) {
  const int nblk = gated_norm_bwd_blocks(p.T, p.D);
  hipLaunchKernelGGL((gated_norm_bwd_wide_kernel<E, W>), dim3(nblk), dim3(64 * W), 0, stream, p, partial);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(gated_norm_colsum_kernel, dim3((2 * p.D + 63) / 64), dim3(1024), 0, stream, nblk, p.D, partial,
                     p.dgamma, p.dbeta);
  return hipGetLastError();
}

template <typename E, int NCH>
static hipError_t bwd_one(const NormBwdArgs& p, float* partial, hipStream_t stream) {
  const int nblk = gated_norm_bwd_blocks(p.T, p.D);
  auto kern = gated_norm_bwd_kernel<E, NCH>;
  const size_t smem = (size_t)2 * p.D * sizeof(float);
  if (smem > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(kern, dim3(nblk), dim3(64 * kBwdWaves), smem, stream, p, partial);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(gated_norm_colsum_kernel, dim3((2 * p.D + 63) / 64), dim3(1024), 0, stream, nblk, p.D, partial,
                     p.dgamma, p.dbeta);
  return hipGetLastError();
}

template <typename E, int NCH>
static hipError_t quant_one(const NormFwdArgs& p, void* q, int64_t sq, float* qscale, hipStream_t stream) {
  const unsigned grid = (unsigned)((p.T + kRowsPerBlock - 1) / kRowsPerBlock);
  hipLaunchKernelGGL((norm_quant_fwd_kernel<E, NCH>), dim3(grid), dim3(64 * kRowsPerBlock), 0, stream, p, (unsigned char*)q, sq, qscale);
  return hipGetLastError();
}

static int chunks_per_lane(int D) {
  const int chunks = (D / 8 + 63) / 64;
  int nch = 1;
  while (nch < chunks) nch <<= 1;
  return nch;
}

hipError_t launch_norm_fwd(const NormFwdArgs& p, hipStream_t stream) {
  const int nch = chunks_per_lane(p.D);
#define FWD_CALL(E, N) fwd_one<E, N>(p, stream)
  if (p.dtype == 0) {
    switch (nch) {
      case 1: return FWD_CALL(__bf16, 1);
      case 2: return FWD_CALL(__bf16, 2);
      case 4: return FWD_CALL(__bf16, 4);
      case 8: return FWD_CALL(__bf16, 8);
      default: return FWD_CALL(__bf16, 16);
    }
  }
  switch (nch) {
    case 1: return FWD_CALL(float, 1);
    case 2: return FWD_CALL(float, 2);
    case 4: return FWD_CALL(float, 4);
    case 8: return FWD_CALL(float, 8);
    default: return FWD_CALL(float, 16);
  }
#undef FWD_CALL
}

hipError_t launch_norm_quant_fwd(const NormFwdArgs& p, void* q, int64_t sq, float* qscale, hipStream_t stream) {
  const int nch = chunks_per_lane(p.D);
#define Q_CALL(E, N) quant_one<E, N>(p, q, sq, qscale, stream)
  if (p.dtype == 0) {
    switch (nch) {
      case 1: return Q_CALL(__bf16, 1);
      case 2: return Q_CALL(__bf16, 2);
      case 4: return Q_CALL(__bf16, 4);
      case 8: return Q_CALL(__bf16, 8);
      default: return Q_CALL(__bf16, 16);
    }
  }
  switch (nch) {
    case 1: return Q_CALL(float, 1);
    case 2: return Q_CALL(float, 2);
    case 4: return Q_CALL(float, 4);
    case 8: return Q_CALL(float, 8);
    default: return Q_CALL(float, 16);
  }
#undef Q_CALL
}

hipError_t launch_norm_bwd(const NormBwdArgs& p, float* partial, hipStream_t stream) {
  if (p.T <= 0) {                                          // no rows: the column sums are zero
    hipLaunchKernelGGL(gated_norm_colsum_kernel, dim3((2 * p.D + 63) / 64), dim3(1024), 0, stream, 0, p.D, partial, p.dgamma, p.dbeta);
    return hipGetLastError();
  }
  const int w = bwd_row_waves(p.D);
#define BWD_WIDE(E)                                        \
  switch (w) {                                             \
    case 1: return bwd_one<E, 1>(p, partial, stream);      \
    case 2: return bwd_wide<E, 2>(p, partial, stream);     \
    case 4: return bwd_wide<E, 4>(p, partial, stream);     \
    case 8: return bwd_wide<E, 8>(p, partial, stream);     \
    default: return bwd_wide<E, 16>(p, partial, stream);   \
  }
  if (p.dtype == 0) { BWD_WIDE(__bf16) }
  BWD_WIDE(float)
#undef BWD_WIDE
}

// contiguous [T, D] tensors, statistics computed: the form behind the C entry points
hipError_t launch_gated_norm_fwd(int64_t T, int D, int dtype, const void* attn, const void* u, const float* gamma,
                                 const float* beta, float eps, void* y, float* mean, float* rstd, hipStream_t stream) {
  NormFwdArgs p = {};
  p.T = T; p.D = D; p.dtype = dtype; p.a = attn; p.sa = D; p.u = u; p.su = D; p.gamma = gamma; p.beta = beta; p.eps = eps;
  p.y = y; p.sy = D; p.mean = mean; p.rstd = rstd; p.stats_in = 0;
  return launch_norm_fwd(p, stream);
}

hipError_t launch_gated_norm_bwd(int64_t T, int D, int dtype, const void* dy, const void* attn, const void* u,
                                 const float* gamma, const float* beta, float eps, void* dattn, void* du, float* dgamma,
                                 float* dbeta, float* partial, hipStream_t stream) {
  NormBwdArgs p = {};
  p.T = T; p.D = D; p.dtype = dtype; p.dy = dy; p.sdy = D; p.a = attn; p.sa = D; p.u = u; p.su = D; p.gamma = gamma;
  p.beta = beta; p.eps = eps; p.da = dattn; p.sda = D; p.du = du; p.sdu = D; p.residual = nullptr; p.sres = D;
  p.dgamma = dgamma; p.dbeta = dbeta;
  return launch_norm_bwd(p, partial, stream);
}

}  // namespace hstu
