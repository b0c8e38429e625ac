// Fused jagged HSTU attention kernels for gfx950 (MI355X): forward, dQ pass and dK/dV pass.
//
// One templated kernel covers the three passes because they share one shape.  A workgroup
// owns a block of "stationary" rows x of one (sequence, head) and streams tiles of the other
// side y through LDS, visiting only tiles that hold a visible pair (tile_ranges /
// row_tile_ranges):
//
//   pass      stationary x      streamed y     scores (y on registers, x on lanes)      outputs (transposed, [feature][x])
//   forward   queries (Q)       keys (K, V)    S^T = K Q^T                              O^T  += V^T  P^T        P = SiLU(S)
//   dQ        queries (Q, dO)   keys (K, V)    S^T = K Q^T, dP^T = V dO^T               dQ^T += K^T  dS^T
//   dK/dV     keys (K, V)       queries(Q,dO)  S   = Q K^T, dP   = dO V^T               dK^T += Q^T  dS,  dV^T += dO^T P
//
// with  S = alpha QK^T + bias,  P = S sigmoid(S),  dS = dP sigmoid(S) (1 + S (1 - sigmoid(S)))  under the mask
// (paper Eq. 3 and its derivative; the 1/N and alpha factors are applied once to the
// accumulators at the end).  There is no softmax: no running max, no row sum, no rescale.
//
// Mapping to CDNA4 matrix cores (wave64, v_mfma_f32_32x32x16_bf16): a wave owns 32 stationary
// rows, which sit on the lane axis of every product.  The stationary operands stay in
// registers as B operands for the whole block.  Scores are produced with the streamed rows
// on the accumulator's register axis, which is exactly the k-slot layout the second product
// wants for its B operand, so P / dS never travel through LDS; the streamed tile is read
// once more through the LDS transpose loads (ds_read_b64_tr_b16) to form the A operand of
// the second product.  The fp32 instantiation uses v_mfma_f32_32x32x2_f32 the same way.
#include "hstu_common.h"
#include "hstu_kernels.h"

namespace hstu {

enum { kFwd = 0, kBwdDQ = 1, kBwdDKDV = 2 };

template <typename E, int D, int MODE, int NWAVES>
struct Cfg {
  static constexpr bool kBf16 = sizeof(E) == 2;
  static constexpr int BX = 32 * NWAVES;                        // stationary rows per workgroup
  static constexpr int BN = kBf16 ? 64 : 32;                    // streamed rows per LDS tile
  static constexpr int NT = 64 * NWAVES;
  static constexpr int ROW_BYTES = D * (int)sizeof(E);
  static constexpr int STRIDE = ROW_BYTES + (kBf16 ? 80 : 16);  // LDS row stride, bytes
  static constexpr int TILE_BYTES = BN * STRIDE;
  static constexpr int CPR = ROW_BYTES / 16;                    // 16-byte chunks per row
  static constexpr int CHUNKS = BN * CPR;
  static constexpr int CPT = (CHUNKS + NT - 1) / NT;            // chunks per thread per tensor
  static constexpr int NRES = (MODE == kFwd) ? 1 : 2;           // resident operands
  static constexpr int NOUT = (MODE == kBwdDKDV) ? 2 : 1;       // output accumulators
  static constexpr int KS = kBf16 ? D / 16 : D / 2;             // k-steps of a score product
  static constexpr int OB = D / 32;                             // 32-feature output blocks
  static constexpr int SMEM_BYTES = 4 * TILE_BYTES;             // 2 stages x 2 tensors
};

template <typename E> struct ResidentFrag;
template <> struct ResidentFrag<__bf16> { typedef bf16x8 type; };
template <> struct ResidentFrag<float> { typedef float type; };

__device__ __forceinline__ float sigmoid_fast(float s) {
  const float e = __builtin_amdgcn_exp2f(s * -1.4426950408889634f);
  return __builtin_amdgcn_rcpf(1.0f + e);
}

template <typename E, int D, int MODE, int NWAVES>
__global__ __launch_bounds__(64 * NWAVES) void attn_kernel(const AttnArgs a) {
  using C = Cfg<E, D, MODE, NWAVES>;
  using RFrag = typename ResidentFrag<E>::type;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  // ---- schedule position -> work item.  Workgroups are dealt to the 8 dies round-robin by
  // workgroup id; groups of kXcdGroup consecutive list entries are kept on one die.
  const int wg = blockIdx.x;
  const int xcd = wg % kNumXcd, slot = wg / kNumXcd;
  const int pos = ((slot / kXcdGroup) * kNumXcd + xcd) * kXcdGroup + slot % kXcdGroup;
  if (pos >= a.header->count) return;
  const WorkItem item = a.items[pos];
  const int b = item.b, xb = item.rb_h >> 8, h = item.rb_h & 255;
  const int seq0 = a.offsets[b];
  const int L = a.offsets[b + 1] - seq0;
  const SeqGeom g = {L, L - (a.num_targets ? a.num_targets[b] : 0), a.K1, a.K2};

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int hf = lane >> 5, l32 = lane & 31, grp16 = lane >> 4, i16 = lane & 15;
  const int x0 = xb * C::BX;
  const int xw0 = x0 + wave * 32;
  const int x = xw0 + l32;
  const bool x_ok = x < L;

  // ---- operand roles
  const E *R1, *R2 = nullptr, *Y1, *Y2;
  int64_t sr1, sr2 = 0, sy1, sy2;
  if (MODE == kFwd) {
    R1 = (const E*)a.q; sr1 = a.sq; Y1 = (const E*)a.k; sy1 = a.sk; Y2 = (const E*)a.v; sy2 = a.sv;
  } else if (MODE == kBwdDQ) {
    R1 = (const E*)a.q; sr1 = a.sq; R2 = (const E*)a.dout; sr2 = a.so;
    Y1 = (const E*)a.k; sy1 = a.sk; Y2 = (const E*)a.v; sy2 = a.sv;
  } else {
    R1 = (const E*)a.k; sr1 = a.sk; R2 = (const E*)a.v; sr2 = a.sv;
    Y1 = (const E*)a.q; sy1 = a.sq; Y2 = (const E*)a.dout; sy2 = a.so;
  }
  const int64_t hoff = (int64_t)h * D;
  R1 += seq0 * sr1 + hoff; Y1 += seq0 * sy1 + hoff; Y2 += seq0 * sy2 + hoff;
  if (C::NRES == 2) R2 += seq0 * sr2 + hoff;

  // ---- resident operands (B operands: lane = row x, registers = 8 (bf16) or 1 (fp32) features per k-step)
  RFrag res[C::NRES][C::KS];
#pragma unroll
  for (int i = 0; i < C::NRES; ++i) {
    const E* rp = (i == 0 ? R1 + (int64_t)x * sr1 : R2 + (int64_t)x * sr2);
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) {
      if constexpr (C::kBf16) {
        u32x4 raw = {0u, 0u, 0u, 0u};
        if (x_ok) raw = *(const u32x4*)(rp + ks * 16 + hf * 8);
        res[i][ks] = __builtin_bit_cast(RFrag, raw);
      } else {
        res[i][ks] = x_ok ? rp[2 * ks + hf] : 0.f;
      }
    }
  }

  f32x16 out[C::NOUT][C::OB];
#pragma unroll
  for (int o = 0; o < C::NOUT; ++o)
#pragma unroll
    for (int ob = 0; ob < C::OB; ++ob)
#pragma unroll
      for (int r = 0; r < 16; ++r) out[o][ob][r] = 0.f;

  const int xlast = min(x0 + C::BX, L) - 1;
  const TileRanges tr = (MODE == kBwdDKDV) ? row_tile_ranges(g, x0, xlast, C::BN) : tile_ranges(g, x0, xlast, C::BN);
  const int ntiles = tr.count();
  const float* bias_h = a.bias ? a.bias + (int64_t)h * a.bias_stride : nullptr;
  const bool unit_alpha = a.alpha == 1.0f;

  // ---- global -> register -> LDS staging of the streamed tiles
  u32x4 pre1[C::CPT], pre2[C::CPT];
  auto gload = [&](int yt) {
#pragma unroll
    for (int c = 0; c < C::CPT; ++c) {
      const int idx = tid + c * C::NT;
      const int row = idx / C::CPR, col = idx % C::CPR;
      const int y = yt * C::BN + row;
      pre1[c] = (u32x4){0u, 0u, 0u, 0u};
      pre2[c] = (u32x4){0u, 0u, 0u, 0u};
      if (idx < C::CHUNKS && y < L) {                                    // rows past the sequence end read as zero
        pre1[c] = *(const u32x4*)((const unsigned char*)(Y1 + (int64_t)y * sy1) + col * 16);
        pre2[c] = *(const u32x4*)((const unsigned char*)(Y2 + (int64_t)y * sy2) + col * 16);
      }
    }
  };
  auto lstore = [&](int stage) {
#pragma unroll
    for (int c = 0; c < C::CPT; ++c) {
      const int idx = tid + c * C::NT;
      const int row = idx / C::CPR, col = idx % C::CPR;
      if (idx < C::CHUNKS) {
        *(u32x4*)(smem + (stage * 2 + 0) * C::TILE_BYTES + row * C::STRIDE + col * 16) = pre1[c];
        *(u32x4*)(smem + (stage * 2 + 1) * C::TILE_BYTES + row * C::STRIDE + col * 16) = pre2[c];
      }
    }
  };

  if (ntiles > 0) {
    gload(tr.at(0));
    lstore(0);
  }
  __syncthreads();

  for (int t = 0; t < ntiles; ++t) {
    const int yt = tr.at(t);
    const int stage = t & 1;
    if (t + 1 < ntiles) gload(tr.at(t + 1));
    const unsigned char* y1s = smem + (stage * 2 + 0) * C::TILE_BYTES;
    const unsigned char* y2s = smem + (stage * 2 + 1) * C::TILE_BYTES;

#pragma unroll
    for (int sb = 0; sb < C::BN / 32; ++sb) {
      const int ys0 = yt * C::BN + sb * 32;
      int kind = (MODE == kBwdDKDV) ? classify_tile(g, ys0, ys0 + 31, xw0, xw0 + 31)
                                    : classify_tile(g, xw0, xw0 + 31, ys0, ys0 + 31);
      if (xw0 >= L) kind = kTileEmpty;
      if (kind == kTileEmpty) continue;                                  // wave-uniform
      if (kind == kTileFull && !unit_alpha) kind = kTilePartial;         // general alpha: generic path

      // ---- scores
      f32x16 sc1, sc2;
#pragma unroll
      for (int r = 0; r < 16; ++r) { sc1[r] = 0.f; sc2[r] = 0.f; }
      if (kind == kTileFull && bias_h) {
        // every pair is visible and i - j >= 0: seed the accumulator with the bias
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int y = ys0 + 8 * (r >> 2) + 4 * hf + (r & 3);
          sc1[r] = bias_h[(MODE == kBwdDKDV) ? y - x : x - y];
        }
      }
      const unsigned char* y1row = y1s + (sb * 32 + l32) * C::STRIDE;
      const unsigned char* y2row = y2s + (sb * 32 + l32) * C::STRIDE;
#pragma unroll
      for (int ks = 0; ks < C::KS; ++ks) {
        if constexpr (C::kBf16) {
          const bf16x8 af = *(const bf16x8*)(y1row + (ks * 16 + hf * 8) * 2);
          sc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, res[0][ks], sc1, 0, 0, 0);
        } else {
          const float af = *(const float*)(y1row + (2 * ks + hf) * 4);
          sc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(af, res[0][ks], sc1, 0, 0, 0);
        }
      }
      if constexpr (MODE != kFwd) {
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
          if constexpr (C::kBf16) {
            const bf16x8 af = *(const bf16x8*)(y2row + (ks * 16 + hf * 8) * 2);
            sc2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, res[1][ks], sc2, 0, 0, 0);
          } else {
            const float af = *(const float*)(y2row + (2 * ks + hf) * 4);
            sc2 = __builtin_amdgcn_mfma_f32_32x32x2f32(af, res[1][ks], sc2, 0, 0, 0);
          }
        }
      }

      // ---- pointwise: SiLU (forward) or its derivative times dP (backward), mask in registers
      float c1[16], c2[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float s = sc1[r];
        bool vis = true;
        if (kind == kTilePartial) {
          const int y = ys0 + 8 * (r >> 2) + 4 * hf + (r & 3);
          int delta;
          vis = (MODE == kBwdDKDV) ? visible(g, y, x, delta) : visible(g, x, y, delta);
          float bv = 0.f;
          if (bias_h && vis) bv = bias_h[delta];
          s = fmaf(s, a.alpha, bv);
        }
        const float sig = sigmoid_fast(s);
        const float p = s * sig;
        if (MODE == kFwd) {
          c1[r] = vis ? p : 0.f;
        } else {
          const float ds = sc2[r] * sig * (1.0f + s * (1.0f - sig));
          c1[r] = vis ? ds : 0.f;
          c2[r] = vis ? p : 0.f;
        }
      }

      // ---- second products: out^T[feature][x] += Y^T[feature][y] * coeff[y][x]
      if constexpr (C::kBf16) {
        uint32_t pk1[8], pk2[8];
#pragma unroll
        for (int m = 0; m < 8; ++m) {
          pk1[m] = pack_bf16x2(c1[2 * m], c1[2 * m + 1]);
          if (MODE == kBwdDKDV) pk2[m] = pack_bf16x2(c2[2 * m], c2[2 * m + 1]);
        }
#pragma unroll
        for (int ks2 = 0; ks2 < 2; ++ks2) {
          // k-slots of this lane: streamed rows ks2*16 + 4*hf + {0..3} and + 8 + {0..3}
          const bf16x8 b1 = __builtin_bit_cast(bf16x8, (u32x4){pk1[4 * ks2], pk1[4 * ks2 + 1], pk1[4 * ks2 + 2], pk1[4 * ks2 + 3]});
          bf16x8 b2 = b1;
          if (MODE == kBwdDKDV)
            b2 = __builtin_bit_cast(bf16x8, (u32x4){pk2[4 * ks2], pk2[4 * ks2 + 1], pk2[4 * ks2 + 2], pk2[4 * ks2 + 3]});
          // transpose load: within a group of 16 lanes, lane 4r+c supplies the address of 4 features
          // (4c..4c+3) of streamed row r and lane i receives feature i of rows 0..3
          const int trow = sb * 32 + ks2 * 16 + 4 * hf + (i16 >> 2);
          const int tcol = 16 * (grp16 & 1) + 4 * (i16 & 3);
#pragma unroll
          for (int ob = 0; ob < C::OB; ++ob) {
            const int off = trow * C::STRIDE + (ob * 32 + tcol) * 2;
            typedef __attribute__((address_space(3))) short4v* lds_s4;
            const unsigned char* src0 = (MODE == kFwd) ? y2s : y1s;      // V (forward), K (dQ), Q (dK)
            const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(src0 + off));
            const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(src0 + off + 8 * C::STRIDE));
            const bf16x8 af = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
            out[0][ob] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, b1, out[0][ob], 0, 0, 0);
            if constexpr (MODE == kBwdDKDV) {                            // dV^T += dO^T P
              const short4v lo2 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(y2s + off));
              const short4v hi2 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(y2s + off + 8 * C::STRIDE));
              const bf16x8 af2 = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo2, hi2, 0, 1, 2, 3, 4, 5, 6, 7));
              out[1][ob] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af2, b2, out[1][ob], 0, 0, 0);
            }
          }
        }
      } else {
#pragma unroll
        for (int ks2 = 0; ks2 < 16; ++ks2) {
          // k-step ks2 contracts the two streamed rows 8*(ks2/4) + ks2%4 (+4 for the upper half-wave)
          const int trow = sb * 32 + 8 * (ks2 >> 2) + 4 * hf + (ks2 & 3);
#pragma unroll
          for (int ob = 0; ob < C::OB; ++ob) {
            const int off = trow * C::STRIDE + (ob * 32 + l32) * 4;
            const unsigned char* src0 = (MODE == kFwd) ? y2s : y1s;
            const float af = *(const float*)(src0 + off);
            out[0][ob] = __builtin_amdgcn_mfma_f32_32x32x2f32(af, c1[ks2], out[0][ob], 0, 0, 0);
            if constexpr (MODE == kBwdDKDV) {
              const float af2 = *(const float*)(y2s + off);
              out[1][ob] = __builtin_amdgcn_mfma_f32_32x32x2f32(af2, c2[ks2], out[1][ob], 0, 0, 0);
            }
          }
        }
      }
    }

    if (t + 1 < ntiles) lstore(stage ^ 1);
    __syncthreads();
  }

  // ---- epilogue: scale once, convert, store.  Lane x holds features ob*32 + 8*(r/4) + 4*hf + r%4.
  if (!x_ok) return;
#pragma unroll
  for (int o = 0; o < C::NOUT; ++o) {
    E* dst;
    int64_t sd;
    float scale;
    if (MODE == kFwd) { dst = (E*)a.out; sd = a.so; scale = a.inv_n; }
    else if (MODE == kBwdDQ) { dst = (E*)a.dq; sd = a.sq; scale = a.inv_n * a.alpha; }
    else if (o == 0) { dst = (E*)a.dk; sd = a.sk; scale = a.inv_n * a.alpha; }
    else { dst = (E*)a.dv; sd = a.sv; scale = a.inv_n; }
    dst += (int64_t)(seq0 + x) * sd + hoff;
#pragma unroll
    for (int ob = 0; ob < C::OB; ++ob)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int f = ob * 32 + 8 * q4 + 4 * hf;
        const float v0 = out[o][ob][4 * q4 + 0] * scale, v1 = out[o][ob][4 * q4 + 1] * scale;
        const float v2 = out[o][ob][4 * q4 + 2] * scale, v3 = out[o][ob][4 * q4 + 3] * scale;
        if constexpr (C::kBf16) {
          *(u32x2*)(dst + f) = (u32x2){pack_bf16x2(v0, v1), pack_bf16x2(v2, v3)};
        } else {
          *(f32x4*)(dst + f) = (f32x4){v0, v1, v2, v3};
        }
      }
  }
}

// ------------------------------------------------------------------------------------------------
template <typename E, int D, int MODE, int NWAVES>
static hipError_t launch_one(const AttnArgs& a, hipStream_t stream) {
  using C = Cfg<E, D, MODE, NWAVES>;
  auto kern = attn_kernel<E, D, MODE, NWAVES>;
  static bool attr_set = false;                                          // per instantiation
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, C::SMEM_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int per = kNumXcd * kXcdGroup;
  const int grid = (a.max_items + per - 1) / per * per;
  if (grid == 0) return hipSuccess;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(C::NT), C::SMEM_BYTES, stream, a);
  return hipGetLastError();
}

template <int MODE, int NW_BF16, int NW_FP32>
static hipError_t dispatch(const AttnArgs& a, int dtype, hipStream_t stream) {
  if (dtype == 0) {
    switch (a.D) {
      case 32: return launch_one<__bf16, 32, MODE, NW_BF16>(a, stream);
      case 64: return launch_one<__bf16, 64, MODE, NW_BF16>(a, stream);
      case 128: return launch_one<__bf16, 128, MODE, NW_BF16>(a, stream);
    }
  } else {
    switch (a.D) {
      case 32: return launch_one<float, 32, MODE, NW_FP32>(a, stream);
      case 64: return launch_one<float, 64, MODE, NW_FP32>(a, stream);
      case 128: return launch_one<float, 128, MODE, NW_FP32>(a, stream);
    }
  }
  return hipErrorInvalidValue;
}

constexpr int kFwdWavesBf16 = 8, kFwdWavesFp32 = 4;
constexpr int kDqWavesBf16 = 8, kDqWavesFp32 = 4;
constexpr int kDkvWavesBf16 = 4, kDkvWavesFp32 = 4;

int fwd_block_rows(int dtype, int) { return 32 * (dtype == 0 ? kFwdWavesBf16 : kFwdWavesFp32); }
int dq_block_rows(int dtype, int) { return 32 * (dtype == 0 ? kDqWavesBf16 : kDqWavesFp32); }
int dkv_block_rows(int dtype, int) { return 32 * (dtype == 0 ? kDkvWavesBf16 : kDkvWavesFp32); }
int stream_tile_rows(int dtype, int) { return dtype == 0 ? 64 : 32; }

hipError_t launch_attn_fwd(const AttnArgs& a, int dtype, hipStream_t stream) {
  return dispatch<kFwd, kFwdWavesBf16, kFwdWavesFp32>(a, dtype, stream);
}
hipError_t launch_attn_bwd_dq(const AttnArgs& a, int dtype, hipStream_t stream) {
  return dispatch<kBwdDQ, kDqWavesBf16, kDqWavesFp32>(a, dtype, stream);
}
hipError_t launch_attn_bwd_dkdv(const AttnArgs& a, int dtype, hipStream_t stream) {
  return dispatch<kBwdDKDV, kDkvWavesBf16, kDkvWavesFp32>(a, dtype, stream);
}

}  // namespace hstu
