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
// (paper Eq. 3 and its derivative; alpha rides on the stationary operand of the score product, and the
// 1/N factor, with the alpha that dQ and dK owe, is applied once to the accumulators at the end).  There is no softmax: no running max, no row sum, no rescale.
//
// Mapping to CDNA4 matrix cores (wave64, v_mfma_f32_32x32x16_bf16): a wave owns 32 stationary
// rows, which sit on the lane axis of every product.  The stationary operands stay in
// registers as B operands for the whole block.  Scores are produced with the streamed rows
// on the accumulator's register axis, which is exactly the k-slot layout the second product
// wants for its B operand, so P / dS never travel through LDS; the streamed tile is read
// once more through the LDS transpose loads (ds_read_b64_tr_b16) to form the A operand of
// the second product.  The fp32 instantiation uses v_mfma_f32_32x32x2_f32 the same way.
#include <type_traits>

#include "hstu_common.h"
#include "hstu_kernels.h"

#ifndef HSTU_DKDV_PF
#define HSTU_DKDV_PF 2
#endif

// Measurement builds only: with HSTU_BWD_TIMELINE defined non-zero, the first lane of every workgroup of the two backward
// passes records the 100 MHz wall clock at its start, after the prologue's barrier, after the tile loop and after its
// stores; hstu_debug_bwd_timeline() copies the records of the last launch out (5 words per work item, in list order).
#ifndef HSTU_BWD_TIMELINE
#define HSTU_BWD_TIMELINE 0
#endif

namespace hstu {

enum { kFwd = 0, kBwdDQ = 1, kBwdDKDV = 2 };

#if HSTU_BWD_TIMELINE
constexpr int kTimelineItems = 16384;
__device__ uint64_t g_timeline_bwd[2][5 * kTimelineItems];
#define HSTU_TLB(k) do { if (MODE != kFwd && threadIdx.x == 0 && pos < kTimelineItems) g_timeline_bwd[MODE == kBwdDQ ? 0 : 1][5 * pos + (k)] = wall_clock64(); } while (0)
#else
#define HSTU_TLB(k) do { } while (0)
#endif

template <typename E, int D, int MODE, int NWAVES>
struct Cfg {
  static constexpr bool kBf16 = sizeof(E) == 2;
  static constexpr int BX = 32 * NWAVES;                        // stationary rows per workgroup
  // dK/dV pass with 128 features: the accumulators alone take 128 registers per lane, so the V rows of the
  // workgroup's keys stay in LDS (not in registers) and the streamed tiles are 32 rows; that fits 256
  // registers and half the LDS, i.e. two workgroups per compute unit like the other passes.
  static constexpr bool kStatLds = kBf16 && D == 128 && MODE == kBwdDKDV;
  // Forward with 128 features: 32-row tiles need 161 registers and 39 KB of LDS, so three workgroups share a compute
  // unit (three independent instruction streams per SIMD); measured 5 % faster than two with 64-row tiles and an
  // in-wave software pipeline.
  static constexpr bool kThreePerCu = kBf16 && D == 128 && MODE == kFwd && NWAVES == 4;
  static constexpr int BN = kBf16 ? ((kStatLds || kThreePerCu) ? 32 : 64) : 32;  // streamed rows per LDS tile
  static constexpr int NT = 64 * NWAVES;
  static constexpr int ROW_BYTES = D * (int)sizeof(E);
  // LDS tiles are read two ways: 16-byte reads with one streamed row per lane (score products)
  // and transpose reads that touch 4 consecutive rows x 64 bytes per 32 lanes (second products).
  //   tensor 0 (Y1): K in the forward (rows only), K in the dQ pass and Q in the dK/dV pass (both ways)
  //   tensor 1 (Y2): V in the forward (transposed only), V in the dQ pass (rows only), dO in dK/dV (both)
  // 256-byte bf16 rows are unpadded and store the 16-byte chunks of row r at chunk ^ swz(r),
  // swz(r) = 4*(r%4) + (r/4)%4: 16 consecutive rows then map one logical chunk to 16 different bank
  // groups, and 4 consecutive rows map 4 consecutive chunks to 16 different ones, so both ways of
  // reading are conflict-free.  Such tiles travel from global memory straight into LDS (no register
  // staging): a wave-level 16-byte load places its 64 lanes in 1 KB of consecutive LDS, and each lane
  // applies the swizzle to its global address instead.  Narrower rows and fp32 are staged through
  // registers into padded rows: the padding that makes the way(s) a tile is read conflict-free
  // (16 bytes for row-per-lane reads, 64 for transpose reads, 80 for both).
  static constexpr bool kBoth0 = MODE != kFwd, kBoth1 = MODE == kBwdDKDV;
  static constexpr bool kDma = kBf16 && D == 128;
  static constexpr bool kSwz0 = kDma, kSwz1 = kDma;
  // 4-wave bf16 workgroups run two per compute unit (two independent instruction streams per SIMD):
  // 256 registers per lane and half of the 160 KB of LDS each.
  static constexpr bool kTwoPerCu = kBf16 && NWAVES == 4 && (MODE != kBwdDKDV || kStatLds);
  static constexpr int kWgPerCu = kThreePerCu ? 3 : (kTwoPerCu ? 2 : 1);
  static constexpr int PAD0 = !kBf16 ? 16 : (kSwz0 ? 0 : (kBoth0 ? 80 : 16));
  static constexpr int PAD1 = !kBf16 ? 16 : (kSwz1 ? 0 : (kBoth1 ? 80 : (MODE == kFwd ? 64 : 16)));
  static constexpr int STRIDE0 = ROW_BYTES + PAD0, STRIDE1 = ROW_BYTES + PAD1;   // LDS row strides, bytes
  static constexpr int TILE0 = BN * STRIDE0, TILE1 = BN * STRIDE1;
  static constexpr int STAGE_BYTES = TILE0 + TILE1;
  static constexpr int CPR = ROW_BYTES / 16;                    // 16-byte chunks per row
  static constexpr int CHUNKS = BN * CPR;
  static constexpr int CPT = (CHUNKS + NT - 1) / NT;            // chunks per thread per tensor
  static constexpr int NRES = (MODE == kFwd) ? 1 : 2;           // stationary operands
  static constexpr int NREG = kStatLds ? 1 : NRES;              // ... of which in registers
  static constexpr int NOUT = (MODE == kBwdDKDV) ? 2 : 1;       // output accumulators
  static constexpr int KS = kBf16 ? D / 16 : D / 2;             // k-steps of a score product
  static constexpr int OB = D / 32;                             // 32-feature output blocks
  // Relative-bias strip of one (block, tile): the bias depends on i - j only, so a tile needs
  // BX + BN - 1 consecutive table entries.  Four copies shifted by 0..3 entries let every lane
  // fetch 4 consecutive entries with one aligned 16-byte LDS read.
  // Copy length = 16 (mod 64) entries keeps the 16 reads of a quarter-wave on 16 different bank groups.
  static constexpr int SLEN = (BX + BN + 4 - 16 + 63) / 64 * 64 + 16;   // entries per copy
  static constexpr int STRIP_BYTES = 4 * SLEN * 4;
  static constexpr int STRIP_BASE = 2 * STAGE_BYTES;
  static constexpr int STAT_BASE = 2 * STAGE_BYTES + 2 * STRIP_BYTES;
  static constexpr int STAT_BYTES = kStatLds ? BX * ROW_BYTES : 0;      // stationary operand 1, same swizzle as the tiles
  static constexpr int SMEM_BYTES = STAT_BASE + STAT_BYTES;             // 2 stages x (2 tensors + strip) [+ stationary rows]
  // bias-gradient variant of the dQ pass: two (double-buffered) strips of per-distance sums behind everything else
  static constexpr int DACC_LEN = (BX + BN - 1 + 63) / 64 * 64;
  static constexpr int DACC_BASE = SMEM_BYTES;
  static constexpr int DACC_COPIES = NWAVES;                     // one strip per wave: plain read-add-write, no LDS atomics
  static constexpr int DACC_BYTES = 2 * DACC_COPIES * DACC_LEN * 4;
};

template <typename E> struct ResidentFrag;
template <> struct ResidentFrag<__bf16> { typedef bf16x8 type; };
template <> struct ResidentFrag<float> { typedef float type; };

// byte offset of logical 16-byte chunk `chunk` of tile row `row`
template <typename C, int TENSOR>
__device__ __forceinline__ int lds_off(int row, int chunk) {
  constexpr int stride = TENSOR == 0 ? C::STRIDE0 : C::STRIDE1;
  if constexpr (TENSOR == 0 ? C::kSwz0 : C::kSwz1) return row * stride + ((chunk ^ (4 * (row & 3) + ((row >> 2) & 3))) << 4);
  else return row * stride + (chunk << 4);
}

// Scores are kept in units of ln 2 inside the kernels (t = s * log2 e): the stationary operand of the
// score product and the expanded bias table are scaled by log2 e once, so the sigmoid needs no multiply
// in front of its exp2, and the ln 2 that P = s * sigmoid(s) = ln2 * t * sigmoid owes is folded into the
// output scale (forward, dV) or into the (1 - sigmoid) term (dS).
constexpr float kLog2e = 1.4426950408889634f, kLn2 = 0.6931471805599453f;
__device__ __forceinline__ float sigmoid_l2(float t) {           // sigmoid(t * ln 2)
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-t));
}
// dS / dP = sigmoid (1 + s (1 - sigmoid)) = sigmoid + (t sigmoid) * ln2 (1 - sigmoid)
__device__ __forceinline__ float dsilu_l2(float tp, float sig) { return fmaf(tp, fmaf(-kLn2, sig, kLn2), sig); }

// One register of the diagonal sum of a 32 x 32 score-gradient block (lane = query 16*a + b of the block, register R
// = key yo = 8*(R/4) + R%4 (+4 for the upper half-wave)).  Rotating register R by rho = yo % 16 lanes inside its
// 16-lane row puts every value next to the others of its diagonal: at lane b' it belongs to strip offset
// 16*j - b' with j = yo/16 + (1 if it came around the row end), so three running sums per lane collect all 16.
template <int R>
__device__ __forceinline__ void diag_step(const float* vals, int bq, float& x0, float& x1, float& x2) {
  constexpr int q = R >> 2, rho = 8 * (q & 1) + (R & 3);
  float rv = vals[R];
  if constexpr (rho != 0)                                                // row_ror:(16 - rho): lane b' reads lane (b' + rho) % 16
    rv = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, rv), 0x120 + (16 - rho), 0xF, 0xF, false));
  const bool wrapped = bq >= 16 - rho;
  const float lo = wrapped ? 0.f : rv, hi = wrapped ? rv : 0.f;
  if constexpr ((q >> 1) == 0) { x0 += lo; x1 += hi; } else { x1 += lo; x2 += hi; }
}
template <int... R>
__device__ __forceinline__ void diag_all(std::integer_sequence<int, R...>, const float* vals, int bq, float& x0, float& x1, float& x2) {
  (diag_step<R>(vals, bq, x0, x1, x2), ...);
}

// DBIAS (dQ pass only): also sum dS along the diagonals of every tile (pairs of equal distance i - j) into
// a.dbias_dist[h, distance]; dbias_reduce_kernel folds distances into buckets afterwards.
// CAND (batches with candidate rows): the fast paths also cover candidate rows against history keys.  A candidate row
// stands at position n for the mask and for the bias, so full and mask-edge tiles of such rows work like those of history
// rows once the bias strip is addressed with the row's effective position (query-stationary passes) or anchored at n
// for a tile of candidate queries (dK/dV pass).  Batches without candidates run the instantiation without it (a few
// scalar instructions per tile less).
// d/dt [t sigmoid(t)]
__device__ __forceinline__ float dsilu(float t) {
  const float sg = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-kLog2e * t));
  return sg * (1.0f + t * (1.0f - sg));
}

template <typename E, int D, int MODE, int NWAVES, bool DBIAS = false, bool CAND = false>
__global__ __launch_bounds__(64 * NWAVES, (Cfg<E, D, MODE, NWAVES>::kWgPerCu)) void attn_kernel(const AttnArgs a) {
  static_assert(!DBIAS || MODE == kBwdDQ, "the bias gradient rides with the dQ pass");
  constexpr bool CANDQ = CAND && MODE != kBwdDKDV, CANDK = CAND && MODE == kBwdDKDV;
  using C = Cfg<E, D, MODE, NWAVES>;
  using RFrag = typename ResidentFrag<E>::type;
  // 256-byte alignment: the fragment reads below form LDS addresses as integers, base included, and XOR the swizzle in
  extern __shared__ __attribute__((aligned(256))) unsigned char smem[];

  // ---- schedule position -> work item.  Workgroups are dealt to the 8 dies round-robin by
  // workgroup id; runs of kXcdGroup consecutive list entries (sorted blocks of one head) are kept on one die.
  const int wg = blockIdx.x;
  const int xcd = wg % kNumXcd, slot = wg / kNumXcd;
  const int pos = ((slot / kXcdGroup) * kNumXcd + xcd) * kXcdGroup + slot % kXcdGroup;
  // (the list's length and the entry are fetched together; an entry beyond the length is read, inside the list's
  // capacity, and dropped)
  const int count = a.header->count;
  const WorkItem item = a.items[min(pos, a.max_items - 1)];
  if (pos >= count) return;
  HSTU_TLB(0);
  const int xb = item.rb_h >> 8, h = item.rb_h & 255;
  const int t_begin = item.t0;
  const int seq0 = item.seq0;
  const int L = item.len;
  const SeqGeom g = {L, item.hist, a.K1, a.K2};

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);           // scalar: per-wave decisions stay on the SALU
  const int hf = lane >> 5, l32 = lane & 31, grp16 = lane >> 4, i16 = lane & 15;
  const int x0 = xb * C::BX;
  const int xw0 = x0 + wave * 32;
  const int x = xw0 + l32;
  const bool x_ok = x < L;
  // forward with a query tail: rows before q0 are neither computed nor written
  const int q0 = (MODE == kFwd && a.query_tail > 0) ? max(g.n - a.query_tail, 0) : 0;

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
  // The operand of the score product carries alpha log2 e: the accumulator then holds (alpha q.k) log2 e, to which the
  // bias (already in those units) is added or with which it is seeded, for any alpha.
  const float score_scale = kLog2e * a.alpha;
  RFrag res[C::NRES][C::KS];
#pragma unroll
  for (int i = 0; i < C::NREG; ++i) {
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
  // (first use further down, after the first tile's loads are issued: the two round trips to memory overlap)
  auto finish_resident = [&]() {
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) {                                 // operand of the score product
      if constexpr (C::kBf16) {
        u32x4 raw = __builtin_bit_cast(u32x4, res[0][ks]);
#pragma unroll
        for (int w = 0; w < 4; ++w)
          raw[w] = pack_bf16x2(__builtin_bit_cast(float, raw[w] << 16) * score_scale,
                               __builtin_bit_cast(float, raw[w] & 0xFFFF0000u) * score_scale);
        res[0][ks] = __builtin_bit_cast(RFrag, raw);
      } else {
        res[0][ks] *= score_scale;
      }
    }
    // The resident operands must have landed before the tile loop: inside it the only global loads
    // in flight are the next tile's, and nothing may force a wait on those before they are needed.
#pragma unroll
    for (int i = 0; i < C::NREG; ++i)
#pragma unroll
      for (int ks = 0; ks < C::KS; ++ks) asm volatile("" : "+v"(res[i][ks]));
  };

  f32x16 out[C::NOUT][C::OB];
#pragma unroll
  for (int o = 0; o < C::NOUT; ++o)
#pragma unroll
    for (int ob = 0; ob < C::OB; ++ob)
#pragma unroll
      for (int r = 0; r < 16; ++r) out[o][ob][r] = 0.f;

  const int xlast = min(x0 + C::BX, L) - 1;
  const TileRanges tr = (MODE == kBwdDKDV) ? row_tile_ranges(g, x0, xlast, C::BN) : tile_ranges(g, x0, xlast, C::BN);
  const int ntiles = min(tr.count(), item.t1);             // this item's share of the block's tile list is [t_begin, ntiles)
  const float* bias_h = a.bias ? a.bias + (int64_t)h * a.bias_stride : nullptr;
  // this lane's start inside the bias strip: copy c = s0 mod 4 makes its 4-entry reads 16-byte aligned
  // Query-stationary passes: a candidate row (x >= n) stands at position n for the mask and for the bias, so the strip is
  // addressed with the row's effective position px, and a block made of candidates only puts the strip's origin at n.
  const int x0v = CANDQ ? min(x0, g.n) : x0;
  const int strip_s0 = C::BX - 1 - ((CANDQ ? min(x, g.n) : x) - x0v) + 4 * hf;
  const int strip_lane = (strip_s0 & 3) * C::SLEN + (strip_s0 & ~3);

  // ---- staging of the streamed tiles: global -> LDS directly, or through registers
  u32x4 pre1[C::CPT], pre2[C::CPT];
  const uint32_t rowb1 = (uint32_t)(sy1 * (int64_t)sizeof(E)), rowb2 = (uint32_t)(sy2 * (int64_t)sizeof(E));
  // Tile loads are raw buffer loads: the descriptor (uniform, built on the scalar unit) carries the
  // address of the piece's first row and the bytes left in the sequence from there, the lane supplies
  // a loop-invariant 32-bit offset.  Rows past the sequence end are out of range and read as zero
  // (every pair that involves them is masked anyway), and no vector arithmetic is needed per tile.
  // The host checks that a sequence spans less than 4 GiB in every tensor.
  static_assert(C::NT % C::CPR == 0 || C::CPT == 1, "a piece must cover whole tile rows");
  static_assert(!C::kDma || (NWAVES % 4 == 0 && C::CPT * NWAVES * 4 == C::BN), "direct-to-LDS pieces are 4-row groups");
  constexpr int PIECE_ROWS = C::NT / C::CPR;
  // register-staged tiles: lane -> chunk tid of the piece.  Direct-to-LDS tiles: a wave fills the 4-row
  // group rg = NWAVES * c + wave of the tile with piece c; lane -> row lane/16 of the group and LDS slot
  // lane%16, which holds logical chunk slot ^ swz(row), swz(row) = 4 * (row%4) + (row/4)%4 = 4 * (lane/16) + wave%4.
  const int dma_chunk = (lane & 15) ^ (4 * (lane >> 4) + (wave & 3));
  uint32_t voff1 = C::kDma ? __umul24((uint32_t)(lane >> 4), rowb1) + (uint32_t)(dma_chunk * 16)
                           : __umul24((uint32_t)(tid / C::CPR), rowb1) + (uint32_t)(tid % C::CPR * 16);
  uint32_t voff2 = C::kDma ? __umul24((uint32_t)(lane >> 4), rowb2) + (uint32_t)(dma_chunk * 16)
                           : __umul24((uint32_t)(tid / C::CPR), rowb2) + (uint32_t)(tid % C::CPR * 16);
  asm volatile("" : "+v"(voff1), "+v"(voff2));
  // strip[s] = bias(distance) for s = (y - tile start) + (BX - 1 - (x - x0)); the distance grows with
  // x - y in the query-stationary passes and with y - x in the key-stationary pass.
  // The bias strip goes to LDS the same direct way, 4 bytes per lane: the 4 * SLEN entries of a stage are 64-entry runs,
  // run i = NWAVES * j + wave belongs to this wave.  Entry e = 64 * i + lane is position m = e % SLEN of copy
  // c = e / SLEN and holds strip[m + c]; 4 * (m + c) is a loop invariant of the lane.
  constexpr int STRIP_RUNS = 4 * C::SLEN / 64, STRIP_J = (STRIP_RUNS + NWAVES - 1) / NWAVES;
  static_assert(4 * C::SLEN % 64 == 0, "strip stages are whole 64-entry runs");
  uint32_t strip_s4[STRIP_J];
#pragma unroll
  for (int j = 0; j < STRIP_J; ++j) {
    const int e = 64 * (NWAVES * j + wave) + lane;
    strip_s4[j] = 4u * (uint32_t)(e % C::SLEN + e / C::SLEN);
    asm volatile("" : "+v"(strip_s4[j]));
  }
  // raw buffer descriptor: 48-bit base, stride 0, bytes in range, 32-bit untyped data format
  auto make_rsrc = [&](uint64_t addr, uint32_t bytes) -> i32x4 {
    return (i32x4){(int)(uint32_t)addr, (int)(uint32_t)(addr >> 32), (int)bytes, 0x00020000};
  };
  auto tile_rsrc = [&](const E* base, uint32_t rowb, int first_row) -> i32x4 {
    return make_rsrc((uint64_t)(uintptr_t)base + (uint64_t)(uint32_t)first_row * rowb, (uint32_t)max(L - first_row, 0) * rowb);
  };
  // One 16-byte-per-lane load straight into LDS: lane l lands at LDS byte dst + 16 * l (dst uniform, passed
  // in M0).  Written as one opaque instruction group so that the compiler does not order the LDS reads of
  // the tile being consumed behind the arrival of the tile being fetched; lstore() below waits for the
  // wave's own pieces and the workgroup barrier after it publishes them.
  auto dma16 = [&](i32x4 rs, uint32_t voff, uint32_t dst) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(dst), "v"(voff), "s"(rs) : "memory", "m0");
  };
  auto dma4 = [&](i32x4 rs, uint32_t voff, uint32_t dst) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds"
                 :: "s"(dst), "v"(voff), "s"(rs) : "memory", "m0");
  };
  auto load16 = [&](uint64_t addr, uint32_t bytes, uint32_t voff) -> u32x4 {
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void*)(uintptr_t)addr, 0, (int)bytes, 0x00020000);
    return __builtin_amdgcn_raw_buffer_load_b128(rs, (int)voff, 0, 0);
  };
  typedef __attribute__((address_space(3))) void* lds_void;
  // The tile to fetch next, as scalars set once per tile: address of this wave's first 4-row group in both
  // tensors, rows left in the sequence from there, strip origin.  A tile that does not exist (end of the list)
  // gets empty descriptors: its loads are still issued, read as zero and land in the stage nobody reads.
  uint64_t nx_a1 = 0, nx_a2 = 0;
  int nx_left = 0, nx_d0x4 = 0, nx_yt = 0;
  uint32_t nx_bias_bytes = 0;
  auto set_next = [&](int yt, bool valid) {
    const int yrow = yt * C::BN + (C::kDma ? 4 * wave : 0);
    nx_yt = yt;
    nx_a1 = (uint64_t)(uintptr_t)Y1 + (uint64_t)(uint32_t)yrow * rowb1;
    nx_a2 = (uint64_t)(uintptr_t)Y2 + (uint64_t)(uint32_t)yrow * rowb2;
    nx_left = valid ? L - yrow : 0;
    // (dK/dV pass, CANDK: a tile of candidate queries stands at position n as a whole: its strip starts there, and entry
    // BX - 1 - (key - x0) of it is the bias of that key against every candidate)
    nx_d0x4 = 4 * ((MODE == kBwdDKDV) ? (CANDK ? min(yt * C::BN, g.n) : yt * C::BN) - x0 - (C::BX - 1) : x0v + (C::BX - 1) - yt * C::BN);
    nx_bias_bytes = valid ? (uint32_t)a.bias_stride * 4u : 0u;
  };
  const uint64_t bias_addr = (uint64_t)(uintptr_t)bias_h;
  // piece c of the next tile, bound for LDS stage `stage`
  auto gload_piece = [&](int c, int stage) {
    if (bias_h) {
#pragma unroll
      for (int j = 0; j < STRIP_J; ++j)
        if (j % C::CPT == c && NWAVES * j + wave < STRIP_RUNS) {
          // byte offset of table entry (distance of strip index s); entries outside [0, bias_stride) are
          // out of range of the descriptor and read as zero
          const uint32_t voff = (MODE == kBwdDKDV) ? (uint32_t)nx_d0x4 + strip_s4[j] : (uint32_t)nx_d0x4 - strip_s4[j];
          const uint32_t dst = (uint32_t)(uintptr_t)(lds_void)(smem + C::STRIP_BASE + stage * C::STRIP_BYTES + 256 * (NWAVES * j + wave));
          dma4(make_rsrc(bias_addr, nx_bias_bytes), voff, dst);
        }
    }
    if constexpr (C::kDma) {
      const int dr = 4 * NWAVES * c;                                     // rows from this wave's group of piece 0 to that of piece c
      const uint32_t left = (uint32_t)max(nx_left - dr, 0);
      const uint32_t dst = (uint32_t)(uintptr_t)(lds_void)(smem + stage * C::STAGE_BYTES + (NWAVES * c + wave) * 1024);
      dma16(make_rsrc(nx_a1 + (uint32_t)dr * rowb1, left * rowb1), voff1, dst);
      dma16(make_rsrc(nx_a2 + (uint32_t)dr * rowb2, left * rowb2), voff2, dst + C::TILE0);
    } else if (C::CHUNKS % C::NT == 0 || tid < C::CHUNKS) {
      const int dr = c * PIECE_ROWS;
      const uint32_t left = (uint32_t)max(nx_left - dr, 0);
      pre1[c] = load16(nx_a1 + (uint32_t)dr * rowb1, left * rowb1, voff1);
      pre2[c] = load16(nx_a2 + (uint32_t)dr * rowb2, left * rowb2, voff2);
    }
  };
  auto gload = [&](int stage) {
#pragma unroll
    for (int c = 0; c < C::CPT; ++c) gload_piece(c, stage);
  };
  auto lstore = [&](int stage) {
    // this wave's direct-to-LDS pieces (strip runs, 256-byte-row tiles) have landed once its load counter
    // drains; the barrier that follows publishes them to the other waves
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if constexpr (!C::kDma) {
#pragma unroll
      for (int c = 0; c < C::CPT; ++c) {
        const int idx = tid + c * C::NT;
        const int row = idx / C::CPR, col = idx % C::CPR;
        if (C::CHUNKS % C::NT == 0 || idx < C::CHUNKS) {
          *(u32x4*)(smem + stage * C::STAGE_BYTES + lds_off<C, 0>(row, col)) = pre1[c];
          *(u32x4*)(smem + stage * C::STAGE_BYTES + C::TILE0 + lds_off<C, 1>(row, col)) = pre2[c];
        }
      }
    }
  };

  if constexpr (C::kStatLds) {
    // this wave's 32 stationary rows of operand 1 (V), straight to LDS; only this wave reads them back
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int rg = wave * 8 + j;                                       // 4-row group inside the block
      const int chunk = (lane & 15) ^ (4 * (lane >> 4) + (rg & 3));
      const uint32_t rowb = (uint32_t)(sr2 * (int64_t)sizeof(E));
      const uint32_t voff = __umul24((uint32_t)(lane >> 4), rowb) + (uint32_t)(chunk * 16);
      const uint32_t dst = (uint32_t)(uintptr_t)(lds_void)(smem + C::STAT_BASE + rg * 1024);
      dma16(tile_rsrc(R2, rowb, x0 + 4 * rg), voff, dst);
    }
  }
  // ---- bias gradient (DBIAS): dacc[p][s] collects dS of tile parity p along strip index
  // s = (y - tile start) + (BX - 1 - (x - x0)), i.e. distance x - y = x0 + BX - 1 - tile start - s
  float* dacc = (float*)(smem + C::DACC_BASE);
  const int dacc_lane = wave * C::DACC_LEN + C::BX - 1 - wave * 32 + 4 * hf - (lane & 15) - 16 * ((lane >> 4) & 1);   // + 32 * sub-block + 16 * class
  auto dacc_flush = [&](int parity, int yt_of) {                         // every wave has passed the barrier after that tile
    if constexpr (DBIAS) {
      if (a.dbias_dist && tid < C::BX + C::BN - 1) {
        float vsum = 0.f;
#pragma unroll
        for (int c = 0; c < C::DACC_COPIES; ++c) {
          vsum += dacc[(parity * C::DACC_COPIES + c) * C::DACC_LEN + tid];
          dacc[(parity * C::DACC_COPIES + c) * C::DACC_LEN + tid] = 0.f;
        }
        const int dist = x0 + C::BX - 1 - yt_of * C::BN - tid;
        if (vsum != 0.f && dist >= 0 && dist < a.bias_stride) atomicAdd(a.dbias_dist + (int64_t)h * a.bias_stride + dist, vsum);
      }
    }
  };
  // adds the 16 scores-gradients this lane holds for one 32-row sub-block of the tile in `stage` (LDS float
  // atomics run one lane per cycle on this part; the private strips make them unnecessary)
  auto dacc_add = [&](int stage, int sub, const float* vals) {
    float x0 = 0.f, x1 = 0.f, x2 = 0.f;
    diag_all(std::make_integer_sequence<int, 16>{}, vals, lane & 15, x0, x1, x2);
    // Strip index of class j at this lane: dacc_lane + 32 * sub + 16 * j.  Two lanes of a wave meet at one address
    // (different half-waves, different classes), so the half-waves and the classes take turns.
    float* base = dacc + stage * C::DACC_COPIES * C::DACC_LEN + dacc_lane + sub * 32;
    const int room = C::DACC_LEN - (dacc_lane - wave * C::DACC_LEN + sub * 32);   // entries from base to the end of the strip
    // (lanes of the two 16-lane rows of a half-wave meet in neighbouring classes, so the classes take turns as well)
#pragma unroll
    for (int hs = 0; hs < 2; ++hs)
#pragma unroll
      for (int j = 0; j < 3; ++j) {
        const float xv = j == 0 ? x0 : (j == 1 ? x1 : x2);
        if (hf == hs && 16 * j < room) {                                 // beyond the strip only zeros would land
          volatile float* p = base + 16 * j;
          *p = *p + xv;
        }
      }
  };
  // A tile that lies far from the diagonal has all its distances inside ONE bucket of the table, or in two neighbouring
  // ones (the buckets of a log-spaced table are hundreds of distances wide there); which distance of a bucket receives a
  // sum does not matter, so such a tile adds plain sums of its dS: one per bucket, kept per lane across consecutive tiles
  // (two open buckets, since the tiles walk from one bucket into the next) and reduced over the wave only when a bucket
  // is left behind.  The test is made for the whole block (its 128 rows against the tile's keys: AttnArgs::bucket_end
  // gives the first distance of the next bucket), so that all waves agree and the per-tile flush of the diagonal strips
  // can be skipped too.
  float run_sum0 = 0.f, run_sum1 = 0.f;
  int run_end0 = 0, run_end1 = 0, run_dist0 = 0, run_dist1 = 0;          // run_end = 0: slot free; a bucket is named by its end
  int run_old = 0;                                                        // the slot opened first
  auto run_flush_slot = [&](float& sum, int& end, int dist) {
    if (end != 0) {
      float v = sum;
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
      if (lane == 0 && v != 0.f) atomicAdd(a.dbias_dist + (int64_t)h * a.bias_stride + dist, v);
      sum = 0.f;
      end = 0;
    }
  };
  auto run_flush = [&]() {
    if constexpr (DBIAS) { run_flush_slot(run_sum0, run_end0, run_dist0); run_flush_slot(run_sum1, run_end1, run_dist1); }
  };
  auto run_to = [&](int end, int dist, float v) {                        // adds v to the bucket that ends at `end` (dist: one of its distances)
    if (run_end0 == end) run_sum0 += v;
    else if (run_end1 == end) run_sum1 += v;
    else if (run_old == 0) {
      run_flush_slot(run_sum0, run_end0, run_dist0);
      run_end0 = end; run_dist0 = dist; run_sum0 = v; run_old = 1;
    } else {
      run_flush_slot(run_sum1, run_end1, run_dist1);
      run_end1 = end; run_dist1 = dist; run_sum1 = v; run_old = 0;
    }
  };
  // vals: the 16 dS of this lane in sub-block `sub` of the tile (keys y0 + 32 sub + 8 (r / 4) + 4 hf + r % 4).  The block's
  // pairs of this tile lie in the bucket that ends at `end` (distances < end) and, if split >= 0, above it in the bucket
  // that ends at `end2`.
  auto run_add = [&](const float* vals, int sub, int y0_, int end, int dist, int end2) {
    float total = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) total += vals[r];
    if (end2 == 0) { run_to(end, dist, total); return; }
    const int thr = x - y0_ - 32 * sub - 4 * hf - end;                   // key offset c <= thr  <=>  distance >= end
    float hi = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) hi += (8 * (r >> 2) + (r & 3) <= thr) ? vals[r] : 0.f;
    run_to(end, dist, total - hi);
    run_to(end2, end, hi);
  };
  if constexpr (DBIAS) {
    for (int i = tid; i < 2 * C::DACC_COPIES * C::DACC_LEN; i += C::NT) dacc[i] = 0.f;
  }
  set_next(t_begin < ntiles ? tr.at(t_begin) : 0, t_begin < ntiles);
  gload(0);
  finish_resident();
  lstore(0);
  __syncthreads();
  HSTU_TLB(1);

  const bool stat_hist = min(xw0 + 32, L) - 1 < g.n;  // this wave's stationary rows are all history rows
  constexpr int NSB = C::BN / 32;                     // 32-row sub-blocks of a streamed tile
  constexpr int SBG = (MODE == kFwd && NSB >= 2) ? 2 : 1;   // sub-blocks whose products are interleaved
  bool prev_fast = false;
  for (int t = t_begin; t < ntiles; ++t) {
    const int yt = nx_yt;                                    // set_next() of the previous round (or of the prologue) named this tile
    const int stage = (t - t_begin) & 1;
    const bool has_next = t + 1 < ntiles;
    set_next(has_next ? tr.at(t + 1) : 0, has_next);
    if constexpr (DBIAS) {
      if (t > t_begin && !prev_fast) dacc_flush(stage ^ 1, tr.at(t - 1));
    }
    const unsigned char* y1s = smem + stage * C::STAGE_BYTES;
    const unsigned char* y2s = y1s + C::TILE0;
    const int y0 = yt * C::BN;
    bool wg_fast = false;                                                 // DBIAS: the whole block's pairs of this tile lie in one or two buckets
    int fast_end = 0, fast_dist = 0, fast_end2 = 0;
    if constexpr (DBIAS) {
      const int xhi = x0 + C::BX - 1, dmin_b = x0 - (y0 + C::BN - 1);
      if (a.bucket_end && a.dbias_dist && dmin_b >= 0 && xhi < g.n && classify_tile(g, x0, xhi, y0, y0 + C::BN - 1, false) == kTileFull) {
        fast_end = a.bucket_end[dmin_b];
        fast_dist = dmin_b;
        wg_fast = true;
        if (fast_end <= xhi - y0) {                                       // a bucket boundary inside the tile's distances
          fast_end2 = a.bucket_end[fast_end];
          wg_fast = fast_end2 > xhi - y0;                                 // ... and only one
        }
      }
      prev_fast = wg_fast;
    }

    // How this wave's 32 stationary rows relate to the tile: nothing visible (skip), everything
    // visible (no mask arithmetic, bias from the strip), or mixed (generic per-element path).
    // Fully visible tiles of candidate rows (all at position n) against history keys are recognised in the instantiations
    // for batches with candidates, but not with the bias gradient, which adds the dS of candidate rows to the table by the
    // distance n - j one by one: those take the masked path.
    int kind = (MODE == kBwdDKDV) ? classify_tile(g, y0, y0 + C::BN - 1, xw0, xw0 + 31, CANDK)
                                  : classify_tile(g, xw0, xw0 + 31, y0, y0 + C::BN - 1, CANDQ && !DBIAS);
    if (xw0 >= L || xw0 + 31 < q0) kind = kTileEmpty;

    // The next tile's global loads are issued piecewise between the score products: the compute unit's
    // memory pipeline takes a 16-byte-per-lane load every few tens of cycles, and a wave that issues
    // its whole share at once sits in that queue instead of feeding the matrix pipe.  A wave with
    // nothing to compute issues them all now.
    if (kind == kTileEmpty) gload(stage ^ 1);

    // Swizzled (direct-to-LDS) tiles: LDS addresses are formed next to each read with one XOR instead of
    // being kept as loop invariants (one register per k-step / feature block otherwise).  For tile row
    // r = 32*sub + l32 the swizzle is a lane constant z, and chunk 2*ks+hf lands at byte
    // 256*r + 16*((2*ks+hf)^z) = 8192*sub + (kb ^ 32*ks).  For the transpose reads (row R + 4*hf + i16/4 + 8*hi,
    // R a multiple of 16, chunk 4*ob + vchunk) z = 4*(i16/4) + hf + 2*hi and the byte is
    // 256*R + 2048*hi + (tb ^ (64*ob | 32*hi)).
    const int vchunk = 2 * (grp16 & 1) + ((i16 & 3) >> 1), vbyte = 8 * (i16 & 1);
    const int zl = 4 * (l32 & 3) + ((l32 >> 2) & 3);
    // (the LDS base rides in kb / tb: reading through `smem + offset` costs an extra vector add per fragment)
    const int smem_base = (int)(uint32_t)(uintptr_t)(lds_void)smem;
    int kb = smem_base + stage * C::STAGE_BYTES + l32 * 256 + ((hf ^ (zl & 1)) << 4) + ((zl >> 1) << 5);
    int tb = smem_base + stage * C::STAGE_BYTES + (4 * hf + (i16 >> 2)) * 256 + ((i16 >> 2) << 6) + ((vchunk ^ hf) << 4) + vbyte;
    asm volatile("" : "+v"(kb), "+v"(tb));
    typedef __attribute__((address_space(3))) short4v* lds_s4;
    typedef __attribute__((address_space(3))) const bf16x8* lds_b8;
    // row fragment (A operand of a score product): tensor, 32-row sub-block, k-step
    auto rowfrag_at = [&](int tensor, int sub, int ks) -> bf16x8 {
      if constexpr (C::kDma) {
        return *(lds_b8)(uintptr_t)(uint32_t)((kb ^ (ks << 5)) + sub * 8192 + tensor * C::TILE0);
      } else {
        return tensor == 0 ? *(const bf16x8*)(y1s + lds_off<C, 0>(sub * 32 + l32, 2 * ks + hf))
                           : *(const bf16x8*)(y2s + lds_off<C, 1>(sub * 32 + l32, 2 * ks + hf));
      }
    };
    // transposed fragment (A operand of an output product): tensor, sub-block, 16-row k-step, feature block
    auto trfrag_at = [&](int tensor, int sub, int ks2, int ob) -> bf16x8 {
      short4v lo, hi;
      if constexpr (C::kDma) {
        const int roff = (sub * 32 + ks2 * 16) * 256 + tensor * C::TILE0;
        lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(uintptr_t)(uint32_t)((tb ^ (ob << 6)) + roff));
        hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(uintptr_t)(uint32_t)((tb ^ ((ob << 6) | 32)) + roff + 2048));
      } else {
        const int trow = sub * 32 + ks2 * 16 + 4 * hf + (i16 >> 2);
        if (tensor == 0) {
          lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(y1s + lds_off<C, 0>(trow, 4 * ob + vchunk) + vbyte));
          hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(y1s + lds_off<C, 0>(trow + 8, 4 * ob + vchunk) + vbyte));
        } else {
          lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(y2s + lds_off<C, 1>(trow, 4 * ob + vchunk) + vbyte));
          hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(y2s + lds_off<C, 1>(trow + 8, 4 * ob + vchunk) + vbyte));
        }
      }
      return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };

    bool done = false;
    if constexpr (MODE != kFwd && C::kBf16 && NSB == 2 && D == 128) {
      if (kind == kTileFull) {
        // Software-pipelined backward for fully visible tiles: the pointwise
        // work of one 32-row sub-block (SiLU, its derivative, packing) is issued between the matrix
        // instructions that do not depend on it:
        //   S,dP(0) | S,dP(1) + pointwise(0) | outputs(0) + pointwise(1) | outputs(1)
        // outputs = dQ^T += K^T dS^T (dQ pass) or dK^T += Q^T dS, dV^T += dO^T P (dK/dV pass).
        static_assert(C::kDma, "256-byte-row tiles only");
        const float* strip = (const float*)(smem + C::STRIP_BASE + stage * C::STRIP_BYTES) + strip_lane;
        // score fragment n: tensor n%2 (S then dP), sub-block n/16, k-step (n/2)%8
        auto rowfrag = [&](int n) -> bf16x8 { return rowfrag_at(n & 1, n >> 4, (n >> 1) & 7); };
        // output fragment n: sub-block n / (8*NOUT), then (k-step, feature block) major, output minor
        auto trfrag = [&](int n) -> bf16x8 {
          const int r = n % (8 * C::NOUT), step = r / C::NOUT;
          return trfrag_at(r % C::NOUT, n / (8 * C::NOUT), step / C::OB, step % C::OB);
        };
        f32x16 sv[2], dp[2];
        uint32_t pds[2][8], pp[2][8];
        float dsf[DBIAS ? 2 : 1][16];                                      // dS in fp32 for the bias gradient
#pragma unroll
        for (int sb = 0; sb < 2; ++sb) {
          if (bias_h) {
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
              const f32x4 bv = *(const f32x4*)(strip + sb * 32 + 8 * q4);
              sv[sb][4 * q4 + 0] = bv[0]; sv[sb][4 * q4 + 1] = bv[1]; sv[sb][4 * q4 + 2] = bv[2]; sv[sb][4 * q4 + 3] = bv[3];
            }
          } else {
#pragma unroll
            for (int r = 0; r < 16; ++r) sv[sb][r] = 0.f;
          }
#pragma unroll
          for (int r = 0; r < 16; ++r) dp[sb][r] = 0.f;
        }
        // elements 2m, 2m+1 of sub-block sb -> packed pairs of dS (and of P for the dK/dV pass);
        auto pointwise = [&](int sb, int m) {
          const float s0v = sv[sb][2 * m], s1v = sv[sb][2 * m + 1];
          const float g0 = sigmoid_l2(s0v), g1 = sigmoid_l2(s1v);
          const float p0v = s0v * g0, p1v = s1v * g1;
          const float ds0 = dp[sb][2 * m] * dsilu_l2(p0v, g0), ds1 = dp[sb][2 * m + 1] * dsilu_l2(p1v, g1);
          pds[sb][m] = pack_bf16x2(ds0, ds1);
          if constexpr (MODE == kBwdDKDV) pp[sb][m] = pack_bf16x2(p0v, p1v);
          if constexpr (DBIAS) { dsf[sb][2 * m] = ds0; dsf[sb][2 * m + 1] = ds1; }
        };
        constexpr int PF = (MODE == kBwdDQ) ? 2 : 4;                      // the dQ pass runs two waves per SIMD: 256 registers
        bf16x8 fr[PF];
#pragma unroll
        for (int i = 0; i < PF; ++i) fr[i] = rowfrag(i);
#pragma unroll
        for (int n = 0; n < 32; ++n) {
          const bf16x8 fa = fr[n % PF];
          if (n + PF < 32) fr[n % PF] = rowfrag(n + PF);
          if (n % (32 / C::CPT) == 0) gload_piece(n / (32 / C::CPT), stage ^ 1);
          __builtin_amdgcn_sched_barrier(0);
          const int sb = n >> 4, ks = (n >> 1) & 7;
          if (n & 1) dp[sb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, res[1][ks], dp[sb], 0, 0, 0);
          else sv[sb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, res[0][ks], sv[sb], 0, 0, 0);
          if (n >= 16 && (n & 1)) pointwise(0, (n - 16) >> 1);
          __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (DBIAS) {                                            // fully visible tile: history rows, distance x - y
          if (wg_fast) run_add(dsf[0], 0, y0, fast_end, fast_dist, fast_end2); else dacc_add(stage, 0, dsf[0]);
        }
        constexpr int NO = 16 * C::NOUT;                                  // output products of the tile
#pragma unroll
        for (int i = 0; i < PF; ++i) fr[i] = trfrag(i);
#pragma unroll
        for (int n = 0; n < NO; ++n) {
          const bf16x8 fa = fr[n % PF];
          if (n + PF < NO) fr[n % PF] = trfrag(n + PF);
          __builtin_amdgcn_sched_barrier(0);
          const int sb = n / (8 * C::NOUT), r = n % (8 * C::NOUT), step = r / C::NOUT, o = r % C::NOUT;
          const int ks2 = step / C::OB, ob = step % C::OB;
          const uint32_t* pk = (o == 0) ? pds[sb] : pp[sb];
          const bf16x8 pb = __builtin_bit_cast(bf16x8, (u32x4){pk[4 * ks2], pk[4 * ks2 + 1], pk[4 * ks2 + 2], pk[4 * ks2 + 3]});
          out[o][ob] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, pb, out[o][ob], 0, 0, 0);
          if (sb == 0 && o == C::NOUT - 1) pointwise(1, step);
          __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (DBIAS) {
          if (wg_fast) run_add(dsf[1], 1, y0, fast_end, fast_dist, fast_end2); else dacc_add(stage, 1, dsf[1]);
        }
        done = true;
      }
    }
    if constexpr (MODE == kBwdDKDV && C::kBf16 && NSB == 1 && D == 128 && C::kStatLds) {
      // Software-pipelined dK/dV pass for fully visible 32-query tiles.  A matrix instruction hides vector instructions
      // only when they follow it in the same wave, so the pointwise work rides behind this wave's own products:
      //   slots  0..7   S  = Q K^T
      //   slots  8..15  dP = dO V^T            | the part of the pointwise work that needs S only (sigmoid, P, dS/dP), as a
      //   slots 16..19  dV^T += dO^T P, q 0..15  |   three-stage rolling chain (exp2; add, rcp; multiply-adds) over the 16
      //   slots 20..23  dK^T += Q^T dS, q 0..15  |   score registers, finishing register 7 in slot 15 and register 15 in slot 23;
      //   slots 24..27  dV^T, q 16..31           | dS = dP * (dS/dP) and its packing: q 0..15 in slots 17..19, q 16..31 in 24..27
      //   slots 28..31  dK^T, q 16..31
      // (score register r of a lane belongs to query 8 (r / 4) + 4 hf + r % 4: registers 0..7 are the queries of the
      // first 16-row k-step of the output products.)
      const bool tile_hist_f = min(y0 + C::BN, L) - 1 < g.n;               // candidate queries take the general path
      if (kind == kTileFull && (!CANDK || tile_hist_f)) {
        f32x16 sv, dp;
        if (bias_h) {
          const float* strip = (const float*)(smem + C::STRIP_BASE + stage * C::STRIP_BYTES) + strip_lane;
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            const f32x4 bv = *(const f32x4*)(strip + 8 * q4);
            sv[4 * q4 + 0] = bv[0]; sv[4 * q4 + 1] = bv[1]; sv[4 * q4 + 2] = bv[2]; sv[4 * q4 + 3] = bv[3];
          }
        } else {
#pragma unroll
          for (int r = 0; r < 16; ++r) sv[r] = 0.f;
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) dp[r] = 0.f;
        auto statfrag = [&](int ks) -> bf16x8 {                           // V rows of this wave's keys: B operand of dP
          return *(lds_b8)(uintptr_t)(uint32_t)(((kb - stage * C::STAGE_BYTES) ^ (ks << 5)) + C::STAT_BASE + wave * 8192);
        };
        // rolling pointwise chain over the score registers: E(r) exp2(-s); R(r) sigmoid; F(r) P (in place of s), dS/dP, packing of P
        float ex[16], sg_[16], fac[16];
        uint32_t pp[8], pds[8];
        auto E_ = [&](int r) { ex[r] = __builtin_amdgcn_exp2f(-sv[r]); };
        auto R_ = [&](int r) { sg_[r] = __builtin_amdgcn_rcpf(1.0f + ex[r]); };
        auto F_ = [&](int r) {
          const float pv = sv[r] * sg_[r];
          fac[r] = dsilu_l2(pv, sg_[r]);
          sv[r] = pv;
          if (r & 1) { pp[r >> 1] = pack_bf16x2(sv[r - 1], sv[r]); asm volatile("" : "+v"(pp[r >> 1])); }
        };
        auto DS_ = [&](int m) {                                           // registers 2m, 2m + 1
          pds[m] = pack_bf16x2(dp[2 * m] * fac[2 * m], dp[2 * m + 1] * fac[2 * m + 1]);
          asm volatile("" : "+v"(pds[m]));
        };
        // what slot `sl` carries of the chain (register r: E in slot 6 + r, but not before slot 8; R one slot later; F two)
        auto chain = [&](int sl) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int e_slot = r < 2 ? 8 : 6 + r;
            if (sl == e_slot) E_(r);
          }
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int e_slot = r < 2 ? 8 : 6 + r;
            if (sl == e_slot + 1) R_(r);
          }
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int e_slot = r < 2 ? 8 : 6 + r;
            if (sl == e_slot + 2) F_(r);
          }
          if (sl == 17) { DS_(0); }
          if (sl == 18) { DS_(1); DS_(2); }
          if (sl == 19) { DS_(3); }
          if (sl >= 24 && sl < 28) DS_(sl - 20);
        };
        constexpr int PF = HSTU_DKDV_PF;                                  // fragments are fetched PF slots ahead of their product
        // A operand of slot n: Q rows (S), dO rows (dP), dO^T (dV), Q^T (dK)
        auto afrag = [&](int n) -> bf16x8 {
          if (n < 8) return rowfrag_at(0, 0, n);
          if (n < 16) return rowfrag_at(1, 0, n - 8);
          const int ks2 = (n - 16) >> 3, o = ((n - 16) >> 2) & 1, ob = n & 3;   // o = 0: dV (dO^T), 1: dK (Q^T)
          return trfrag_at(o == 0 ? 1 : 0, 0, ks2, ob);
        };
        bf16x8 fr[PF], fv[PF];
#pragma unroll
        for (int i = 0; i < PF; ++i) fr[i] = afrag(i);
#pragma unroll
        for (int n = 0; n < 32; ++n) {
          const bf16x8 fa = fr[n % PF];
          const bf16x8 fb = fv[n % PF];
          if (n + PF < 32) fr[n % PF] = afrag(n + PF);
          if (n + PF >= 8 && n + PF < 16) fv[n % PF] = statfrag(n + PF - 8);
          if (n % (8 / C::CPT) == 0 && n < 8) gload_piece(n / (8 / C::CPT), stage ^ 1);
          __builtin_amdgcn_sched_barrier(0);
          if (n < 8) sv = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, res[0][n], sv, 0, 0, 0);
          else if (n < 16) dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, dp, 0, 0, 0);
          else {
            const int ks2 = (n - 16) >> 3, o = ((n - 16) >> 2) & 1, ob = n & 3;
            const uint32_t* pk = (o == 0) ? pp : pds;
            const bf16x8 pb = __builtin_bit_cast(bf16x8, (u32x4){pk[4 * ks2], pk[4 * ks2 + 1], pk[4 * ks2 + 2], pk[4 * ks2 + 3]});
            out[1 - o][ob] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, pb, out[1 - o][ob], 0, 0, 0);
          }
          __builtin_amdgcn_sched_barrier(0);
          chain(n);
          __builtin_amdgcn_sched_barrier(0);
        }
        done = true;
      }
    }
    if (kind != kTileEmpty && !done) {                                   // wave-uniform
#pragma unroll
      for (int sg = 0; sg < NSB; sg += SBG) {
        // ---- scores of SBG sub-blocks at once: independent accumulators keep the matrix pipe fed
        f32x16 sc1[SBG], sc2[SBG];
        // Mixed tile whose (existing) query rows are all history rows: every visible pair has distance i - j >= 0, which is
        // what the strip is indexed by, so the scores are seeded like a full tile's and only the mask is applied
        // per element (no table gathers, whose wait would also wait for the tile being fetched).
        // In the dK/dV pass the query rows are the streamed tile's.
        // In the query-stationary passes candidate rows against history keys work the same way with the rows' effective
        // position n; in the dK/dV pass a tile of candidate queries has its strip anchored at n (see set_next).
        const bool tile_hist = min(y0 + C::BN, L) - 1 < g.n;                 // the streamed rows are all history
        // dK/dV pass with candidates: a tile of candidate queries against a wave of history keys
        const bool cand_tile = CANDK && y0 >= g.n && stat_hist;
        const bool seeded = kind == kTilePartial && (MODE == kBwdDKDV ? (tile_hist || cand_tile) : (stat_hist || (CANDQ && tile_hist)));
        if (CANDK && cand_tile && (kind == kTileFull || seeded) && bias_h) {
          // entry BX - 1 - (x - x0) of the strip anchored at n (strip_lane also carries this lane's 4 hf register offset)
          const float bias_c = *((const float*)(smem + C::STRIP_BASE + stage * C::STRIP_BYTES) + strip_lane - 4 * hf);
#pragma unroll
          for (int u = 0; u < SBG; ++u)
#pragma unroll
            for (int r = 0; r < 16; ++r) sc1[u][r] = bias_c;
        } else if ((kind == kTileFull || seeded) && bias_h) {
          // the distance of every pair that counts is >= 0: seed the accumulators with the bias strip
          const float* strip = (const float*)(smem + C::STRIP_BASE + stage * C::STRIP_BYTES) + strip_lane;
#pragma unroll
          for (int u = 0; u < SBG; ++u)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
              const f32x4 bv = *(const f32x4*)(strip + (sg + u) * 32 + 8 * q4);
              sc1[u][4 * q4 + 0] = bv[0]; sc1[u][4 * q4 + 1] = bv[1];
              sc1[u][4 * q4 + 2] = bv[2]; sc1[u][4 * q4 + 3] = bv[3];
            }
        } else {
          // (opaque moves: otherwise the compiler clears the registers ahead of the branch, on the strip's path too)
#pragma unroll
          for (int u = 0; u < SBG; ++u)
#pragma unroll
            for (int r = 0; r < 16; ++r) asm volatile("v_mov_b32 %0, 0" : "=v"(sc1[u][r]));
        }
        if constexpr (MODE != kFwd) {
#pragma unroll
          for (int u = 0; u < SBG; ++u)
#pragma unroll
            for (int r = 0; r < 16; ++r) sc2[u][r] = 0.f;
        }
        if constexpr (C::kBf16) {
          // A-operand fragments are fetched one k-step ahead of the product that consumes them
          bf16x8 f1[2][SBG], f2[2][SBG], fs[2];
          // stationary operand 1 when it lives in LDS: B fragment of this wave's row x
          auto statfrag = [&](int ks) -> bf16x8 {
            return *(lds_b8)(uintptr_t)(uint32_t)(((kb - stage * C::STAGE_BYTES) ^ (ks << 5)) + C::STAT_BASE + wave * 8192);
          };
          if constexpr (C::kStatLds) fs[0] = statfrag(0);
#pragma unroll
          for (int u = 0; u < SBG; ++u) {
            f1[0][u] = rowfrag_at(0, sg + u, 0);
            if (MODE != kFwd) f2[0][u] = rowfrag_at(1, sg + u, 0);
          }
#pragma unroll
          for (int ks = 0; ks < C::KS; ++ks) {
            if (ks + 1 < C::KS) {
              if constexpr (C::kStatLds) fs[(ks + 1) & 1] = statfrag(ks + 1);
#pragma unroll
              for (int u = 0; u < SBG; ++u) {
                f1[(ks + 1) & 1][u] = rowfrag_at(0, sg + u, ks + 1);
                if (MODE != kFwd) f2[(ks + 1) & 1][u] = rowfrag_at(1, sg + u, ks + 1);
              }
            }
            if constexpr (C::KS % C::CPT == 0) {
              if (sg == 0 && ks % (C::KS / C::CPT) == 0) gload_piece(ks / (C::KS / C::CPT), stage ^ 1);
            } else {
              if (sg == 0 && ks == 0) gload(stage ^ 1);
            }
            __builtin_amdgcn_sched_barrier(0);                           // keep the fetches ahead of the products
#pragma unroll
            for (int u = 0; u < SBG; ++u) {
              sc1[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1[ks & 1][u], res[0][ks], sc1[u], 0, 0, 0);
              if constexpr (MODE != kFwd) {
                if constexpr (C::kStatLds) sc2[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f2[ks & 1][u], fs[ks & 1], sc2[u], 0, 0, 0);
                else sc2[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f2[ks & 1][u], res[1][ks], sc2[u], 0, 0, 0);
              }
            }
          }
        } else {
          if (sg == 0) gload(stage ^ 1);
#pragma unroll
          for (int ks = 0; ks < C::KS; ++ks)
#pragma unroll
            for (int u = 0; u < SBG; ++u) {
              const int roff = ((sg + u) * 32 + l32) * C::STRIDE0 + (2 * ks + hf) * 4;   // STRIDE0 == STRIDE1 in fp32
              sc1[u] = __builtin_amdgcn_mfma_f32_32x32x2f32(*(const float*)(y1s + roff), res[0][ks], sc1[u], 0, 0, 0);
              if constexpr (MODE != kFwd)
                sc2[u] = __builtin_amdgcn_mfma_f32_32x32x2f32(*(const float*)(y2s + roff), res[1][ks], sc2[u], 0, 0, 0);
            }
        }

        // ---- pointwise: SiLU (forward) or its derivative times dP (backward), mask in registers
        float c1[SBG][16], c2[SBG][16];
        if (kind == kTileFull) {
#pragma unroll
          for (int u = 0; u < SBG; ++u)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const float sv = sc1[u][r];
              const float sig = sigmoid_l2(sv);
              if (MODE == kFwd) {
                c1[u][r] = sv * sig;
              } else {
                c1[u][r] = sc2[u][r] * dsilu_l2(sv * sig, sig);
                c2[u][r] = sv * sig;
              }
            }
        } else {
          // one score of the mixed path: t = score in ln 2 units, vis = pair visible
          auto mixed = [&](int u, int r, float t, bool vis) {
            const float sig = sigmoid_l2(t);
            const float p = t * sig;
            if (MODE == kFwd) {
              c1[u][r] = vis ? p : 0.f;
            } else {
              const float ds = sc2[u][r] * dsilu_l2(p, sig);
              c1[u][r] = vis ? ds : 0.f;
              c2[u][r] = vis ? p : 0.f;
            }
          };
          if (CANDK && seeded && cand_tile) {
            // candidate queries (all at position n) against history keys: one yes/no per key, and the rows past the end
            const bool key_vis = x_ok && (g.K1 < 0 || g.n - x < g.K1 || x < g.K2);
            const int up = key_vis ? L - 1 - y0 - 4 * hf : -1;
#pragma unroll
            for (int u = 0; u < SBG; ++u)
#pragma unroll
              for (int r = 0; r < 16; ++r) mixed(u, r, sc1[u][r], (sg + u) * 32 + 8 * (r >> 2) + (r & 3) <= up);
          } else if (seeded && MODE == kBwdDKDV) {
            // History rows only, seen from key x: the queries y >= x with y - x < K1 (any y >= x for a key of the global
            // prefix or a dense mask), and y < L.  Query = y0 + c + 4 hf, c a compile-time constant per register.
            const int lo = (x_ok ? x - y0 : (1 << 30)) - 4 * hf;                              // c >= lo  <=>  y >= x
            const int band = (g.K1 < 0 || x < g.K2) ? (1 << 30) : x + g.K1 - 1 - y0;           // last query of the band
            const int up = min(band, L - 1 - y0) - 4 * hf;                                     // c <= up
            const int kfirst = max(xw0, g.K2);                                                 // first key of the wave outside the prefix
            const bool need_lo = y0 < min(xw0 + 31, L - 1);
            const bool need_up = y0 + C::BN > L || (g.K1 >= 0 && kfirst <= xw0 + 31 && y0 + C::BN - 1 - kfirst >= g.K1);
            if (need_lo && !need_up) {
#pragma unroll
              for (int u = 0; u < SBG; ++u)
#pragma unroll
                for (int r = 0; r < 16; ++r) mixed(u, r, sc1[u][r], (sg + u) * 32 + 8 * (r >> 2) + (r & 3) >= lo);
            } else if (need_up && !need_lo) {
#pragma unroll
              for (int u = 0; u < SBG; ++u)
#pragma unroll
                for (int r = 0; r < 16; ++r) mixed(u, r, sc1[u][r], (sg + u) * 32 + 8 * (r >> 2) + (r & 3) <= up);
            } else {
#pragma unroll
              for (int u = 0; u < SBG; ++u)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                  const int c = (sg + u) * 32 + 8 * (r >> 2) + (r & 3);
                  mixed(u, r, sc1[u][r], c >= lo && c <= up);
                }
            }
          } else if (seeded) {
            // History rows only: row x sees the keys y <= x with x - y < K1 or y < K2.  Relative to the tile's first key and
            // to this lane's register pattern (key = y0 + c + 4 hf, c a compile-time constant per register) these are three
            // per-lane bounds, and the ones that cannot bind anywhere in this wave's 32 x BN pairs are dropped for the tile.
            // (a candidate row stands at px = n; then the tile holds history keys only and the first bound never binds)
            const int px = CANDQ ? min(x, g.n) : x;
            const int up = (x_ok ? px - y0 : -1) - 4 * hf;               // c <= up   <=>  y <= x (no key for a row past the end)
            const int lo = px - g.K1 + 1 - y0 - 4 * hf;                   // c >= lo   <=>  x - y < K1
            const int pre = g.K2 - y0 - 4 * hf;                           // c <  pre  <=>  y < K2
            const bool need_lo = g.K1 >= 0 && min(min(xw0 + 31, L - 1), g.n) - y0 >= g.K1;
            const bool need_pre = need_lo && g.K2 > y0;
            if (!need_lo) {
#pragma unroll
              for (int u = 0; u < SBG; ++u)
#pragma unroll
                for (int r = 0; r < 16; ++r) mixed(u, r, sc1[u][r], (sg + u) * 32 + 8 * (r >> 2) + (r & 3) <= up);
            } else if (!need_pre) {
#pragma unroll
              for (int u = 0; u < SBG; ++u)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                  const int c = (sg + u) * 32 + 8 * (r >> 2) + (r & 3);
                  mixed(u, r, sc1[u][r], c <= up && c >= lo);
                }
            } else {
#pragma unroll
              for (int u = 0; u < SBG; ++u)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                  const int c = (sg + u) * 32 + 8 * (r >> 2) + (r & 3);
                  mixed(u, r, sc1[u][r], c <= up && (c >= lo || c < pre));
                }
            }
          } else {
#pragma unroll
            for (int u = 0; u < SBG; ++u)
#pragma unroll
              for (int r = 0; r < 16; ++r) {
                const int y = y0 + (sg + u) * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
                int delta;
                const bool vis = (MODE == kBwdDKDV) ? visible(g, y, x, delta) : visible(g, x, y, delta);
                float bv = 0.f;
                if (bias_h) bv = bias_h[vis ? delta : 0];
                mixed(u, r, sc1[u][r] + bv, vis);
              }
          }
        }

        if constexpr (DBIAS) {
          // dS per distance: history rows add along the tile's diagonals in LDS; candidate rows (their distance
          // is n - j, not i - j) are few and add to the global table directly
#pragma unroll
          for (int u = 0; u < SBG; ++u) {
            float hv[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              hv[r] = x < g.n ? c1[u][r] : 0.f;
              if (x >= g.n && c1[u][r] != 0.f) {
                int delta;
                if (visible(g, x, y0 + (sg + u) * 32 + 8 * (r >> 2) + 4 * hf + (r & 3), delta))
                  atomicAdd(a.dbias_dist + (int64_t)h * a.bias_stride + delta, c1[u][r]);
              }
            }
            if (wg_fast) run_add(hv, sg + u, y0, fast_end, fast_dist, fast_end2); else dacc_add(stage, sg + u, hv);
          }
        }

        // ---- second products: out^T[feature][x] += Y^T[feature][y] * coeff[y][x]
        if constexpr (C::kBf16) {
          // transpose load: within a group of 16 lanes, lane 4r+c supplies the address of 4 features
          // (4c..4c+3) of streamed row r and lane i receives feature i of rows 0..3.  The 8 k-slots of
          // this lane in k-step ks2 are streamed rows ks2*16 + 4*hf + {0..3} and + 8 + {0..3}.
          constexpr int NSTEP = SBG * 2 * C::OB;                          // (sub-block, k-step, feature block)
          constexpr int TSRC = (MODE == kFwd) ? 1 : 0;                    // V (forward), K (dQ), Q (dK)
          auto fetch = [&](int step, int tensor) -> bf16x8 {
            return trfrag_at(tensor, sg + step / (2 * C::OB), (step / C::OB) & 1, step % C::OB);
          };
          uint32_t pk1[SBG][8], pk2[SBG][8];
#pragma unroll
          for (int u = 0; u < SBG; ++u)
#pragma unroll
            for (int m = 0; m < 8; ++m) {
              pk1[u][m] = pack_bf16x2(c1[u][2 * m], c1[u][2 * m + 1]);
              if (MODE == kBwdDKDV) pk2[u][m] = pack_bf16x2(c2[u][2 * m], c2[u][2 * m + 1]);
            }
          bf16x8 a1[2], a2[2];
          a1[0] = fetch(0, TSRC);
          if (MODE == kBwdDKDV) a2[0] = fetch(0, 1);
#pragma unroll
          for (int step = 0; step < NSTEP; ++step) {
            if (step + 1 < NSTEP) {
              a1[(step + 1) & 1] = fetch(step + 1, TSRC);
              if (MODE == kBwdDKDV) a2[(step + 1) & 1] = fetch(step + 1, 1);
            }
            __builtin_amdgcn_sched_barrier(0);
            const int u = step / (2 * C::OB), ks2 = (step / C::OB) & 1, ob = step % C::OB;
            const bf16x8 b1 = __builtin_bit_cast(bf16x8, (u32x4){pk1[u][4 * ks2], pk1[u][4 * ks2 + 1], pk1[u][4 * ks2 + 2], pk1[u][4 * ks2 + 3]});
            out[0][ob] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1[step & 1], b1, out[0][ob], 0, 0, 0);
            if constexpr (MODE == kBwdDKDV) {                            // dV^T += dO^T P
              const bf16x8 b2 = __builtin_bit_cast(bf16x8, (u32x4){pk2[u][4 * ks2], pk2[u][4 * ks2 + 1], pk2[u][4 * ks2 + 2], pk2[u][4 * ks2 + 3]});
              out[1][ob] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2[step & 1], b2, out[1][ob], 0, 0, 0);
            }
          }
        } else {
#pragma unroll
          for (int u = 0; u < SBG; ++u)
#pragma unroll
            for (int ks2 = 0; ks2 < 16; ++ks2) {
              // k-step ks2 contracts the two streamed rows 8*(ks2/4) + ks2%4 (+4 for the upper half-wave)
              const int trow = (sg + u) * 32 + 8 * (ks2 >> 2) + 4 * hf + (ks2 & 3);
#pragma unroll
              for (int ob = 0; ob < C::OB; ++ob) {
                const int off = trow * C::STRIDE0 + (ob * 32 + l32) * 4;
                const unsigned char* src0 = (MODE == kFwd) ? y2s : y1s;
                const float af = *(const float*)(src0 + off);
                out[0][ob] = __builtin_amdgcn_mfma_f32_32x32x2f32(af, c1[u][ks2], out[0][ob], 0, 0, 0);
                if constexpr (MODE == kBwdDKDV) {
                  const float af2 = *(const float*)(y2s + off);
                  out[1][ob] = __builtin_amdgcn_mfma_f32_32x32x2f32(af2, c2[u][ks2], out[1][ob], 0, 0, 0);
                }
              }
            }
        }
      }
    }

    lstore(stage ^ 1);                                      // also after the last tile: its (empty) loads must have landed before the LDS is given up
    __syncthreads();
  }

  if constexpr (DBIAS) {
    if (ntiles > t_begin && !prev_fast) dacc_flush((ntiles - 1 - t_begin) & 1, tr.at(ntiles - 1));
    run_flush();
  }
  HSTU_TLB(2);
  // ---- epilogue: scale once, convert, store.  Lane x holds features ob*32 + 8*(r/4) + 4*hf + r%4.
  {
    if (item.slot >= 0) {
      // a piece of a cut block: raw fp32 sums go to its slot [outputs][block row][D]; the combine kernel finishes
      float* dst = a.partial + (((int64_t)item.slot * C::NOUT) * C::BX + (wave * 32 + l32)) * D;
#pragma unroll
      for (int o = 0; o < C::NOUT; ++o)
#pragma unroll
        for (int ob = 0; ob < C::OB; ++ob)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4)
            *(f32x4*)(dst + (int64_t)o * C::BX * D + ob * 32 + 8 * q4 + 4 * hf) =
                (f32x4){out[o][ob][4 * q4 + 0], out[o][ob][4 * q4 + 1], out[o][ob][4 * q4 + 2], out[o][ob][4 * q4 + 3]};
      HSTU_TLB(3);
      return;
    }
  }
  if (!x_ok || x < q0) { HSTU_TLB(3); return; }
#pragma unroll
  for (int o = 0; o < C::NOUT; ++o) {
    E* dst;
    int64_t sd;
    float scale;
    if (MODE == kFwd) { dst = (E*)a.out; sd = a.so; scale = a.inv_n * kLn2; }
    else if (MODE == kBwdDQ) { dst = (E*)a.dq; sd = a.sq; scale = a.inv_n * a.alpha; }
    else if (o == 0) { dst = (E*)a.dk; sd = a.sk; scale = a.inv_n * a.alpha; }
    else { dst = (E*)a.dv; sd = a.sv; scale = a.inv_n * kLn2; }
    dst += (int64_t)(seq0 + x) * sd + hoff;
    // the operand was SiLU(pre): hand back the gradient of pre
    const __bf16* pre = nullptr;
    if constexpr (C::kBf16 && MODE != kFwd) {
      pre = (const __bf16*)(MODE == kBwdDQ ? a.pre_q : (o == 0 ? a.pre_k : a.pre_v));
      if (pre) pre += (int64_t)(seq0 + x) * a.s_pre + hoff;
    }
#pragma unroll
    for (int ob = 0; ob < C::OB; ++ob)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int f = ob * 32 + 8 * q4 + 4 * hf;
        float v0 = out[o][ob][4 * q4 + 0] * scale, v1 = out[o][ob][4 * q4 + 1] * scale;
        float v2 = out[o][ob][4 * q4 + 2] * scale, v3 = out[o][ob][4 * q4 + 3] * scale;
        if constexpr (C::kBf16 && MODE != kFwd) {
          if (pre) {
            const u32x2 t = *(const u32x2*)(pre + f);
            v0 *= dsilu(__uint_as_float(t[0] << 16)); v1 *= dsilu(__uint_as_float(t[0] & 0xFFFF0000u));
            v2 *= dsilu(__uint_as_float(t[1] << 16)); v3 *= dsilu(__uint_as_float(t[1] & 0xFFFF0000u));
          }
        }
        if constexpr (C::kBf16) {
          *(u32x2*)(dst + f) = (u32x2){pack_bf16x2(v0, v1), pack_bf16x2(v2, v3)};
        } else {
          *(f32x4*)(dst + f) = (f32x4){v0, v1, v2, v3};
        }
      }
  }
#if HSTU_BWD_TIMELINE
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  HSTU_TLB(3);
#endif
}

// Adds the partial sums of one cut block in piece order (fixed order: deterministic), applies the output scale and
// writes the rows: dK and dV of a key block cut along the query axis, or the attention output (forward) or dQ (dQ pass) of
// a query block cut along the key axis (small batches; the forward over a query tail: few rows against long histories).
// Grid: (possible cut blocks, 8); block (b, rb, h) rows split 8 ways.
enum { kCombineDKDV = 0, kCombineFwd = 1, kCombineDQ = 2 };
template <typename E, int D, int WHAT>
__global__ __launch_bounds__(256) void combine_kernel(const AttnArgs a, int block_rows) {
  constexpr bool FWD = WHAT == kCombineFwd;
  const int si = blockIdx.x;
  if (si >= a.header->splits) return;
  const SplitItem it = a.splits[si];
  const int seq0 = a.offsets[it.b], L = a.offsets[it.b + 1] - seq0;
  const int xb = it.rb_h >> 8, h = it.rb_h & 255;
  constexpr int VPR = D / 4;                                           // float4 per row
  constexpr int NOUT = WHAT == kCombineDKDV ? 2 : 1;
  int q0 = 0;
  if (FWD && a.query_tail > 0) q0 = max(L - (a.num_targets ? a.num_targets[it.b] : 0) - a.query_tail, 0);
  const int rows_here = block_rows / 8;
  for (int i = threadIdx.x; i < NOUT * rows_here * VPR; i += 256) {
    const int o = i / (rows_here * VPR), r = blockIdx.y * rows_here + (i / VPR) % rows_here, c4 = i % VPR;
    const int x = xb * block_rows + r;
    if (x >= L || x < q0) continue;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int pc = 0; pc < it.pieces; ++pc)
      acc += *(const f32x4*)(a.partial + ((((int64_t)(it.first_slot + pc) * NOUT + o) * block_rows + r) * D) + 4 * c4);
    const float scale = (!FWD && o == 0) ? a.inv_n * a.alpha : a.inv_n * kLn2;      // dQ and dK owe alpha, the forward and dV ln 2
    acc *= scale;
    E* base = FWD ? (E*)a.out : (WHAT == kCombineDQ ? (E*)a.dq : (E*)(o == 0 ? a.dk : a.dv));
    const int64_t stride = FWD ? a.so : (WHAT == kCombineDQ ? a.sq : (o == 0 ? a.sk : a.sv));
    E* dst = base + (int64_t)(seq0 + x) * stride + (int64_t)h * D + 4 * c4;
    if constexpr (sizeof(E) == 2 && !FWD) {
      const __bf16* pre = (const __bf16*)(WHAT == kCombineDQ ? a.pre_q : (o == 0 ? a.pre_k : a.pre_v));
      if (pre) {
        const u32x2 t = *(const u32x2*)(pre + (int64_t)(seq0 + x) * a.s_pre + (int64_t)h * D + 4 * c4);
        acc[0] *= dsilu(__uint_as_float(t[0] << 16)); acc[1] *= dsilu(__uint_as_float(t[0] & 0xFFFF0000u));
        acc[2] *= dsilu(__uint_as_float(t[1] << 16)); acc[3] *= dsilu(__uint_as_float(t[1] & 0xFFFF0000u));
      }
    }
    if constexpr (sizeof(E) == 2) *(u32x2*)dst = (u32x2){pack_bf16x2(acc[0], acc[1]), pack_bf16x2(acc[2], acc[3])};
    else *(f32x4*)dst = acc;
  }
}

// ------------------------------------------------------------------------------------------------
template <typename E, int D, int MODE, int NWAVES, bool DBIAS = false, bool CAND = false>
static hipError_t launch_one(const AttnArgs& a, hipStream_t stream) {
  using C = Cfg<E, D, MODE, NWAVES>;
  auto kern = attn_kernel<E, D, MODE, NWAVES, DBIAS, CAND>;
  constexpr int smem_bytes = C::SMEM_BYTES + (DBIAS ? C::DACC_BYTES : 0);
  static bool attr_set[64] = {};                                         // per instantiation and device
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return hipErrorInvalidDevice;
  if (dev < 0 || dev >= 64 || !attr_set[dev]) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem_bytes);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64) attr_set[dev] = true;
  }
  const int per = kNumXcd * kXcdGroup;
  const int grid = (a.max_items + per - 1) / per * per;
  if (grid == 0) return hipSuccess;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(C::NT), smem_bytes, stream, a);
  return hipGetLastError();
}

template <int MODE, int NW_BF16, int NW_FP32, bool DBIAS = false, bool CAND = false>
static hipError_t dispatch(const AttnArgs& a, int dtype, hipStream_t stream) {
  if (dtype == 0) {
    switch (a.D) {
      case 32: return launch_one<__bf16, 32, MODE, NW_BF16, DBIAS, CAND>(a, stream);
      case 64: return launch_one<__bf16, 64, MODE, NW_BF16, DBIAS, CAND>(a, stream);
      case 128: return launch_one<__bf16, 128, MODE, NW_BF16, DBIAS, CAND>(a, stream);
    }
  } else {
    switch (a.D) {
      case 32: return launch_one<float, 32, MODE, NW_FP32, DBIAS, CAND>(a, stream);
      case 64: return launch_one<float, 64, MODE, NW_FP32, DBIAS, CAND>(a, stream);
      case 128: return launch_one<float, 128, MODE, NW_FP32, DBIAS, CAND>(a, stream);
    }
  }
  return hipErrorInvalidValue;
}

constexpr int kFwdWavesBf16 = 4, kFwdWavesFp32 = 4;
constexpr int kDqWavesBf16 = 4, kDqWavesFp32 = 4;
constexpr int kDkvWavesBf16 = 4, kDkvWavesFp32 = 4;

int fwd_block_rows(int dtype, int) { return 32 * (dtype == 0 ? kFwdWavesBf16 : kFwdWavesFp32); }
int dq_block_rows(int dtype, int) { return 32 * (dtype == 0 ? kDqWavesBf16 : kDqWavesFp32); }
int dkv_block_rows(int dtype, int) { return 32 * (dtype == 0 ? kDkvWavesBf16 : kDkvWavesFp32); }
int stream_tile_rows(int dtype, int) { return dtype == 0 ? 64 : 32; }
int fwd_tile_rows(int dtype, int D) { return dtype == 0 ? (D == 128 ? 32 : 64) : 32; }
int dkv_tile_rows(int dtype, int D) { return dtype == 0 ? (D == 128 ? 32 : 64) : 32; }

hipError_t launch_attn_fwd(const AttnArgs& a, int dtype, hipStream_t stream) {
  // bf16 with 128 features: the pipelined kernel (a forward restricted to a query tail keeps the kernel below, which
  // skips the waves in front of the tail)
  if (dtype == 0 && a.D == 128 && a.seed && a.query_tail == 0) return launch_attn_fwd_pipe(a, stream);
  if (a.num_targets) return dispatch<kFwd, kFwdWavesBf16, kFwdWavesFp32, false, true>(a, dtype, stream);
  return dispatch<kFwd, kFwdWavesBf16, kFwdWavesFp32>(a, dtype, stream);
}
hipError_t launch_attn_bwd_dq(const AttnArgs& a, int dtype, hipStream_t stream) {
  if (a.dbias_dist && a.num_targets) return dispatch<kBwdDQ, kDqWavesBf16, kDqWavesFp32, true, true>(a, dtype, stream);
  if (a.dbias_dist) return dispatch<kBwdDQ, kDqWavesBf16, kDqWavesFp32, true>(a, dtype, stream);
  if (a.num_targets) return dispatch<kBwdDQ, kDqWavesBf16, kDqWavesFp32, false, true>(a, dtype, stream);
  return dispatch<kBwdDQ, kDqWavesBf16, kDqWavesFp32>(a, dtype, stream);
}

// dtable[h, c] = scale * sum of dist[h, x] over the distances x of bucket c (bounds[c] <= x < bounds[c+1], x < len).
// One workgroup per (bucket, head); fixed-order tree reduction.
__global__ __launch_bounds__(256) void dbias_reduce_kernel(const float* __restrict__ dist, const int32_t* __restrict__ bounds,
                                                           int nb, int len, float scale, float* __restrict__ dtable) {
  __shared__ float red[256];
  const int c = blockIdx.x, h = blockIdx.y;
  const int lo = min(bounds[c], len), hi = c + 1 < nb ? min(bounds[c + 1], len) : len;
  float acc = 0.f;
  for (int x = lo + threadIdx.x; x < hi; x += 256) acc += dist[(size_t)h * len + x];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) dtable[(size_t)h * nb + c] = red[0] * scale;
}

__global__ __launch_bounds__(256) void fill_zero_kernel(float* __restrict__ p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = 0.f;
}

hipError_t launch_fill_zero(float* p, size_t n, hipStream_t stream) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)min((n + 255) / 256, (size_t)1024)), dim3(256), 0, stream, p, n);
  return hipGetLastError();
}

hipError_t launch_dbias_reduce(const float* dist, const int32_t* bounds, int num_buckets, int H, int len, float scale,
                               float* dtable, hipStream_t stream) {
  hipLaunchKernelGGL(dbias_reduce_kernel, dim3(num_buckets, H), dim3(256), 0, stream, dist, bounds, num_buckets, len, scale,
                     dtable);
  return hipGetLastError();
}
hipError_t launch_attn_bwd_dkdv(const AttnArgs& a, int dtype, hipStream_t stream) {
  if (a.num_targets) return dispatch<kBwdDKDV, kDkvWavesBf16, kDkvWavesFp32, false, true>(a, dtype, stream);
  return dispatch<kBwdDKDV, kDkvWavesBf16, kDkvWavesFp32>(a, dtype, stream);
}

template <int FWD>
static hipError_t launch_combine(const AttnArgs& a, int dtype, int rows, int max_splits, hipStream_t stream) {
  if (max_splits <= 0) return hipSuccess;
  const dim3 grid(max_splits, 8), block(256);
  if (dtype == 0) {
    switch (a.D) {
      case 32: hipLaunchKernelGGL((combine_kernel<__bf16, 32, FWD>), grid, block, 0, stream, a, rows); break;
      case 64: hipLaunchKernelGGL((combine_kernel<__bf16, 64, FWD>), grid, block, 0, stream, a, rows); break;
      case 128: hipLaunchKernelGGL((combine_kernel<__bf16, 128, FWD>), grid, block, 0, stream, a, rows); break;
      default: return hipErrorInvalidValue;
    }
  } else {
    switch (a.D) {
      case 32: hipLaunchKernelGGL((combine_kernel<float, 32, FWD>), grid, block, 0, stream, a, rows); break;
      case 64: hipLaunchKernelGGL((combine_kernel<float, 64, FWD>), grid, block, 0, stream, a, rows); break;
      case 128: hipLaunchKernelGGL((combine_kernel<float, 128, FWD>), grid, block, 0, stream, a, rows); break;
      default: return hipErrorInvalidValue;
    }
  }
  return hipGetLastError();
}

hipError_t launch_dkdv_combine(const AttnArgs& a, int dtype, int max_splits, hipStream_t stream) {
  return launch_combine<kCombineDKDV>(a, dtype, dkv_block_rows(dtype, a.D), max_splits, stream);
}

hipError_t launch_fwd_combine(const AttnArgs& a, int dtype, int max_splits, hipStream_t stream) {
  return launch_combine<kCombineFwd>(a, dtype, fwd_block_rows(dtype, a.D), max_splits, stream);
}

hipError_t launch_dq_combine(const AttnArgs& a, int dtype, int max_splits, hipStream_t stream) {
  return launch_combine<kCombineDQ>(a, dtype, dq_block_rows(dtype, a.D), max_splits, stream);
}

}  // namespace hstu

#if HSTU_BWD_TIMELINE
// out: 5 * items words per pass (0: dQ pass, 1: dK/dV pass): start, prologue done, loop done, stores done in 10 ns ticks
extern "C" int hstu_debug_bwd_timeline(uint64_t* out, int items, int pass) {
  const int n = items < hstu::kTimelineItems ? items : hstu::kTimelineItems;
  if (n <= 0 || !out || pass < 0 || pass > 1) return 0;
  if (hipDeviceSynchronize() != hipSuccess) return -1;
  if (hipMemcpyFromSymbol(out, HIP_SYMBOL(hstu::g_timeline_bwd), (size_t)n * 5 * sizeof(uint64_t),
                          (size_t)pass * 5 * hstu::kTimelineItems * sizeof(uint64_t), hipMemcpyDeviceToHost) != hipSuccess)
    return -1;
  return n;
}
#endif
