// Forward attention for bf16 with 128 features per head: the tile loop as a software pipeline inside every wave.
//
// Computes what attn_kernel<..., forward, ...> computes (paper Eq. 3 under the masks of Section 4.2.1, same work items, same
// LDS tile format), with the instruction stream arranged for the way a gfx950 SIMD issues.  Measured on the part: a
// matrix instruction hides vector instructions only when they follow it in the SAME wave (a second wave's vector work
// does not overlap with this wave's matrix work), and every instruction a wave issues, scalar ones included, delays its
// next matrix instruction.  So:
//
// 1. Every matrix instruction is followed by its share of the pointwise work of a neighbouring 32-key sub-block:
//      step s, first half  (8 slots):  S(s) += K(s) Q^T, one 16-feature k-step per slot   |  SiLU of keys 16..31 of sub-block s-1
//      step s, second half (8 slots):  O += V(s-1)^T P(s-1), keys 0..15 then 16..31       |  SiLU of keys 0..15 of sub-block s
//    P(s-1) is complete exactly when its second product starts; a slot carries one matrix instruction, one SiLU (exp2,
//    add, rcp, mul) per lane and half a bf16 packing, the SiLU as a rolling pipeline over the slots so that nothing waits
//    for the transcendental in front of it.
// 2. The mask costs nothing in the loop: the score accumulators are SEEDED with a function of the distance
//    position - key (AttnArgs::seed): the relative bias where the key is visible, -1e30 where it is not (later keys;
//    keys beyond the local band).  Such a score stays at -1e30 through the product, exp2(1e30) = inf, rcp(inf) = 0 and
//    t * 0 = -0 enters the second product: exactly no contribution.  Rows and keys past the end of the sequence need no
//    mask at all (their Q, K, V rows read as zero).  Only the few sub-blocks whose mask is not a function of the
//    distance (keys on both sides of the end of the global prefix; candidate keys) are patched element by element,
//    and those are moved to the end of the item's list and run in a second copy of the loop.
// 3. K, V and the seed strip sit in two-stage rings in LDS, filled by direct-to-LDS loads that are issued a whole
//    half-step before the barrier that publishes them:
//      first half of step s:  loads V(s);               at its end: K(s+1), strip(s+1) have landed -> barrier
//      second half of step s: loads K(s+2), strip(s+2); at its end: V(s) has landed                -> barrier
//    Fragments for the first slots after a barrier are read before it (they belong to tiles published one barrier
//    earlier), and the descriptors of a sub-block are built once, on the scalar unit.
#include <type_traits>

#include "hstu_common.h"
#include "hstu_kernels.h"

namespace hstu {
namespace {

constexpr int kBX = 128, kBN = 32, kWaves = 4, kThreads = 64 * kWaves, kD = 128;
constexpr int kTile = kBN * 256;                                       // one 32-row tile of 256-byte rows
// Seed strip of one (block, sub-block): the kBX + kBN - 1 distances a sub-block needs, in 4 copies shifted by one entry so
// that a lane fetches 4 consecutive entries with one aligned 16-byte read.  Wave c loads copy c with one 16-byte-per-lane
// load (entries 4 l .. 4 l + 3 from lane l; the seed table is stored by descending distance for this).  Copies are 1088
// bytes apart: 1 KB that the load fills plus 64 bytes that put the 16 reads of a quarter-wave on 16 different bank groups.
constexpr int kStripCopy = 1088, kStripBytes = 4 * kStripCopy;
constexpr int kKBase = 0, kVBase = 2 * kTile, kStripBase = 4 * kTile;
// The last kQLds of the 8 Q fragments of a lane wait in LDS (16 bytes per lane and fragment) instead of in registers: that
// is what lets three workgroups share a compute unit (168 registers per lane).
constexpr int kQLds = 2;
constexpr int kQBase = kStripBase + 2 * kStripBytes;
constexpr int kSmemBytes = kQBase + kQLds * kThreads * 16;
#ifndef HSTU_FP_PF
#define HSTU_FP_PF 1
#endif
constexpr int kPF = HSTU_FP_PF;                                         // slots between a fragment's LDS read and its product
constexpr float kLog2e = 1.4426950408889634f, kLn2 = 0.6931471805599453f;
constexpr float kMasked = -1e30f;
constexpr int kNoTile = 1 << 28;
// Measurement builds only (results are wrong): HSTU_FWD_ABLATE is a bit mask of parts of the tile loop to leave out, to
// see what each costs in time and in the clock the chip sustains.  1: the global -> LDS loads of the loop; 2: the two
// transcendentals of SiLU; 4: the LDS reads of K / V fragments and seeds (16 / 32 / 64: those of K / of V / of the seeds
// alone); 8: the matrix instructions; 128: the K fragments are read but a constant register goes into the product in
// their place (the reads stay, the operand stops changing); 256: four neighbouring blocks stream the same K and V tiles
// (those of the first of the four), which is what perfect sharing of a semi-local window in the L2 would look like.  Every memory access an ablated build still makes is one
// the normal build makes.
#ifndef HSTU_FWD_ABLATE
#define HSTU_FWD_ABLATE 0
#endif
constexpr bool kNoDma = HSTU_FWD_ABLATE & 1, kNoSilu = HSTU_FWD_ABLATE & 2, kNoMfma = HSTU_FWD_ABLATE & 8;
constexpr bool kNoLdsK = HSTU_FWD_ABLATE & (4 | 16), kNoLdsV = HSTU_FWD_ABLATE & (4 | 32), kNoLdsSeed = HSTU_FWD_ABLATE & (4 | 64);
template <class T> __device__ __forceinline__ T undefined_value() { T v; asm volatile("" : "=v"(v)); return v; }
__device__ __forceinline__ f32x16 mfma(bf16x8 x, bf16x8 y, f32x16 acc) {
  if constexpr (kNoMfma) { asm volatile("" :: "v"(x), "v"(y)); return acc; }
  else return __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, acc, 0, 0, 0);
}

// Measurement builds only: with HSTU_FWD_TIMELINE defined non-zero, the first lane of every workgroup records the 100 MHz
// wall clock at its start, after the prologue's barrier, after the tile loop and after its stores, and the compute unit it
// ran on; hstu_debug_fwd_timeline() copies the records of the last launch out (5 words per work item, in list order).
#ifndef HSTU_FWD_TIMELINE
#define HSTU_FWD_TIMELINE 0
#endif
#if HSTU_FWD_TIMELINE
constexpr int kTimelineItems = 16384;
__device__ uint64_t g_timeline[5 * kTimelineItems];
#define HSTU_TL(k) do { if (threadIdx.x == 0 && pos < kTimelineItems) g_timeline[5 * pos + (k)] = wall_clock64(); } while (0)
#else
#define HSTU_TL(k) do { } while (0)
#endif

typedef __attribute__((address_space(3))) void* lds_void;
typedef __attribute__((address_space(3))) short4v* lds_s4;
typedef __attribute__((address_space(3))) const bf16x8* lds_b8;
typedef __attribute__((address_space(3))) const f32x4* lds_f4;

template <int N> using IC = std::integral_constant<int, N>;

template <bool CAND>
__global__ __launch_bounds__(kThreads, 3) void attn_fwd_pipe_kernel(const AttnArgs a) {
  extern __shared__ __attribute__((aligned(256))) unsigned char smem[];
  const int wg = blockIdx.x;
  const int xcd = wg % kNumXcd, slot_id = wg / kNumXcd;
  const int pos = ((slot_id / kXcdGroup) * kNumXcd + xcd) * kXcdGroup + slot_id % kXcdGroup;
  const int count = a.header->count;                                   // (fetched together with the entry, which is dropped if beyond)
  const WorkItem item = a.items[min(pos, a.max_items - 1)];
  if (pos >= count) return;
  HSTU_TL(0);
#if HSTU_FWD_TIMELINE
  if (threadIdx.x == 0 && pos < kTimelineItems) {
    uint32_t hw;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw));
    uint32_t xcc;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
    g_timeline[5 * pos + 4] = ((uint64_t)xcc << 32) | hw;
  }
#endif
  const int xb = item.rb_h >> 8, h = item.rb_h & 255;
  const int seq0 = item.seq0;
  const int L = item.len;
  const SeqGeom g = {L, item.hist, a.K1, a.K2};

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int hf = lane >> 5, l32 = lane & 31, grp16 = lane >> 4, i16 = lane & 15;
  const int x0 = xb * kBX, xw0 = x0 + wave * 32, x = xw0 + l32;
  const bool x_ok = x < L;
  const int q0 = a.query_tail > 0 ? max(g.n - a.query_tail, 0) : 0;    // rows before q0 are not written

  const int64_t hoff = (int64_t)h * kD;
  const __bf16* Qp = (const __bf16*)a.q + seq0 * a.sq + hoff;
  const __bf16* Kp = (const __bf16*)a.k + seq0 * a.sk + hoff;
  const __bf16* Vp = (const __bf16*)a.v + seq0 * a.sv + hoff;

  // ---- this lane's query row as B operands of the score product, times alpha log2 e (scores in units of ln 2)
  const float score_scale = kLog2e * a.alpha;
  bf16x8 qf[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    u32x4 raw = {0u, 0u, 0u, 0u};
    if (x_ok) raw = *(const u32x4*)(Qp + (int64_t)x * a.sq + ks * 16 + hf * 8);
    qf[ks] = __builtin_bit_cast(bf16x8, raw);
  }
  typedef __attribute__((address_space(3))) bf16x8* lds_b8w;
  const int qaddr = (int)(uint32_t)(uintptr_t)(lds_void)smem + kQBase + tid * 16;
  // (first use in the prologue, after the first sub-blocks' loads are issued: the two round trips to memory overlap)
  auto finish_q = [&]() {
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      u32x4 raw = __builtin_bit_cast(u32x4, qf[ks]);
#pragma unroll
      for (int w = 0; w < 4; ++w)
        raw[w] = pack_bf16x2(__builtin_bit_cast(float, raw[w] << 16) * score_scale,
                             __builtin_bit_cast(float, raw[w] & 0xFFFF0000u) * score_scale);
      qf[ks] = __builtin_bit_cast(bf16x8, raw);
    }
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) asm volatile("" : "+v"(qf[ks]));    // landed before the loop: nothing in it may wait on them
#pragma unroll
    for (int i = 0; i < kQLds; ++i) *(lds_b8w)(uintptr_t)(uint32_t)(qaddr + i * kThreads * 16) = qf[8 - kQLds + i];
  };

  f32x16 out[4];
#pragma unroll
  for (int ob = 0; ob < 4; ++ob)
#pragma unroll
    for (int r = 0; r < 16; ++r) out[ob][r] = 0.f;

  // ---- the item's sub-blocks: positions [t_begin, t_end) of the block's ascending tile list, reordered so that the
  // sub-blocks whose mask needs patching come last: those with candidate keys (a suffix of the list) and the one that
  // holds the end of the global prefix when that is not a multiple of 32.
  const int xlast = min(x0 + kBX, L) - 1;
  const TileRanges tr = tile_ranges(g, x0, xlast, kBN);
  const int t_begin = item.t0, t_end = max(min(tr.count(), item.t1), item.t0);
  const int n = t_end - t_begin;
  const int na = tr.a1 - tr.a0, nb = tr.b1 - tr.b0, nc = tr.c1 - tr.c0;
  const int cand_t0 = (CAND && g.n < L) ? g.n / kBN : kNoTile;         // first tile with a candidate key
  const int pc = min(max(cand_t0 - tr.a0, 0), na) + min(max(cand_t0 - tr.b0, 0), nb) + min(max(cand_t0 - tr.c0, 0), nc);
  const int suf0 = min(max(pc, t_begin), t_end);                        // the special suffix is [suf0, t_end)
  const int straddle_t = (g.K1 >= 0 && (g.K2 % kBN) != 0) ? g.K2 / kBN : -1;
  const int ps_raw = straddle_t - tr.a0;                                // its position, if it is on the list
  const bool has_ps = straddle_t >= tr.a0 && straddle_t < tr.a1 && ps_raw >= t_begin && ps_raw < suf0;
  const int ps = has_ps ? ps_raw : kNoTile;
  const int nfast = (suf0 - t_begin) - (has_ps ? 1 : 0);
  // (measurement build 256: the block streams the tiles of the first block of its aligned group of four)
  const int x0m = (xb & ~3) * kBX;
  const int mshift = tr.b0 - tile_ranges(g, x0m, min(x0m + kBX, L) - 1, kBN).b0;
  auto tile_of = [&](int idx) -> int {                                  // idx-th sub-block of the reordered list
    int p;
    if (idx < nfast) { p = t_begin + idx; p += (p >= ps) ? 1 : 0; }
    else { const int j = idx - nfast; p = (suf0 + j < t_end) ? suf0 + j : ps_raw; }
    if constexpr ((HSTU_FWD_ABLATE & 256) != 0) { const int yt = tr.at(p); return yt >= tr.b0 ? yt - mshift : yt; }
    return tr.at(p);
  };

  const int px = CAND ? min(x, g.n) : x;                               // a candidate row stands at position n
  const int x0v = CAND ? min(x0, g.n) : x0;
  const int strip_s0 = kBX - 1 - (px - x0v) + 4 * hf;
  const float* seed_h = a.seed + (int64_t)h * a.seed_len;               // variant 0; variant 1 is H * seed_len further
  const uint32_t seed_bytes = (uint32_t)a.seed_len * 4u;
  const int64_t seed_var1 = (int64_t)a.H * a.seed_len;
  const float bias0 = CAND ? seed_h[a.seed_dmax] : 0.f;                 // seed of distance 0: a candidate's own key

  // ---- global -> LDS: raw buffer loads with the LDS destination in M0 (lane l lands at M0 + 16 l)
  const uint32_t rowbK = (uint32_t)(a.sk * 2), rowbV = (uint32_t)(a.sv * 2);
  const int dma_chunk = (lane & 15) ^ (4 * (lane >> 4) + (wave & 3));
  uint32_t voffK = __umul24((uint32_t)(lane >> 4), rowbK) + (uint32_t)(dma_chunk * 16);
  uint32_t voffV = __umul24((uint32_t)(lane >> 4), rowbV) + (uint32_t)(dma_chunk * 16);
  // the second 4-row group of a wave (16 rows further down) uses the same descriptor with a lane offset 16 rows larger
  uint32_t voffK1 = voffK + 16u * rowbK, voffV1 = voffV + 16u * rowbV;
  uint32_t voffS = 16u * (uint32_t)lane + 4u * (uint32_t)wave;           // this wave loads copy `wave` of the strip
  asm volatile("" : "+v"(voffK), "+v"(voffV), "+v"(voffK1), "+v"(voffV1), "+v"(voffS));
  // (every word goes through readfirstlane: the descriptor of a load must sit in scalar registers, and the compiler is
  // otherwise free to assemble a uniform 128-bit value in vector registers; on a scalar input it is a plain copy)
  auto make_rsrc = [&](uint64_t addr, uint32_t bytes) -> i32x4 {
    return (i32x4){__builtin_amdgcn_readfirstlane((int)(uint32_t)addr), __builtin_amdgcn_readfirstlane((int)(uint32_t)(addr >> 32)),
                   __builtin_amdgcn_readfirstlane((int)bytes), 0x00020000};
  };
  // (M0 = a per-wave base + a constant: one scalar instruction; one idle cycle between the write of M0 and its use)
  const uint32_t smem_base = (uint32_t)(uintptr_t)(lds_void)smem;
  const uint32_t m0_rows = smem_base + (uint32_t)wave * 1024u;
  const uint32_t m0_strip = smem_base + (uint32_t)kStripBase + (uint32_t)wave * (uint32_t)kStripCopy;
  auto dma16 = [&](i32x4 rs, uint32_t voff, uint32_t m0_base, uint32_t dst_off) {
    asm volatile("s_add_u32 m0, %0, %1\n\ts_nop 0\n\tbuffer_load_dwordx4 %2, %3, 0 offen lds"
                 :: "s"(m0_base), "s"(dst_off), "v"(voff), "s"(rs) : "memory", "m0", "scc");
  };
  // Where sub-block idx of the list sits, as scalars computed once: descriptors of this wave's rows of K and of V (the
  // tile's rows from 4 * wave on, range = what is left of the sequence: rows past its end read as zero), the seed
  // table that applies (band tiles of a semi-local mask: the one that also masks by distance) and the strip origin.
  // A sub-block beyond the list gets empty ranges: its loads are still issued (the waits count loads), read zeros and
  // land in stages whose products then contribute nothing (score 0, SiLU(0) = 0).
  struct Rows { uint64_t addr; int left; };                             // a wave's rows of one tile: first row, rows left in the sequence (<= 0: none)
  struct Src { Rows k, v; uint64_t seed; uint32_t seed_bytes, s_off; int yt; };
  auto src_of = [&](int idx) -> Src {
    const bool valid = idx < n;
    const int yt = valid ? tile_of(idx) : 0;
    const int yrow = yt * kBN + 4 * wave;
    const int left = valid ? L - yrow : 0;
    const bool band = g.K1 >= 0 && yt >= tr.b0 && yt < tr.b1;
    Src r;
    r.k = {(uint64_t)(uintptr_t)Kp + (uint64_t)(uint32_t)yrow * rowbK, left};
    r.v = {(uint64_t)(uintptr_t)Vp + (uint64_t)(uint32_t)yrow * rowbV, left};
    r.seed = (uint64_t)(uintptr_t)(seed_h + (band ? seed_var1 : 0));
    r.seed_bytes = valid ? seed_bytes : 0u;
    // strip index s <-> distance d0 - s, d0 = x0v + kBX - 1 - yt * kBN  <->  table index seed_dmax - d0 + s
    r.s_off = 4u * (uint32_t)(a.seed_dmax - (x0v + (kBX - 1) - yt * kBN));
    r.yt = valid ? yt : kNoTile;
    return r;
  };
  // The sub-block after `prev` (list index idx): nearly always the next tile of the same sequence, whose descriptors are
  // a few scalar additions away (one 32-row tile further down, 32 distances closer); anything else is built from scratch.
  const uint32_t stepK = 32u * rowbK, stepV = 32u * rowbV;
  auto next_src = [&](const Src& prev, int idx) -> Src {
    const int yt = idx < n ? tile_of(idx) : kNoTile;
    if (__builtin_expect(yt != prev.yt + 1 || (g.K1 >= 0 && yt == tr.b0), 0)) return src_of(idx);
    Src r = prev;
    r.k.addr = prev.k.addr + stepK; r.k.left = prev.k.left - kBN;
    r.v.addr = prev.v.addr + stepV; r.v.left = prev.v.left - kBN;
    r.s_off = prev.s_off + 4u * kBN;
    r.yt = yt;
    return r;
  };
  // piece c (0, 1): the 4-row group 4 c + wave of the tile
  auto load_k = [&](const Src& sr, int stage, int c) { dma16(make_rsrc(sr.k.addr, (uint32_t)max(sr.k.left, 0) * rowbK), c ? voffK1 : voffK, m0_rows, (uint32_t)(kKBase + stage * kTile + 4096 * c)); };
  auto load_vd = [&](const Rows& vd, int stage, int c) { dma16(make_rsrc(vd.addr, (uint32_t)max(vd.left, 0) * rowbV), c ? voffV1 : voffV, m0_rows, (uint32_t)(kVBase + stage * kTile + 4096 * c)); };
  auto load_v = [&](const Src& sr, int stage, int c) { load_vd(sr.v, stage, c); };
  auto load_strip = [&](const Src& sr, int stage) { dma16(make_rsrc(sr.seed, sr.seed_bytes), voffS + sr.s_off, m0_strip, (uint32_t)(stage * kStripBytes)); };

  // ---- LDS fragment addresses of stage 0 (the stage and the position inside the tile are immediate offsets).
  // Row r stores its logical 16-byte chunk c at chunk c ^ (4 (r % 4) + (r / 4) % 4).
  const int zl = 4 * (l32 & 3) + ((l32 >> 2) & 3);
  const int kb = (int)smem_base + kKBase + l32 * 256 + ((hf ^ (zl & 1)) << 4) + ((zl >> 1) << 5);
  const int vchunk = 2 * (grp16 & 1) + ((i16 & 3) >> 1), vbyte = 8 * (i16 & 1);
  const int tb = (int)smem_base + kVBase + (4 * hf + (i16 >> 2)) * 256 + ((i16 >> 2) << 6) + ((vchunk ^ hf) << 4) + vbyte;
  int kaddr[8], vaddr[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    kaddr[i] = kb ^ (i << 5);                                          // k-step i of a score product
    vaddr[i] = tb ^ (((i >> 1) << 6) | ((i & 1) << 5));                // feature block i / 2, rows +0 (i even) or +8 (i odd)
    asm volatile("" : "+v"(kaddr[i]), "+v"(vaddr[i]));
  }
  const int saddr = (int)smem_base + kStripBase + (strip_s0 & 3) * kStripCopy + (strip_s0 & ~3) * 4;
  auto kfrag = [&](int stage, int ks) -> bf16x8 {
    if constexpr (kNoLdsK) return undefined_value<bf16x8>();
    if constexpr ((HSTU_FWD_ABLATE & 128) != 0) {
      const bf16x8 f = *(lds_b8)(uintptr_t)(uint32_t)(kaddr[ks] + stage * kTile);
      asm volatile("" :: "v"(f));
      return undefined_value<bf16x8>();
    }
    return *(lds_b8)(uintptr_t)(uint32_t)(kaddr[ks] + stage * kTile);
  };
  // A operand of an output product: features 32 ob .. 32 ob + 31 (rows) x keys 16 ks2 + 4 hf + {0..3}, + 8 + {0..3}
  auto vfrag = [&](int stage, int ks2, int ob) -> bf16x8 {
    if constexpr (kNoLdsV) return undefined_value<bf16x8>();
    const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(uintptr_t)(uint32_t)(vaddr[2 * ob] + stage * kTile + ks2 * 4096));
    const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(uintptr_t)(uint32_t)(vaddr[2 * ob + 1] + stage * kTile + ks2 * 4096 + 2048));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  };

  // Patch of the seeds of a sub-block whose mask is not a function of the distance: element by element, with per-lane
  // bounds on c = key - y0 - 4 hf (a compile-time constant per score register):
  //   visible <=> (c <= up && (c >= lo || c < pre)) || c == selfc
  auto mask_seed = [&](f32x16& acc, int yt) {
    const int y0 = yt * kBN + 4 * hf;
    const int up = x_ok ? min(px, g.n - 1) - y0 : -1;                  // history keys up to the row's position
    const int lo = g.K1 < 0 ? -(1 << 28) : px - g.K1 + 1 - y0;         // inside the local band
    const int pre = g.K2 - y0;                                         // inside the global prefix
    const int selfc = (CAND && x_ok && x >= g.n) ? x - y0 : -1000;     // a candidate sees itself, at distance 0
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int c = 8 * (r >> 2) + (r & 3);
      const bool vis = c <= up && (c >= lo || c < pre);
      float t = vis ? acc[r] : kMasked;
      if (CAND) t = (c == selfc) ? bias0 : t;
      acc[r] = t;
    }
  };

  // ---- pipeline state
  f32x16 sacc[2];
  uint32_t plo[2][4], phi[4];
  bf16x8 kfn[kPF];                                                      // K fragments of the first kPF slots of the next step
  // seeds the score accumulators of a sub-block from its strip
  auto seed = [&](f32x16& acc, int stage) {
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const f32x4 bv = kNoLdsSeed ? undefined_value<f32x4>() : *(lds_f4)(uintptr_t)(uint32_t)(saddr + stage * kStripBytes + 32 * q4);
      acc[4 * q4 + 0] = bv[0]; acc[4 * q4 + 1] = bv[1]; acc[4 * q4 + 2] = bv[2]; acc[4 * q4 + 3] = bv[3];
    }
  };

  // ---- prologue: K and strip of sub-blocks 0 and 1.  src0 / src1 describe the sub-blocks s and s + 1 of the coming step.
  // Carried from step to step: `cur` describes the newest sub-block whose K and strip loads were issued (s + 1 when step
  // s starts); of the two before it only the V descriptors (their V loads are issued two steps after their K loads).
  Src cur = src_of(0);
  Rows vdesc0 = cur.v, vdesc1;                                         // V of sub-blocks s and s + 1
  const int yt_first = cur.yt;
  load_k(cur, 0, 0); load_k(cur, 0, 1); load_strip(cur, 0);
  cur = next_src(cur, 1);
  vdesc1 = cur.v;
  load_k(cur, 1, 0); load_k(cur, 1, 1); load_strip(cur, 1);
  {                                                                     // V stage 1 is read by step 0 ("sub-block -1"): zeros
    const Src none = src_of(n);
    load_v(none, 1, 0); load_v(none, 1, 1);
  }
  finish_q();
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  HSTU_TL(1);
#pragma unroll
  for (int i = 0; i < kPF; ++i) kfn[i] = kfrag(0, i);
  seed(sacc[0], 0);
  if (nfast == 0 && n > 0) mask_seed(sacc[0], yt_first);
#pragma unroll
  for (int r = 0; r < 16; ++r) sacc[1][r] = kMasked;                    // "sub-block -1": contributes nothing
#pragma unroll
  for (int i = 0; i < 4; ++i) { plo[0][i] = plo[1][i] = 0u; phi[i] = 0u; }

  // The SiLU of consecutive scores as a rolling pipeline: a slot starts the new score (exp2, add, rcp) and finishes the
  // previous one (its multiply, and the bf16 packing of every second one), so that no instruction needs the result of
  // the transcendental right in front of it.  Returns the finished previous score.
  float st_t = kMasked, st_r = 0.f, st_p = 0.f;
  auto silu_roll = [&](float t) -> float {
    const float e = kNoSilu ? -t : __builtin_amdgcn_exp2f(-t);
    const float pp = st_t * st_r;
    const float r = kNoSilu ? 1.0f + e : __builtin_amdgcn_rcpf(1.0f + e);
    st_t = t; st_r = r;
    asm volatile("" : "+v"(st_r));                                       // the pointwise work stays in its slot
    return pp;
  };

  // One step: sub-block s enters (score product, SiLU of its first 16 keys), sub-block s - 1 leaves (SiLU of its last 16
  // keys, output product).  P = parity of s.  PATCH: sub-block s + 1, seeded in this step, may need its mask patched.
  auto step = [&](int s, auto par_c, auto patch_c) {
    constexpr int P = decltype(par_c)::value;
    constexpr bool PATCH = decltype(patch_c)::value;
    // ---------------- first half: S(s) products, SiLU of keys 16..31 of s - 1
    bf16x8 kf[kPF + 1], vf[kPF + 1];                                    // fragments are fetched kPF slots ahead of their product
    bf16x8 qx[kQLds];
#pragma unroll
    for (int i = 0; i < kPF; ++i) kf[i] = kfn[i];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (i < 2 && !kNoDma) load_vd(vdesc0, P, i);
      if (i >= 8 - kQLds - 2 && i < 8 - 2) qx[i - (8 - kQLds - 2)] = *(lds_b8)(uintptr_t)(uint32_t)(qaddr + (i - (8 - kQLds - 2)) * kThreads * 16);
      if (i + kPF < 8) kf[(i + kPF) % (kPF + 1)] = kfrag(P, i + kPF);
      else vf[(i + kPF - 8) % (kPF + 1)] = vfrag(P ^ 1, (i + kPF - 8) >> 2, (i + kPF - 8) & 3);
      __builtin_amdgcn_sched_barrier(0);
      sacc[P] = mfma(kf[i % (kPF + 1)], i < 8 - kQLds ? qf[i] : qx[i - (8 - kQLds)], sacc[P]);
      __builtin_amdgcn_sched_barrier(0);
      {
        const float pp = silu_roll(sacc[P ^ 1][8 + i]);                 // finishes the previous score (keys 16.. of s - 1, or key 15 of its first half)
        if (i == 0) { plo[P ^ 1][3] = pack_bf16x2(st_p, pp); asm volatile("" : "+v"(plo[P ^ 1][3])); }
        else if (i & 1) st_p = pp;
        else { phi[(i - 1) >> 1] = pack_bf16x2(st_p, pp); asm volatile("" : "+v"(phi[(i - 1) >> 1])); }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    asm volatile("s_waitcnt vmcnt(2)" ::: "memory");                    // K(s+1), strip(s+1) landed (V(s) may still fly)
    __syncthreads();

    // ---------------- second half: O += V(s-1)^T P(s-1), SiLU of keys 0..15 of s
    const int yt_seed = cur.yt;                                         // sub-block s + 1, seeded in this half
    cur = next_src(cur, s + 2);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if (j == 4) {                                                     // (the last 8 scores of s - 1 went into P in the first half)
        seed(sacc[P ^ 1], P ^ 1);
        if (PATCH) { if (s + 1 >= nfast && s + 1 < n) mask_seed(sacc[P ^ 1], yt_seed); }
      }
      if (j < 2 && !kNoDma) load_k(cur, P, j);
      else if (j == 2 && !kNoDma) load_strip(cur, P);
      if (j + kPF < 8) vf[(j + kPF) % (kPF + 1)] = vfrag(P ^ 1, (j + kPF) >> 2, (j + kPF) & 3);
      else kfn[j + kPF - 8] = kfrag(P ^ 1, j + kPF - 8);
      __builtin_amdgcn_sched_barrier(0);
      {
        const uint32_t* pk = (j < 4) ? plo[P ^ 1] : phi;
        const bf16x8 pb = __builtin_bit_cast(bf16x8, (u32x4){pk[0], pk[1], pk[2], pk[3]});
        out[j & 3] = mfma(vf[j % (kPF + 1)], pb, out[j & 3]);
      }
      __builtin_amdgcn_sched_barrier(0);
      {
        const float pp = silu_roll(sacc[P][j]);
        if (j == 0) { phi[3] = pack_bf16x2(st_p, pp); asm volatile("" : "+v"(phi[3])); }
        else if (j & 1) st_p = pp;
        else { plo[P][(j - 1) >> 1] = pack_bf16x2(st_p, pp); asm volatile("" : "+v"(plo[P][(j - 1) >> 1])); }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    asm volatile("s_waitcnt vmcnt(3)" ::: "memory");                    // V(s) landed (only the 3 loads of this half may still fly)
    __syncthreads();
    vdesc0 = vdesc1; vdesc1 = cur.v;
  };

  // steps whose seeded sub-block needs no patch, in pairs; then the rest (patched sub-blocks and the two draining steps)
  int s = 0;
  for (; s + 2 < nfast; s += 2) {
    step(s, IC<0>{}, std::false_type{});
    step(s + 1, IC<1>{}, std::false_type{});
  }
  for (; s <= n; s += 2) {
    step(s, IC<0>{}, std::true_type{});
    if (s + 1 > n) break;
    step(s + 1, IC<1>{}, std::true_type{});
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                      // nothing may still be landing in LDS when the wave ends
  HSTU_TL(2);

  // ---- epilogue.  Lane x holds features 32 ob + 8 (r / 4) + 4 hf + r % 4.
  if (item.slot >= 0) {                                                 // a piece of a cut block: raw sums, the combine kernel finishes
    float* dst = a.partial + ((int64_t)item.slot * kBX + (wave * 32 + l32)) * kD;
#pragma unroll
    for (int ob = 0; ob < 4; ++ob)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4)
        *(f32x4*)(dst + ob * 32 + 8 * q4 + 4 * hf) =
            (f32x4){out[ob][4 * q4 + 0], out[ob][4 * q4 + 1], out[ob][4 * q4 + 2], out[ob][4 * q4 + 3]};
    HSTU_TL(3);
    return;
  }
  if (!x_ok || x < q0) { HSTU_TL(3); return; }
  const float scale = a.inv_n * kLn2;
  __bf16* dst = (__bf16*)a.out + (int64_t)(seq0 + x) * a.so + hoff;
#pragma unroll
  for (int ob = 0; ob < 4; ++ob)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const int f = ob * 32 + 8 * q4 + 4 * hf;
      *(u32x2*)(dst + f) = (u32x2){pack_bf16x2(out[ob][4 * q4 + 0] * scale, out[ob][4 * q4 + 1] * scale),
                                    pack_bf16x2(out[ob][4 * q4 + 2] * scale, out[ob][4 * q4 + 3] * scale)};
    }
#if HSTU_FWD_TIMELINE
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  HSTU_TL(3);
#endif
}

}  // namespace

hipError_t launch_attn_fwd_pipe(const AttnArgs& a, hipStream_t stream) {
  const int per = kNumXcd * kXcdGroup;
  const int grid = (a.max_items + per - 1) / per * per;
  if (grid == 0) return hipSuccess;
  if (!a.seed) return hipErrorInvalidValue;
  const dim3 gd(grid), bd(kThreads);
  if (a.num_targets) hipLaunchKernelGGL((attn_fwd_pipe_kernel<true>), gd, bd, kSmemBytes, stream, a);
  else hipLaunchKernelGGL((attn_fwd_pipe_kernel<false>), gd, bd, kSmemBytes, stream, a);
  return hipGetLastError();
}

}  // namespace hstu

#if HSTU_FWD_TIMELINE
// out: 5 * items words (start, prologue done, loop done, stores done in 10 ns ticks; hardware id); returns the number of items copied
extern "C" int hstu_debug_fwd_timeline(uint64_t* out, int items) {
  const int n = items < hstu::kTimelineItems ? items : hstu::kTimelineItems;
  if (n <= 0 || !out) return 0;
  if (hipDeviceSynchronize() != hipSuccess) return -1;
  if (hipMemcpyFromSymbol(out, HIP_SYMBOL(hstu::g_timeline), (size_t)n * 5 * sizeof(uint64_t), 0, hipMemcpyDeviceToHost) != hipSuccess) return -1;
  return n;
}
#endif
