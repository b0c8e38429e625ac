// C-ABI entry points of the jagged HSTU attention library: argument validation, workspace
// layout and kernel launches.  Declarations and the meaning of every argument: include/hstu_attn.h.
#include "../../include/hstu_attn.h"
#include "hstu_common.h"
#include "hstu_kernels.h"
#include "profile.h"

#include <mutex>

using namespace hstu;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Upper bound of the schedule length: every sequence adds at most one ragged block.
inline int64_t max_items_for(const hstu_attn_params* p, int block_rows) {
  return ((int64_t)p->total_tokens / block_rows + p->batch) * p->num_heads;
}

struct Layout {           // byte offsets inside a workspace
  size_t header[2], items[2], seq_base[2], bias, seed, splits, partial, splits_dq, partial_dq, dbias, total;
  int max_items[2];
  int slot_cap;           // partial-sum slots of the dK/dV pass (key blocks cut along the query axis) or of the forward
  int slot_cap_dq;        // ... of the dQ pass (query blocks of a small batch cut along the key axis)
};

// Slots for the pieces of cut key blocks: at most 768 (about 1.5 per workgroup slot of the chip), never more than
// twice the number of key blocks, none without a mask that can make a key block long (dense causal and local-only
// masks never have one block much longer than the rest of its sequence... they may still be cut when sequences differ
// a lot in length, which the same bound covers).
inline int slot_cap_for(int max_items) { return max_items < 384 ? 2 * max_items : 768; }

// One schedule for the forward; two (dQ pass, dK/dV pass) for the backward.
Layout make_layout(const hstu_attn_params* p, int for_backward) {
  Layout l = {};
  size_t off = 0;
  const int nsched = for_backward ? 2 : 1;
  for (int s = 0; s < nsched; ++s) {
    const int rows = !for_backward ? fwd_block_rows(p->dtype, p->head_dim)
                                   : (s == 0 ? dq_block_rows(p->dtype, p->head_dim) : dkv_block_rows(p->dtype, p->head_dim));
    l.max_items[s] = (int)max_items_for(p, rows);
    // the dK/dV list also holds the pieces of cut key blocks; so does the forward list (query blocks longer than a
    // workgroup slot's share of the batch, or the few blocks of a query tail against long histories: their key axis is cut)
    if ((for_backward && s == 1) || !for_backward) {
      l.slot_cap = slot_cap_for(l.max_items[s]);
      l.max_items[s] += l.slot_cap;
    } else {
      l.slot_cap_dq = slot_cap_for(l.max_items[s]);
      l.max_items[s] += l.slot_cap_dq;
    }
    l.header[s] = off; off += kAlign;
    l.items[s] = off; off += align_up((size_t)l.max_items[s] * sizeof(WorkItem));
    l.seq_base[s] = off; off += align_up(((size_t)p->batch + 1) * sizeof(int32_t));
  }
  l.bias = off;
  off += align_up((size_t)p->num_heads * ((size_t)p->max_seqlen + 1) * sizeof(float));
  l.seed = off;                                        // score seeds by distance (bias + mask) of the pipelined kernels
  off += align_up((size_t)kSeedVariants * p->num_heads * (size_t)seed_len_for(p->max_seqlen) * sizeof(float));
  if (!for_backward) {
    l.splits = off; off += align_up((size_t)(l.slot_cap / 2 + 1) * sizeof(SplitItem));
    l.partial = off;
    off += align_up((size_t)l.slot_cap * fwd_block_rows(p->dtype, p->head_dim) * p->head_dim * sizeof(float));
  }
  if (for_backward) {
    l.splits = off; off += align_up((size_t)(l.slot_cap / 2 + 1) * sizeof(SplitItem));
    l.partial = off;
    off += align_up((size_t)l.slot_cap * 2 * dkv_block_rows(p->dtype, p->head_dim) * p->head_dim * sizeof(float));
    l.splits_dq = off; off += align_up((size_t)(l.slot_cap_dq / 2 + 1) * sizeof(SplitItem));
    l.partial_dq = off;
    off += align_up((size_t)l.slot_cap_dq * dq_block_rows(p->dtype, p->head_dim) * p->head_dim * sizeof(float));
    l.dbias = off;                                     // per-distance sums of dS for the bias-table gradient, then the bucket ends per distance
    off += align_up((size_t)(p->num_heads + 1) * ((size_t)p->max_seqlen + 1) * sizeof(float));
  }
  l.total = off;
  return l;
}

int validate(const hstu_attn_params* p) {
  if (!p) return HSTU_ERR_NULL;
  if (p->batch < 0 || p->total_tokens < 0 || p->max_seqlen < 0 || p->num_heads < 1 || p->num_heads > 256) return HSTU_ERR_SHAPE;
  if (p->dtype != HSTU_BF16 && p->dtype != HSTU_FP32) return HSTU_ERR_UNSUPPORTED;
  if (p->head_dim != 32 && p->head_dim != 64 && p->head_dim != 128) return HSTU_ERR_UNSUPPORTED;
  const int64_t hd = (int64_t)p->num_heads * p->head_dim;
  const int64_t quantum = p->dtype == HSTU_BF16 ? 8 : 4;     // rows must start on 16-byte boundaries
  const int64_t strides[4] = {p->row_stride_q, p->row_stride_k, p->row_stride_v, p->row_stride_o};
  for (int i = 0; i < 4; ++i)
    if (strides[i] < hd || strides[i] % quantum != 0) return HSTU_ERR_SHAPE;
  // the kernels address a tile row as (sequence base) + 32-bit byte offset = 24-bit row * 24-bit stride
  const int64_t esize = p->dtype == HSTU_BF16 ? 2 : 4;
  if (p->max_seqlen >= 1 << 24) return HSTU_ERR_UNSUPPORTED;
  for (int i = 0; i < 4; ++i)
    if (strides[i] * esize >= 1 << 24 || strides[i] * esize * ((int64_t)p->max_seqlen + 1) >= (int64_t)1 << 32)
      return HSTU_ERR_UNSUPPORTED;
  if (p->batch > 0 && !p->seq_offsets) return HSTU_ERR_NULL;
  if (p->global_prefix < 0) return HSTU_ERR_SHAPE;
  if ((p->rab_table == nullptr) != (p->rab_bounds == nullptr)) return HSTU_ERR_NULL;
  if (p->rab_table && (p->num_buckets < 1 || p->num_buckets > 4096)) return HSTU_ERR_SHAPE;
  if (p->d_rab_table && !p->rab_table) return HSTU_ERR_NULL;
  if (p->query_tail < 0) return HSTU_ERR_SHAPE;
  if (p->reuse_schedule != 0 && p->reuse_schedule != 1) return HSTU_ERR_SHAPE;
  if ((int64_t)p->total_tokens * p->num_heads / 32 + (int64_t)p->batch * p->num_heads > 0x7FFFFF00) return HSTU_ERR_SHAPE;
  if (p->seq_offsets_host) {
    const int32_t* o = p->seq_offsets_host;
    if (o[0] != 0) return HSTU_ERR_SHAPE;
    for (int b = 0; b < p->batch; ++b) {
      const int64_t len = (int64_t)o[b + 1] - o[b];
      if (len < 0 || len > p->max_seqlen) return HSTU_ERR_SHAPE;
    }
    if (o[p->batch] != p->total_tokens) return HSTU_ERR_SHAPE;
  }
  return HSTU_OK;
}

inline bool misaligned(const void* ptr) { return ((uintptr_t)ptr & 15u) != 0; }

AttnArgs make_args(const hstu_attn_params* p, const void* q, const void* k, const void* v) {
  AttnArgs a = {};
  a.q = q; a.k = k; a.v = v;
  a.sq = p->row_stride_q; a.sk = p->row_stride_k; a.sv = p->row_stride_v; a.so = p->row_stride_o;
  a.offsets = p->seq_offsets; a.num_targets = p->num_targets;
  a.B = p->batch; a.H = p->num_heads; a.D = p->head_dim; a.T = p->total_tokens; a.max_seqlen = p->max_seqlen;
  // sequences are shorter than 2^24 tokens: windows beyond 2^28 mean the same and keep the kernels' index sums inside int32
  a.K1 = p->local_window < 0 ? -1 : (p->local_window < (1 << 28) ? p->local_window : (1 << 28));
  a.K2 = p->global_prefix < (1 << 28) ? p->global_prefix : (1 << 28);
  a.alpha = p->alpha; a.inv_n = p->inv_n;
  a.query_tail = p->query_tail > 0 ? p->query_tail : 0;
  return a;
}

// Enqueues the bias expansion (if any) and fills the bias fields.
hipError_t prepare_bias(const hstu_attn_params* p, AttnArgs& a, unsigned char* ws, const Layout& l, hipStream_t stream,
                        bool for_forward) {
  a.bias = nullptr;
  a.bias_stride = p->max_seqlen + 1;
  a.seed = nullptr;
  if (p->dtype == HSTU_BF16 && p->head_dim == 128 && p->query_tail == 0 && for_forward) {   // the pipelined forward takes bias and mask from the seed tables
    a.seed = (const float*)(ws + l.seed);
    a.seed_len = seed_len_for(p->max_seqlen);
    a.seed_dmax = seed_dmax_for(p->max_seqlen);
    return launch_seed_expand(p->rab_table, p->rab_bounds, p->num_buckets, p->num_heads, p->max_seqlen, a.K1,
                              (float*)(ws + l.seed), stream);           // (that kernel needs no other table)
  }
  if (!p->rab_table) return hipSuccess;
  float* bias = (float*)(ws + l.bias);
  a.bias = bias;
  int32_t* bucket_end = nullptr;                      // only the bias-table gradient needs the bucket ends
  if (!for_forward && p->d_rab_table) bucket_end = (int32_t*)(ws + l.dbias) + (size_t)p->num_heads * a.bias_stride;
  a.bucket_end = bucket_end;
  return launch_bias_expand(p->rab_table, p->rab_bounds, p->num_buckets, p->num_heads, a.bias_stride, bias, bucket_end, stream);
}

}  // namespace

// ---- optional per-kernel timing (for benchmarks): HIP events around every launch, on the launch stream
namespace hstu {
constexpr int kProfSlots = 64;
struct ProfSlot { const char* name; hipEvent_t e0, e1; bool used; };
static ProfSlot g_prof[kProfSlots];
static bool g_prof_on = false, g_prof_init = false;
static int g_prof_n = 0;

ProfScope::ProfScope(const char* name, hipStream_t st) : s(nullptr), stream(st) {
  if (!g_prof_on || g_prof_n >= kProfSlots) return;
  s = &g_prof[g_prof_n++];
  s->name = name;
  s->used = hipEventRecord(s->e0, stream) == hipSuccess;
}
ProfScope::~ProfScope() {
  if (s && s->used) s->used = hipEventRecord(s->e1, stream) == hipSuccess;
}
}  // namespace hstu

extern "C" {

int hstu_profile_enable(int on) {
  if (on && !g_prof_init) {
    for (int i = 0; i < kProfSlots; ++i) {
      if (hipEventCreate(&g_prof[i].e0) != hipSuccess || hipEventCreate(&g_prof[i].e1) != hipSuccess) return HSTU_ERR_LAUNCH;
      g_prof[i].used = false;
    }
    g_prof_init = true;
  }
  g_prof_on = on != 0;
  g_prof_n = 0;
  return HSTU_OK;
}

int hstu_profile_read(int max_entries, const char** names, float* ms) {
  int n = 0;
  for (int i = 0; i < g_prof_n && n < max_entries; ++i) {
    if (!g_prof[i].used) continue;
    if (hipEventSynchronize(g_prof[i].e1) != hipSuccess) return HSTU_ERR_LAUNCH;
    float t = 0.f;
    if (hipEventElapsedTime(&t, g_prof[i].e0, g_prof[i].e1) != hipSuccess) return HSTU_ERR_LAUNCH;
    names[n] = g_prof[i].name;
    ms[n] = t;
    ++n;
  }
  g_prof_n = 0;
  return n;
}

const char* hstu_status_string(int status) {
  switch (status) {
    case HSTU_OK: return "HSTU_OK";
    case HSTU_ERR_NULL: return "HSTU_ERR_NULL: required pointer is NULL";
    case HSTU_ERR_SHAPE: return "HSTU_ERR_SHAPE: invalid sizes, strides, alignment or offsets";
    case HSTU_ERR_UNSUPPORTED: return "HSTU_ERR_UNSUPPORTED: head_dim, dtype or feature count not supported";
    case HSTU_ERR_WORKSPACE: return "HSTU_ERR_WORKSPACE: workspace missing, misaligned or too small";
    case HSTU_ERR_LAUNCH: return "HSTU_ERR_LAUNCH: HIP runtime refused a launch";
    default: return "unknown hstu_status";
  }
}

size_t hstu_attn_workspace_bytes(const hstu_attn_params* p, int for_backward) {
  if (validate(p) != HSTU_OK) return 0;
  return make_layout(p, for_backward).total;
}

int hstu_attn_fwd(const hstu_attn_params* p, const void* q, const void* k, const void* v, void* out, void* workspace,
                  size_t workspace_bytes, void* stream_) {
  const int st = validate(p);
  if (st != HSTU_OK) return st;
  if (p->total_tokens == 0 || p->batch == 0) return HSTU_OK;
  if (!q || !k || !v || !out) return HSTU_ERR_NULL;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out)) return HSTU_ERR_SHAPE;
  const Layout l = make_layout(p, 0);
  if (!workspace || ((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < l.total) return HSTU_ERR_WORKSPACE;
  hipStream_t stream = (hipStream_t)stream_;
  unsigned char* ws = (unsigned char*)workspace;

  AttnArgs a = make_args(p, q, k, v);
  a.out = out;
  a.max_items = l.max_items[0];
  a.header = (const SchedHeader*)(ws + l.header[0]);
  a.items = (const WorkItem*)(ws + l.items[0]);
  a.splits = (const SplitItem*)(ws + l.splits);
  a.partial = (float*)(ws + l.partial);
  if (!p->reuse_schedule) {
    ProfScope ps("schedule_fwd", stream);
    if (launch_schedule(a, fwd_block_rows(p->dtype, p->head_dim), fwd_tile_rows(p->dtype, p->head_dim), false,
                        (SchedHeader*)(ws + l.header[0]), (WorkItem*)(ws + l.items[0]), (int32_t*)(ws + l.seq_base[0]),
                        (SplitItem*)(ws + l.splits), l.slot_cap, stream) != hipSuccess)
      return HSTU_ERR_LAUNCH;
  }
  {
    ProfScope ps("bias_expand_fwd", stream);
    if (prepare_bias(p, a, ws, l, stream, true) != hipSuccess) return HSTU_ERR_LAUNCH;
  }
  {
    ProfScope ps("attn_fwd", stream);                      // includes the kernel that combines the pieces of cut blocks
    if (launch_attn_fwd(a, p->dtype, stream) != hipSuccess) return HSTU_ERR_LAUNCH;
    if (launch_fwd_combine(a, p->dtype, l.slot_cap / 2, stream) != hipSuccess) return HSTU_ERR_LAUNCH;
  }
  return HSTU_OK;
}

int hstu_attn_bwd(const hstu_attn_params* p, const void* q, const void* k, const void* v, const void* dout, void* dq,
                  void* dk, void* dv, void* workspace, size_t workspace_bytes, void* stream_) {
  return hstu::attn_bwd_through_silu(p, q, k, v, nullptr, nullptr, nullptr, 0, dout, dq, dk, dv, workspace, workspace_bytes, stream_);
}

}  // extern "C"

int hstu::attn_bwd_through_silu(const hstu_attn_params* p, const void* q, const void* k, const void* v, const void* pre_q,
                                const void* pre_k, const void* pre_v, int64_t s_pre, const void* dout, void* dq, void* dk,
                                void* dv, void* workspace, size_t workspace_bytes, void* stream_) {
  const int st = validate(p);
  if (st != HSTU_OK) return st;
  if (pre_q || pre_k || pre_v) {
    if (p->dtype != HSTU_BF16) return HSTU_ERR_UNSUPPORTED;
    if (!pre_q || !pre_k || !pre_v) return HSTU_ERR_NULL;
    if (misaligned(pre_q) || misaligned(pre_k) || misaligned(pre_v) || s_pre % 8 != 0 ||
        s_pre < (int64_t)p->num_heads * p->head_dim)
      return HSTU_ERR_SHAPE;
  }
  if (p->query_tail > 0) return HSTU_ERR_UNSUPPORTED;    // the query tail is a forward (inference) feature
  if (p->total_tokens == 0 || p->batch == 0) {           // no pairs: the only output that still exists is a zero table gradient
    if (p->d_rab_table &&
        launch_fill_zero(p->d_rab_table, (size_t)p->num_heads * p->num_buckets, (hipStream_t)stream_) != hipSuccess)
      return HSTU_ERR_LAUNCH;
    return HSTU_OK;
  }
  if (!q || !k || !v || !dout || !dq || !dk || !dv) return HSTU_ERR_NULL;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(dout) || misaligned(dq) || misaligned(dk) ||
      misaligned(dv))
    return HSTU_ERR_SHAPE;
  const Layout l = make_layout(p, 1);
  if (!workspace || ((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < l.total) return HSTU_ERR_WORKSPACE;
  hipStream_t stream = (hipStream_t)stream_;
  unsigned char* ws = (unsigned char*)workspace;

  AttnArgs a = make_args(p, q, k, v);
  a.dout = dout; a.dq = dq; a.dk = dk; a.dv = dv;
  a.pre_q = pre_q; a.pre_k = pre_k; a.pre_v = pre_v; a.s_pre = s_pre;
  const int tile = stream_tile_rows(p->dtype, p->head_dim);
  {
    ProfScope ps("bias_expand_bwd", stream);
    if (prepare_bias(p, a, ws, l, stream, false) != hipSuccess) return HSTU_ERR_LAUNCH;
  }
  if (!p->reuse_schedule) {
    ProfScope ps("schedule_bwd", stream);
    const int rows[2] = {dq_block_rows(p->dtype, p->head_dim), dkv_block_rows(p->dtype, p->head_dim)};
    const int cols[2] = {tile, dkv_tile_rows(p->dtype, p->head_dim)};
    SchedHeader* const hd[2] = {(SchedHeader*)(ws + l.header[0]), (SchedHeader*)(ws + l.header[1])};
    WorkItem* const it[2] = {(WorkItem*)(ws + l.items[0]), (WorkItem*)(ws + l.items[1])};
    int32_t* const sb[2] = {(int32_t*)(ws + l.seq_base[0]), (int32_t*)(ws + l.seq_base[1])};
    SplitItem* const sp[2] = {(SplitItem*)(ws + l.splits_dq), (SplitItem*)(ws + l.splits)};
    const int caps[2] = {l.slot_cap_dq, l.slot_cap};
    if (launch_schedule_pair(a, rows, cols, hd, it, sb, sp, caps, stream) != hipSuccess)
      return HSTU_ERR_LAUNCH;
  }
  if (p->d_rab_table) {
    ProfScope ps("dbias_zero", stream);
    a.dbias_dist = (float*)(ws + l.dbias);
    if (launch_fill_zero(a.dbias_dist, (size_t)p->num_heads * a.bias_stride, stream) != hipSuccess) return HSTU_ERR_LAUNCH;
  }
  for (int s = 0; s < 2; ++s) {                          // s = 0: dQ pass (query blocks), s = 1: dK/dV pass (key blocks)
    a.max_items = l.max_items[s];
    a.header = (const SchedHeader*)(ws + l.header[s]);
    a.items = (const WorkItem*)(ws + l.items[s]);
    a.partial = (float*)(ws + (s == 0 ? l.partial_dq : l.partial));
    a.splits = (const SplitItem*)(ws + (s == 0 ? l.splits_dq : l.splits));
    {
      ProfScope ps(s == 0 ? "attn_bwd_dq" : "attn_bwd_dkdv", stream);     // each figure includes its combine kernel
      const hipError_t e = s == 0 ? launch_attn_bwd_dq(a, p->dtype, stream) : launch_attn_bwd_dkdv(a, p->dtype, stream);
      if (e != hipSuccess) return HSTU_ERR_LAUNCH;
      if (s == 0 && launch_dq_combine(a, p->dtype, l.slot_cap_dq / 2, stream) != hipSuccess) return HSTU_ERR_LAUNCH;
      if (s == 1 && launch_dkdv_combine(a, p->dtype, l.slot_cap / 2, stream) != hipSuccess) return HSTU_ERR_LAUNCH;
    }
    if (s == 0 && p->d_rab_table) {
      ProfScope ps2("dbias_reduce", stream);
      if (launch_dbias_reduce(a.dbias_dist, p->rab_bounds, p->num_buckets, p->num_heads, a.bias_stride, p->inv_n,
                              p->d_rab_table, stream) != hipSuccess)
        return HSTU_ERR_LAUNCH;
    }
  }
  return HSTU_OK;
}

extern "C" {

int hstu_attn_schedule_stats(const hstu_attn_params* p, const void* workspace, int for_backward, int64_t out[3]) {
  const int st = validate(p);
  if (st != HSTU_OK) return st;
  if (!workspace || !out) return HSTU_ERR_NULL;
  const Layout l = make_layout(p, for_backward);
  SchedHeader h;
  if (hipMemcpy(&h, (const unsigned char*)workspace + l.header[0], sizeof(h), hipMemcpyDeviceToHost) != hipSuccess)
    return HSTU_ERR_LAUNCH;
  out[0] = h.count; out[1] = h.tiles; out[2] = h.dense_tiles;
  return h.bad_batch ? HSTU_ERR_SHAPE : HSTU_OK;          // the scheduler found the device-side offsets inconsistent
}

static int validate_norm(int64_t T, int32_t D, int32_t dtype) {
  if (T < 0 || D < 1) return HSTU_ERR_SHAPE;
  if (dtype != HSTU_BF16 && dtype != HSTU_FP32) return HSTU_ERR_UNSUPPORTED;
  if (D % 8 != 0 || D > 8192) return HSTU_ERR_UNSUPPORTED;
  return HSTU_OK;
}

int hstu_gated_norm_fwd(int64_t T, int32_t D, int32_t dtype, const void* attn, const void* u, const float* gamma,
                        const float* beta, float eps, void* y, float* mean, float* rstd, void* stream) {
  const int st = validate_norm(T, D, dtype);
  if (st != HSTU_OK) return st;
  if (T == 0) return HSTU_OK;
  if (!attn || !u || !gamma || !y) return HSTU_ERR_NULL;
  if (misaligned(attn) || misaligned(u) || misaligned(gamma) || misaligned(y) || (beta && misaligned(beta))) return HSTU_ERR_SHAPE;
  ProfScope ps("gated_norm_fwd", (hipStream_t)stream);
  if (launch_gated_norm_fwd(T, D, dtype, attn, u, gamma, beta, eps, y, mean, rstd, (hipStream_t)stream) != hipSuccess)
    return HSTU_ERR_LAUNCH;
  return HSTU_OK;
}

size_t hstu_gated_norm_bwd_workspace_bytes(int64_t T, int32_t D) {
  if (T < 0 || D < 1) return 0;
  const size_t blocks = (size_t)gated_norm_bwd_blocks(T, D);
  return align_up((blocks > 0 ? blocks : 1) * 2 * (size_t)D * sizeof(float));
}

int hstu_gated_norm_bwd(int64_t T, int32_t D, int32_t dtype, const void* dy, const void* attn, const void* u,
                        const float* gamma, const float* beta, float eps, void* dattn, void* du, float* dgamma,
                        float* dbeta, void* workspace, size_t workspace_bytes, void* stream) {
  const int st = validate_norm(T, D, dtype);
  if (st != HSTU_OK) return st;
  if (!gamma || !dgamma) return HSTU_ERR_NULL;
  if (T > 0 && (!dy || !attn || !u || !dattn || !du)) return HSTU_ERR_NULL;
  if (misaligned(dy) || misaligned(attn) || misaligned(u) || misaligned(gamma) || misaligned(dattn) || misaligned(du) ||
      (beta && misaligned(beta)))
    return HSTU_ERR_SHAPE;
  if (!workspace || ((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < hstu_gated_norm_bwd_workspace_bytes(T, D))
    return HSTU_ERR_WORKSPACE;
  ProfScope ps("gated_norm_bwd", (hipStream_t)stream);
  if (launch_gated_norm_bwd(T, D, dtype, dy, attn, u, gamma, beta, eps, dattn, du, dgamma, dbeta, (float*)workspace,
                            (hipStream_t)stream) != hipSuccess)
    return HSTU_ERR_LAUNCH;
  return HSTU_OK;
}

// ---- the gated-norm backward for callers that cannot allocate -------------------------------------------------
// Same kernels as hstu_gated_norm_bwd; the partial column sums live in a file-scope device array instead of a
// caller-provided workspace.  In host code the array's name is only a stand-in: the address the kernels get is the one
// hipGetSymbolAddress reports for the current device (every GPU holds its own copy), looked up once per device.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxScratchDevices = 64;
static void* g_scratch_ptr[kMaxScratchDevices];
static std::mutex g_scratch_mutex;

static int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxScratchDevices) return HSTU_ERR_LAUNCH;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return HSTU_ERR_LAUNCH;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return HSTU_OK;
}

size_t hstu_gated_norm_bwd_static_max_bytes(void) { return kStaticScratchBytes; }

int hstu_gated_norm_bwd_static(int64_t T, int32_t D, int32_t dtype, const void* dy, const void* attn, const void* u,
                               const float* gamma, const float* beta, float eps, void* dattn, void* du, float* dgamma,
                               float* dbeta, void* stream) {
  const int st = validate_norm(T, D, dtype);
  if (st != HSTU_OK) return st;
  if (!gamma || !dgamma) return HSTU_ERR_NULL;
  if (T > 0 && (!dy || !attn || !u || !dattn || !du)) return HSTU_ERR_NULL;
  if (misaligned(dy) || misaligned(attn) || misaligned(u) || misaligned(gamma) || misaligned(dattn) || misaligned(du) ||
      (beta && misaligned(beta)))
    return HSTU_ERR_SHAPE;
  if (hstu_gated_norm_bwd_workspace_bytes(T, D) > kStaticScratchBytes) return HSTU_ERR_WORKSPACE;
  void* partial = nullptr;
  const int sp = static_scratch(&partial);
  if (sp != HSTU_OK) return sp;
  // every workgroup overwrites its whole row of partial sums and the column-sum kernel reads only the rows of this
  // launch, so nothing left by an earlier call is ever read and nothing needs clearing
  if (launch_gated_norm_bwd(T, D, dtype, dy, attn, u, gamma, beta, eps, dattn, du, dgamma, dbeta, (float*)partial,
                            (hipStream_t)stream) != hipSuccess)
    return HSTU_ERR_LAUNCH;
  return HSTU_OK;
}

// ---- attention truncation (Section 4.3) ------------------------------------------------------------------------
static bool bad16(const void* ptr) { return ((uintptr_t)ptr & 15) != 0; }
static int validate_rows(int64_t row_bytes, int64_t stride_a, int64_t stride_b) {
  if (row_bytes < 0 || (row_bytes & 15) || (stride_a & 15) || (stride_b & 15) || stride_a < row_bytes || stride_b < row_bytes)
    return HSTU_ERR_SHAPE;
  return HSTU_OK;
}

int hstu_truncate_offsets(int32_t batch, int32_t keep, const int32_t* seq_offsets, const int32_t* num_targets,
                          int32_t* out_offsets, void* stream) {
  if (batch < 0 || keep < 0) return HSTU_ERR_SHAPE;
  if (!seq_offsets || !out_offsets) return HSTU_ERR_NULL;
  ProfScope ps("truncate_offsets", (hipStream_t)stream);
  if (launch_truncate_offsets(batch, keep, seq_offsets, num_targets, out_offsets, (hipStream_t)stream) != hipSuccess)
    return HSTU_ERR_LAUNCH;
  return HSTU_OK;
}

int hstu_truncate_fwd(int32_t batch, const int32_t* seq_offsets, const int32_t* out_offsets, int64_t row_bytes,
                      const void* x, int64_t x_stride_bytes, void* y, int64_t y_stride_bytes, int64_t y_rows,
                      void* stream) {
  if (batch < 0 || y_rows < 0) return HSTU_ERR_SHAPE;
  const int st = validate_rows(row_bytes, x_stride_bytes, y_stride_bytes);
  if (st != HSTU_OK) return st;
  if (batch == 0 || y_rows == 0 || row_bytes == 0) return HSTU_OK;
  if (!seq_offsets || !out_offsets || !x || !y) return HSTU_ERR_NULL;
  if (bad16(x) || bad16(y)) return HSTU_ERR_SHAPE;
  ProfScope ps("truncate_fwd", (hipStream_t)stream);
  if (launch_truncate_gather(batch, seq_offsets, out_offsets, row_bytes, x, x_stride_bytes, y, y_stride_bytes, y_rows,
                             (hipStream_t)stream) != hipSuccess)
    return HSTU_ERR_LAUNCH;
  return HSTU_OK;
}

int hstu_truncate_bwd(int32_t batch, int64_t total_tokens, const int32_t* seq_offsets, const int32_t* out_offsets,
                      int64_t row_bytes, const void* dy, int64_t dy_stride_bytes, void* dx, int64_t dx_stride_bytes,
                      void* stream) {
  if (batch < 0 || total_tokens < 0 || total_tokens > 0x7fffffff) return HSTU_ERR_SHAPE;
  const int st = validate_rows(row_bytes, dy_stride_bytes, dx_stride_bytes);
  if (st != HSTU_OK) return st;
  if (batch == 0 || total_tokens == 0 || row_bytes == 0) return HSTU_OK;
  if (!seq_offsets || !out_offsets || !dx) return HSTU_ERR_NULL;   // dy may be NULL when no row survives (never read then)
  if (bad16(dy) || bad16(dx)) return HSTU_ERR_SHAPE;
  ProfScope ps("truncate_bwd", (hipStream_t)stream);
  if (launch_truncate_scatter(batch, total_tokens, seq_offsets, out_offsets, row_bytes, dy, dy_stride_bytes, dx,
                              dx_stride_bytes, (hipStream_t)stream) != hipSuccess)
    return HSTU_ERR_LAUNCH;
  return HSTU_OK;
}

// ---- FP8 around the projections (Section 4.2.2) ------------------------------------------------------------------
int hstu_norm_quant_fp8(int64_t T, int32_t D, int32_t dtype, const void* a, const void* u, const float* gamma,
                        const float* beta, float eps, void* q, float* q_scale, float* mean, float* rstd, void* stream) {
  const int st = validate_norm(T, D, dtype);
  if (st != HSTU_OK) return st;
  if (T == 0) return HSTU_OK;
  if (!a || !q || !q_scale) return HSTU_ERR_NULL;
  if (beta && !gamma) return HSTU_ERR_NULL;
  if (misaligned(a) || (u && misaligned(u)) || (gamma && misaligned(gamma)) || (beta && misaligned(beta)) ||
      ((uintptr_t)q & 7u))
    return HSTU_ERR_SHAPE;
  NormFwdArgs p = {};
  p.T = T; p.D = D; p.dtype = dtype; p.a = a; p.sa = D; p.u = u; p.su = D; p.gamma = gamma; p.beta = beta; p.eps = eps;
  p.y = nullptr; p.sy = D; p.mean = mean; p.rstd = rstd; p.stats_in = 0;
  ProfScope ps("norm_quant_fp8", (hipStream_t)stream);
  if (launch_norm_quant_fwd(p, q, D, q_scale, (hipStream_t)stream) != hipSuccess) return HSTU_ERR_LAUNCH;
  return HSTU_OK;
}

int hstu_fp8_gemm_bias2d(int64_t M, int32_t N, int32_t K, const void* a_q, const float* a_scale, const void* b_q,
                         const float* b_scale, const void* c, void* d, void* stream) {
  if (M < 0 || N < 1 || K < 1) return HSTU_ERR_SHAPE;
  if (!fp8_gemm_supported(N, K)) return HSTU_ERR_UNSUPPORTED;
  if (M == 0) return HSTU_OK;
  if (!a_q || !a_scale || !b_q || !b_scale || !d) return HSTU_ERR_NULL;
  if (misaligned(a_q) || misaligned(b_q) || misaligned(b_scale) || (c && misaligned(c)) || misaligned(d)) return HSTU_ERR_SHAPE;
  if ((M + 127) / 128 > 0x7fffffff) return HSTU_ERR_SHAPE;
  ProfScope ps("fp8_gemm_bias2d", (hipStream_t)stream);
  if (launch_fp8_gemm_bias2d(M, N, K, a_q, a_scale, b_q, b_scale, c, d, (hipStream_t)stream) != hipSuccess) return HSTU_ERR_LAUNCH;
  return HSTU_OK;
}

}  // extern "C"
