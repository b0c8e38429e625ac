// Internal launch interface between the C-ABI layer (api.hip) and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

struct hstu_attn_params;

namespace hstu {

// First 256 bytes of every attention workspace.
struct SchedHeader {
  int32_t count;          // scheduled work items (row block x head, or pieces of one)
  int32_t splits;         // row blocks that were cut into pieces (entries of the SplitItem list)
  int64_t tiles;          // scheduled (row block, column block) tiles, all heads
  int64_t dense_tiles;    // tiles of the full L x L grids, all heads
  int32_t chunk_tiles;    // piece size used for the cut blocks
  int32_t bad_batch;      // 1: seq_offsets / num_targets on the device contradict the description (then count = 0: no kernel
                          // touches a token row)
};

struct WorkItem {
  int32_t b;              // sequence
  int32_t rb_h;           // (block index << 8) | head
  int32_t t0, t1;         // positions [t0, min(t1, tiles of the block)) of the block's tile list
  int32_t slot;           // partial-sum slot of a piece, -1: the item writes its block's output itself
  // the item's sequence, copied here so that a workgroup's first loads do not wait for a look-up by b:
  int32_t seq0, len, hist;   // first token row, length, history length (length minus candidates)
};

struct SplitItem {        // a row block whose pieces left partial sums in slots [first_slot, first_slot + pieces)
  int32_t b, rb_h, first_slot, pieces;
};

// Everything a kernel needs to know about the attention problem.
struct AttnArgs {
  const void* q; const void* k; const void* v; const void* dout;
  void* out; void* dq; void* dk; void* dv;
  int64_t sq, sk, sv, so;           // row strides in elements
  const int32_t* offsets;
  const int32_t* num_targets;
  int32_t B, H, D, T, max_seqlen;
  int32_t K1, K2;
  float alpha, inv_n;
  const float* bias;                // expanded table [H, bias_stride] indexed by distance, or nullptr
  int32_t bias_stride;
  const SchedHeader* header;
  const WorkItem* items;
  int32_t max_items;
  float* partial;                   // dK/dV pass: fp32 partial sums [slot][dK, dV][block row][D] of cut key blocks
  const SplitItem* splits;
  int32_t query_tail;               // forward only, > 0: compute only the last query_tail history rows and the candidates of every sequence
  float* dbias_dist;                // dQ pass, optional: sum of dS per head and distance [H, bias_stride] (zeroed by the caller)
  // optional (bf16 backward): q, k, v = SiLU(pre_q / pre_k / pre_v) [T, H, D] with row stride s_pre; dq, dk, dv then leave
  // as the gradients of those pre-activations (multiplied by SiLU' on the way out)
  const void* pre_q; const void* pre_k; const void* pre_v; int64_t s_pre;
  const int32_t* bucket_end;        // with dbias_dist: [bias_stride], the first distance of the bucket after the one that holds distance i (INT_MAX: none)
  // Score seeds of the pipelined kernels: bias and mask of a (position, key) pair as a function of the distance
  // d = position - key alone, [variant][H][seed_len] floats:  seed[i] <-> d = seed_dmax - i (descending distances, so that
  // 4 consecutive floats are the seeds of 4 consecutive keys).  d < 0 (a later key): -1e30 (which the pointwise step
  // turns into an exact zero); 0 <= d: bias of d in units of ln 2 (0 without a bias table); variant 1 (band tiles of a
  // semi-local mask) also has -1e30 for d >= K1.  seed_dmax >= max_seqlen + 128, seed_len >= seed_dmax + 1 + 192.
  const float* seed;
  int32_t seed_len, seed_dmax;
};
constexpr int kSeedVariants = 2;
inline int seed_dmax_for(int max_seqlen) { return max_seqlen + 128; }
inline int seed_len_for(int max_seqlen) { return (seed_dmax_for(max_seqlen) + 1 + 192 + 63) / 64 * 64; }

// schedule.hip
// Builds the work list for blocks of `block_rows` rows (query rows in the forward and the dQ pass,
// key rows when `key_major` is set) against column tiles of `tile_cols`.
// `splits` / `slot_cap` (optional): blocks much longer than the rest may be cut into pieces that leave partial sums in slots.
hipError_t launch_schedule(const AttnArgs& a, int block_rows, int tile_cols, bool key_major, SchedHeader* header,
                           WorkItem* items, int32_t* seq_base, SplitItem* splits, int slot_cap, hipStream_t stream);
// The two lists of the backward pass in one launch: [0] query blocks (dQ pass), [1] key blocks (dK/dV pass).
// `splits` / `slot_cap`: list of cut key blocks and number of partial-sum slots available to the dK/dV list.
hipError_t launch_schedule_pair(const AttnArgs& a, const int block_rows[2], const int tile_cols[2], SchedHeader* const header[2],
                                WorkItem* const items[2], int32_t* const seq_base[2], SplitItem* const splits[2],
                                const int slot_cap[2], hipStream_t stream);
// bucket_end (optional, [len]): for every distance the first distance of the next bucket
hipError_t launch_bias_expand(const float* table, const int32_t* bounds, int num_buckets, int H, int len, float* out, int32_t* bucket_end,
                              hipStream_t stream);
// fills AttnArgs::seed (table may be nullptr: no bias)
hipError_t launch_seed_expand(const float* table, const int32_t* bounds, int num_buckets, int H, int max_seqlen, int K1,
                              float* out, hipStream_t stream);

// attn_core.hip
int fwd_block_rows(int dtype, int D);     // query rows per workgroup, forward
int dq_block_rows(int dtype, int D);      // query rows per workgroup, dQ pass
int dkv_block_rows(int dtype, int D);     // key rows per workgroup, dK/dV pass
int stream_tile_rows(int dtype, int D);   // rows of one streamed LDS tile (dQ pass)
int fwd_tile_rows(int dtype, int D);      // ... in the forward
int dkv_tile_rows(int dtype, int D);      // ... in the dK/dV pass
hipError_t launch_attn_fwd(const AttnArgs& a, int dtype, hipStream_t stream);
// attn_fwd_pipe.hip: the forward for bf16 and 128 features per head (same work lists as launch_attn_fwd: 128-row blocks, 32-key tiles)
hipError_t launch_attn_fwd_pipe(const AttnArgs& a, hipStream_t stream);
// hstu_attn_bwd for operands that are SiLU of pre-activations (bf16 only; pre_* [T, H, D] with row stride s_pre, all three
// or none): dq, dk, dv leave as the gradients of the pre-activations.  Same checks and error codes as hstu_attn_bwd.
int attn_bwd_through_silu(const hstu_attn_params* p, const void* q, const void* k, const void* v, const void* pre_q,
                          const void* pre_k, const void* pre_v, int64_t s_pre, const void* dout, void* dq, void* dk, void* dv,
                          void* workspace, size_t workspace_bytes, void* stream);
hipError_t launch_attn_bwd_dq(const AttnArgs& a, int dtype, hipStream_t stream);
hipError_t launch_attn_bwd_dkdv(const AttnArgs& a, int dtype, hipStream_t stream);
// bias-table gradient: clear the per-distance sums, fold them into buckets (times `scale`) after the dQ pass
hipError_t launch_fill_zero(float* p, size_t n, hipStream_t stream);
hipError_t launch_dbias_reduce(const float* dist, const int32_t* bounds, int num_buckets, int H, int len, float scale,
                               float* dtable, hipStream_t stream);
// adds the partial sums of every cut key block in piece order, scales, converts and writes dK, dV
hipError_t launch_dkdv_combine(const AttnArgs& a, int dtype, int max_splits, hipStream_t stream);
// the same for query blocks of the forward whose key axis was cut (forward over a query tail): writes the output rows
hipError_t launch_fwd_combine(const AttnArgs& a, int dtype, int max_splits, hipStream_t stream);
hipError_t launch_dq_combine(const AttnArgs& a, int dtype, int max_splits, hipStream_t stream);

// gated_norm.hip
// Row-wise layer norm with weight (and optional bias), optionally gated by U; row strides in elements.
struct NormFwdArgs {
  int64_t T; int32_t D; int32_t dtype;
  const void* a; int64_t sa;                // input rows
  const void* u; int64_t su;                // gate, or nullptr: plain layer norm
  const float* gamma; const float* beta;    // beta may be nullptr
  float eps;
  void* y; int64_t sy;
  float* mean; float* rstd;                 // outputs (may be nullptr), or inputs when stats_in is set
  int32_t stats_in;
};
struct NormBwdArgs {
  int64_t T; int32_t D; int32_t dtype;
  const void* dy; int64_t sdy;
  const void* a; int64_t sa;
  const void* u; int64_t su;                // nullptr: plain layer norm (du is not written)
  const float* gamma; const float* beta;
  float eps;
  void* da; int64_t sda;
  void* du; int64_t sdu;
  void* y_out; int64_t sy_out;              // optional (with a gate): the forward's output Y = (LN(a) gamma + beta) * u, rebuilt along the way
  const void* du_pre; int64_t sdu_pre;      // optional: u = SiLU(du_pre); du then leaves as the gradient of du_pre (du * SiLU'(du_pre))
  const void* residual; int64_t sres;       // optional rows added to da (gradient of a residual connection)
  float* dgamma; float* dbeta;              // dbeta may be nullptr
};
hipError_t launch_norm_fwd(const NormFwdArgs& p, hipStream_t stream);
// same rows as launch_norm_fwd (p.y unused; p.gamma == nullptr: no normalisation), written as E4M3 codes q [T, D] (row stride
// sq bytes) with one fp32 scale per row
hipError_t launch_norm_quant_fwd(const NormFwdArgs& p, void* q, int64_t sq, float* qscale, hipStream_t stream);
hipError_t launch_norm_bwd(const NormBwdArgs& p, float* partial, hipStream_t stream);   // partial: gated_norm_bwd_blocks(T, D) x 2 x D floats
int gated_norm_bwd_blocks(int64_t T, int D);
hipError_t launch_gated_norm_fwd(int64_t T, int D, int dtype, const void* attn, const void* u, const float* gamma,
                                 const float* beta, float eps, void* y, float* mean, float* rstd, hipStream_t stream);
hipError_t launch_gated_norm_bwd(int64_t T, int D, int dtype, const void* dy, const void* attn, const void* u,
                                 const float* gamma, const float* beta, float eps, void* dattn, void* du, float* dgamma,
                                 float* dbeta, float* partial, hipStream_t stream);


// pointwise.hip: SiLU of the [T, C] projection (bf16, contiguous, C a multiple of 8) and its backward
hipError_t launch_silu_fwd(int64_t T, int C, const void* pre, void* act, void* u_out, int u_cols, hipStream_t stream, int skip_cols = 0);
hipError_t launch_silu_bwd(int64_t T, int C, const void* pre, void* dact, hipStream_t stream);

// gemm.hip: row-major bf16 products with fp32 accumulation through hipBLASLt.
//   kGemmNT: D[M,N] = A[M,K] B[N,K]^T    kGemmNN: D[M,N] = A[M,K] B[K,N]    kGemmTN: D[M,N] = A[K,M]^T B[K,N]
// C: optional bf16 [M,N] added to the product (nullptr: none); D bf16 or fp32 (d_fp32); ld*: row strides in elements.
// silu: SiLU applied to the product in the library's epilogue, before the one rounding to bf16.
// Returns 0, -1 (library error) or -2 (no kernel for this problem).  gemm_bf16_tunings: how often candidates were timed.
enum { kGemmNT = 0, kGemmNN = 1, kGemmTN = 2 };
long gemm_bf16_tunings();
int gemm_bf16(int op, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B, int64_t ldb, const void* C,
              int64_t ldc, void* D, int64_t ldd, bool d_fp32, void* ws, size_t ws_bytes, hipStream_t stream, bool silu = false);

// fp8_gemm.hip: D[M,N] (bf16) = a_scale[m] b_scale[n] (Aq[M,K] Bq[N,K]^T) + C[M,N] (bf16 or nullptr), E4M3 codes
bool fp8_gemm_supported(int N, int K);
hipError_t launch_fp8_gemm_bias2d(int64_t M, int N, int K, const void* A, const float* a_scale, const void* B, const float* b_scale,
                                  const void* C, void* D, hipStream_t stream);
// the same product followed by x sigmoid(x); output features [0, u_cols) go to u_out [M, u_cols] instead of D (u_cols a multiple of 64)
hipError_t launch_fp8_gemm_silu(int64_t M, int N, int K, const void* A, const float* a_scale, const void* B, const float* b_scale,
                                void* D, void* u_out, int u_cols, hipStream_t stream);

// gemm_tn.hip: C[N1, N2] (fp32) = A[T, N1]^T B[T, N2] (bf16, row strides lda, ldb in elements), reduction cut into slabs
// of token rows with fp32 partial tiles in `partial` (gemm_tn_workspace_bytes) added in a fixed order.  N1, N2 multiples of 128.
bool gemm_tn_supported(int N1, int N2);
size_t gemm_tn_workspace_bytes(int64_t T, int N1, int N2);
hipError_t launch_gemm_tn(int64_t T, int N1, int N2, const void* A, int64_t lda, const void* B, int64_t ldb, float* C, float* partial,
                          hipStream_t stream);

// truncate.hip (strides and row sizes in bytes, multiples of 16)
hipError_t launch_truncate_offsets(int B, int keep, const int32_t* offsets, const int32_t* num_targets, int32_t* out,
                                   hipStream_t stream);
hipError_t launch_truncate_gather(int B, const int32_t* offsets, const int32_t* out_offsets, int64_t row_bytes, const void* x,
                                  int64_t x_stride, void* y, int64_t y_stride, int64_t y_rows, hipStream_t stream);
hipError_t launch_truncate_scatter(int B, int64_t T, const int32_t* offsets, const int32_t* out_offsets, int64_t row_bytes,
                                   const void* dy, int64_t dy_stride, void* dx, int64_t dx_stride, hipStream_t stream);

}  // namespace hstu
