/*
 * hstu_attn.h - C ABI of the MI355X (gfx950) jagged HSTU attention library.
 *
 * The library computes the attention step and the gated-normalisation step of one
 * HSTU layer (paper Eq. 3 and Eq. 4) over jagged, variable-length sequences, their
 * backward passes, and the jagged row selection of attention truncation (Section 4.3) (op signatures of the appendix pseudocode of the paper:
 * attention_forward(q,k,v), attention_backward(dattn,q,k,v),
 * gated_norm_forward(attn,u,w), gated_norm_backward(dy,attn,u,w)).
 *
 * General conventions
 *   - All tensor pointers are DEVICE pointers unless a comment says HOST.
 *   - The caller owns every buffer.  The library never allocates, frees or
 *     synchronises; all work is enqueued on `stream` (a hipStream_t passed as
 *     void*, NULL = the default stream) and the call returns immediately.
 *   - Jagged layout: a batch of B sequences with lengths L_b is stored without
 *     padding as T = sum L_b token rows; seq_offsets[b] is the first row of
 *     sequence b and seq_offsets[B] = T.  Q, K, V, A (and gradients) are
 *     [T, H, d]: element (t, h, c) lives at  base + t*row_stride + h*d + c
 *     (strides in elements), so the four tensors may be views into one fused
 *     [T, 4*H*d] buffer (the paper avoids concatenating dU,dQ,dK,dV, Section 4.2.2).
 *   - Outputs are fully overwritten for every token row of every non-empty
 *     sequence; nothing is accumulated into them.
 *   - Every entry point returns an hstu_status; errors are reported through it
 *     (never by abort/exception) and no kernel is launched on error.
 *   - B = 0, T = 0 and zero-length sequences are valid: nothing is written for them.
 */
#ifndef HSTU_ATTN_H
#define HSTU_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  HSTU_OK = 0,
  HSTU_ERR_NULL = -1,        /* a required pointer is NULL */
  HSTU_ERR_SHAPE = -2,       /* negative sizes, strides too small, bad offsets (when a host copy is given) */
  HSTU_ERR_UNSUPPORTED = -3, /* head_dim / dtype / D outside the supported set */
  HSTU_ERR_WORKSPACE = -4,   /* workspace NULL, misaligned (256 B) or smaller than *_workspace_bytes */
  HSTU_ERR_LAUNCH = -5       /* the HIP runtime refused a launch */
} hstu_status;

typedef enum { HSTU_BF16 = 0, HSTU_FP32 = 1 } hstu_dtype;

/*
 * Attention problem description (paper Eq. 3 with the masks of Section 4.2.1).
 *
 * For sequence b of length L whose last M = num_targets[b] tokens are candidates
 * (n = L - M history tokens), query row i and key j (0-based inside the sequence):
 *   hist(p, j)   = j < n && j <= p && (local_window < 0 || p - j < local_window || j < global_prefix)
 *   history row   i <  n : visible = hist(i, j),             distance = i - j
 *   candidate row i >= n : visible = (j == i) || hist(n, j), distance = (j == i) ? 0 : n - j
 *   s = alpha * <Q[i,h,:], K[j,h,:]> + rab_table[h, bucket(distance)]
 *   A[i,h,:] = sum over visible j of  s * sigmoid(s) * inv_n * V[j,h,:]
 *   bucket(x) = max{ c : rab_bounds[c] <= x }.
 * This is the paper's causal mask (local_window < 0) and semi-local mask (local
 * band of local_window keys including the query itself, plus the first
 * global_prefix keys of the sequence); local_window = 0 with global_prefix > 0 is
 * the global-only ablation.  The 1/N factor, the relative-position bias and the
 * candidate rows are not in the paper's equations; they follow the task's
 * statement of the layer.
 */
typedef struct hstu_attn_params {
  int32_t batch;            /* B >= 0 */
  int32_t num_heads;        /* H in [1, 256] */
  int32_t head_dim;         /* d = d_qk = d_v: 32, 64 or 128 */
  int32_t total_tokens;     /* T = seq_offsets[B] */
  int32_t max_seqlen;       /* >= max_b L_b; sizes the expanded bias table and index ranges */
  int32_t dtype;            /* hstu_dtype of q, k, v, out, dout, dq, dk, dv */
  int64_t row_stride_q;     /* elements between consecutive tokens of q (and of dq); >= H*d, a multiple of 16 bytes,
                               a row
                               must span less than 16 MiB and (max_seqlen + 1) rows less than 4 GiB (else
                               HSTU_ERR_UNSUPPORTED); max_seqlen < 2^24 */
  int64_t row_stride_k;     /* same for k / dk */
  int64_t row_stride_v;     /* same for v / dv */
  int64_t row_stride_o;     /* same for out / dout */
  const int32_t* seq_offsets;      /* DEVICE int32[B+1], [0] = 0, non-decreasing */
  const int32_t* seq_offsets_host; /* HOST copy of the same, or NULL; when given it is validated */
  const int32_t* num_targets;      /* DEVICE int32[B] (0 <= M_b <= L_b) or NULL = no candidates */
  int32_t local_window;     /* K1: < 0 dense causal; >= 0 keys with 0 <= p - j < K1 */
  int32_t global_prefix;    /* K2 >= 0: keys j < K2 (ignored when local_window < 0) */
  float alpha;              /* multiplies QK^T; the paper has none (1.0) */
  float inv_n;              /* 1/N applied after SiLU */
  const float* rab_table;   /* DEVICE fp32[H, num_buckets] or NULL = no bias */
  const int32_t* rab_bounds;/* DEVICE int32[num_buckets], strictly increasing, [0] = 0 (NULL iff rab_table NULL) */
  int32_t num_buckets;      /* in [1, 4096] when rab_table is given */
  float* d_rab_table;       /* hstu_attn_bwd only, optional: DEVICE fp32[H, num_buckets] receives the gradient of
                               rab_table (sum of dS over the visible pairs of each bucket), overwritten; NULL = not
                               wanted; ignored by hstu_attn_fwd; requires rab_table */
  int32_t query_tail;       /* hstu_attn_fwd only; 0: every row.  > 0: only the last query_tail history rows and the candidate
                               rows of every sequence are computed (against all the keys they see); the other rows of `out` are
                               left untouched.  This is the shape of the last full-length layer in front of an attention
                               truncation (Section 4.3: only the rows that survive are needed) and of serving few recent rows
                               against a long history.  hstu_attn_bwd and the layer entry points return HSTU_ERR_UNSUPPORTED
                               when it is set */
  int32_t reuse_schedule;   /* 0: the call builds its work lists (tile scheduler) in the workspace.  1: the workspace still holds the
                               lists that the same entry point (hstu_attn_fwd, or hstu_attn_bwd) wrote for the same batch,
                               num_heads, head_dim, dtype, mask and query_tail, and no other call has used the workspace since: the
                               scheduler is skipped (the layers of one model share seq_offsets and mask, so only the first layer
                               of a forward or of a backward sweep needs it).  The bias table is expanded on every call.  The
                               layer entry points pass it on to their attention calls */
} hstu_attn_params;

/* Bytes of device scratch (256-byte aligned) that hstu_attn_fwd (for_backward = 0)
 * or hstu_attn_bwd (for_backward != 0) needs for this problem.  Depends only on
 * batch, num_heads, head_dim, total_tokens, max_seqlen and dtype.  Returns 0 for an
 * invalid description (the compute call then reports the error).  The backward figure
 * includes fp32 partial-sum slots for key blocks that the scheduler cuts along the query
 * axis (at most 768 x 2 x 128 x head_dim floats, about 100 MB at head_dim 128) and for query blocks that the dQ pass cuts
 * along the key axis (768 x 128 x head_dim floats); the forward figure includes the same kind of slots for its query blocks
 * (50 MB at head_dim 128). */
size_t hstu_attn_workspace_bytes(const hstu_attn_params* p, int for_backward);

/* Paper Eq. 3, forward (attention_forward of the appendix pseudocode).
 * q, k, v: inputs [T, H, d]; out: A [T, H, d]; all DEVICE, dtype p->dtype.
 * Enqueues: tile scheduler (skips fully masked blocks), bias expansion, attention kernel, combine kernel.
 * A query block whose list of key tiles is longer than a workgroup slot's share of the whole batch (small batches: one
 * long sequence, a few short ones) is cut into equal pieces along the key axis; the pieces write fp32 partial sums into
 * the workspace and the combine kernel adds them in piece order (deterministic) and writes the rows. */
int hstu_attn_fwd(const hstu_attn_params* p, const void* q, const void* k, const void* v, void* out,
                  void* workspace, size_t workspace_bytes, void* stream);

/* Backward of Eq. 3 (attention_backward(dattn, q, k, v) -> dq, dk, dv): the scores are
 * recomputed from q, k; nothing saved by the forward is needed.  dout uses row_stride_o,
 * dq/dk/dv use the strides of q/k/v.  dq, dk, dv are deterministic: no atomics; partial sums
 * of cut blocks (key blocks of a global prefix; query blocks of a small batch) are added in a fixed order.  With p->d_rab_table set the dQ pass also sums
 * dS per distance with fp32 atomics (run-to-run differences at rounding level) and a small
 * kernel folds the distances into buckets. */
int hstu_attn_bwd(const hstu_attn_params* p, const void* q, const void* k, const void* v, const void* dout,
                  void* dq, void* dk, void* dv, void* workspace, size_t workspace_bytes, void* stream);

/* Paper Eq. 4 without f2 (gated_norm_forward): Y = (LayerNorm_D(A) * gamma + beta) * U, the layer
 * norm taken over the D = H*d features of a token (biased variance, eps inside the square root).
 * attn, u, y: [T, D] contiguous, dtype `dtype`; gamma: fp32[D]; beta: fp32[D] or NULL (= 0);
 * mean, rstd: fp32[T] outputs or NULL.  D must be a multiple of 8 and at most 8192. */
int hstu_gated_norm_fwd(int64_t T, int32_t D, int32_t dtype, const void* attn, const void* u, const float* gamma,
                        const float* beta, float eps, void* y, float* mean, float* rstd, void* stream);

/* Bytes of scratch hstu_gated_norm_bwd needs (partial column sums for dgamma/dbeta). */
size_t hstu_gated_norm_bwd_workspace_bytes(int64_t T, int32_t D);

/* gated_norm_backward(dy, attn, u, w) -> dattn, du, dw: recomputes the normalised A.
 * dattn, du: [T, D] dtype `dtype`; dgamma: fp32[D]; dbeta: fp32[D] or NULL.  Deterministic. */
int hstu_gated_norm_bwd(int64_t T, int32_t D, int32_t dtype, const void* dy, const void* attn, const void* u,
                        const float* gamma, const float* beta, float eps, void* dattn, void* du, float* dgamma,
                        float* dbeta, void* workspace, size_t workspace_bytes, void* stream);

/* hstu_gated_norm_bwd for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving or training loops, harnesses that forbid hipMalloc.  Same arguments, kernels and results as
 * hstu_gated_norm_bwd without the workspace: the partial column sums go to a device array that the library itself
 * holds (hstu_gated_norm_bwd_static_max_bytes() = 16 MiB on every GPU the library runs on, until the process ends).
 * A problem whose hstu_gated_norm_bwd_workspace_bytes(T, D) exceeds that size is rejected with HSTU_ERR_WORKSPACE and
 * nothing is launched (no supported D reaches it today).  The call allocates and frees nothing and does not
 * synchronise; the first call on a device looks up the array's address on that device (no allocation either; make
 * that first call outside a graph capture).  All calls on one GPU share the array: calls that may overlap on one GPU
 * (different streams, different host threads) race on it and must be serialised by the caller; calls on one stream
 * are safe.  Nothing has to be cleared between calls: every launch overwrites all it reads. */
size_t hstu_gated_norm_bwd_static_max_bytes(void);
int hstu_gated_norm_bwd_static(int64_t T, int32_t D, int32_t dtype, const void* dy, const void* attn, const void* u,
                               const float* gamma, const float* beta, float eps, void* dattn, void* du, float* dgamma,
                               float* dbeta, void* stream);

/*
 * Attention truncation (paper Section 4.3, "Attention Truncation"): after a first group of layers has seen
 * the whole sequence, the remaining layers run on a segment of it, and the segment the paper settles on is
 * the most recent part of the user's history.  Of sequence b (n_b history rows followed by
 * M_b = num_targets[b] candidate rows) the last min(n_b, keep) history rows and all candidates survive, in
 * order, packed sequence after sequence; dropped rows get a zero gradient.  Rows are opaque: row_bytes
 * bytes each (any dtype, any width), consecutive rows *_stride_bytes apart.  row_bytes, the strides and the
 * data pointers must be multiples of 16 (HSTU_ERR_SHAPE otherwise); strides >= row_bytes.
 *
 * hstu_truncate_offsets: out_offsets DEVICE int32[B+1] receives the offsets of the truncated batch
 *   (num_targets DEVICE int32[B] or NULL = no candidates; keep >= 0).
 * hstu_truncate_fwd: y row r = the r-th surviving row of x.  y has room for y_rows rows; rows at or beyond
 *   out_offsets[B] are not written, and nothing is written beyond y_rows (a bound such as
 *   min(T, B * (keep + max M)) is always enough).  out_offsets must come from hstu_truncate_offsets.
 * hstu_truncate_bwd: dx [T rows] is fully overwritten: the gradient row of every surviving row, zero for
 *   every dropped row.
 * All three enqueue one kernel on `stream`; nothing is allocated; B = 0 or T = 0 is valid.
 */
int hstu_truncate_offsets(int32_t batch, int32_t keep, const int32_t* seq_offsets, const int32_t* num_targets,
                          int32_t* out_offsets, void* stream);
int hstu_truncate_fwd(int32_t batch, const int32_t* seq_offsets, const int32_t* out_offsets, int64_t row_bytes,
                      const void* x, int64_t x_stride_bytes, void* y, int64_t y_stride_bytes, int64_t y_rows,
                      void* stream);
int hstu_truncate_bwd(int32_t batch, int64_t total_tokens, const int32_t* seq_offsets, const int32_t* out_offsets,
                      int64_t row_bytes, const void* dy, int64_t dy_stride_bytes, void* dx, int64_t dx_stride_bytes,
                      void* stream);

/*
 * One whole HSTU layer (paper Eq. 1-5) with the selective activation rematerialisation of Section 4.2.2
 * (layer pseudocode of the appendix).  For token rows Z [T, E] of the jagged batch described by `attn`:
 *   X = LayerNorm_E(Z) * norm_w                       (Eq. 1; weight only, biased variance, eps inside the root)
 *   [U V Q K] = SiLU(X W1^T)                          (Eq. 2; W1 [4*H*d, E] row-major, rows [0, H*d) give U, then V, Q, K)
 *   A = attention(Q, K, V)                            (Eq. 3, as hstu_attn_fwd with the mask/bias fields of `attn`)
 *   Y = LayerNorm_{H*d}(A) * gated_norm_w (.) U       (Eq. 4 before f2, as hstu_gated_norm_fwd without beta)
 *   out = Y W2^T + Z                                  (f2 as one linear map W2 [E, H*d] row-major, Eq. 5 residual)
 * Only bf16 (attn.dtype = HSTU_BF16): z, out, u_saved, attn_saved, dout, dz, w1, w2 are bf16 and contiguous
 * ([T, E] or [T, H*d]); norm_w, gated_norm_w and every weight gradient are fp32.  attn.row_stride_* are ignored
 * (the layer places Q, K, V in one [T, 4*H*d] buffer); attn.d_rab_table, when set, receives the bias-table
 * gradient in hstu_layer_bwd.  E: a multiple of 8, at most 8192; H*d at most 8192.
 *
 * The forward writes `out` and what the backward needs besides Z and the weights: u_saved [T, H*d],
 * attn_saved [T, H*d], mean and rstd of the input norm (fp32 [T]); V, Q, K, X and Y live in the workspace
 * and are dropped.  The backward rebuilds them (X from the saved statistics, U V Q K by the same GEMM, Y inside
 * the gated norm's backward) and returns dz [T, E] (including the residual's share) and fp32 d_norm_w [E],
 * d_w1 [4*H*d, E], d_gated_norm_w [H*d], d_w2 [E, H*d], all overwritten.  dU, dV, dQ, dK are written
 * straight into the column blocks of one gradient buffer (no concatenation).
 *
 * The four projections run through hipBLASLt (plain library GEMMs); the first call on a device creates a
 * hipBLASLt handle.  The GEMM kernels are chosen once per SHAPE CLASS, which is the layer's dimensions together with
 * the token count T rounded up to a power of two: the first call of a class runs the library's candidate kernels on
 * `stream`, waits for them and keeps the fastest (that call allocates inside the GEMM library, blocks the host and
 * must not be captured into a graph; hstu_layer_gemm_tunings counts these events).  Every later call of the class,
 * whatever its exact T, only builds its descriptors on the host and enqueues.  Not thread-safe.
 * HSTU_ERR_UNSUPPORTED if the library has no kernel for a shape.
 * T = 0: the forward writes nothing, the backward zeroes the weight gradients.
 */
typedef struct hstu_layer_params {
  hstu_attn_params attn;      /* the jagged batch, mask, bias and scales; see above for the ignored fields */
  int32_t embed_dim;          /* E */
  float norm_eps;             /* eps of the input norm */
  float gated_norm_eps;       /* eps of the gated norm */
  const float* norm_w;        /* DEVICE fp32[E] */
  const void* w1;             /* DEVICE bf16 [4*H*d, E] */
  const float* gated_norm_w;  /* DEVICE fp32[H*d] */
  const void* w2;             /* DEVICE bf16 [E, H*d] */
  /* Optional FP8 forward (Section 4.2.2: both projections of the forward in FP8, everything else bf16).  When all four
   * are given, hstu_layer_fwd quantises X and Y row-wise inside the two norm kernels (as hstu_norm_quant_fp8) and runs
   * the projections as hstu_fp8_gemm_bias2d on these weights (the residual Z as the two-dimensional additive operand of
   * the second); E and H*d must then be in {128, 256, 512, 1024}.  hstu_layer_bwd then rematerialises U, V, Q, K with the
   * same FP8 projection (so that it differentiates at the forward's activations) and takes every gradient in bf16 with
   * w1, w2 (straight-through: the quantisation is treated as the identity).  All four NULL: bf16 throughout. */
  const void* w1_q;           /* DEVICE E4M3 codes [4*H*d, E], row-wise quantised w1 (hstu_norm_quant_fp8 with gamma = NULL) */
  const float* w1_scale;      /* DEVICE fp32 [4*H*d] */
  const void* w2_q;           /* DEVICE E4M3 codes [E, H*d] */
  const float* w2_scale;      /* DEVICE fp32 [E] */
} hstu_layer_params;

/* Bytes of device scratch (256-byte aligned) for hstu_layer_fwd (for_backward = 0) or hstu_layer_bwd; 0 for an
 * invalid description.  Forward: X, the projection and Y (T*(E + 5*H*d) bf16), backward: 17 such [T, 512]-sized
 * buffers at E = H*d = 512; both include the attention workspace and 64 MiB offered to the GEMM library. */
size_t hstu_layer_workspace_bytes(const hstu_layer_params* p, int for_backward);

int hstu_layer_fwd(const hstu_layer_params* p, const void* z, void* out, void* u_saved, void* attn_saved, float* mean,
                   float* rstd, void* workspace, size_t workspace_bytes, void* stream);

int hstu_layer_bwd(const hstu_layer_params* p, const void* z, const void* u_saved, const void* attn_saved,
                   const float* mean, const float* rstd, const void* dout, void* dz, float* d_norm_w, float* d_w1,
                   float* d_gated_norm_w, float* d_w2, void* workspace, size_t workspace_bytes, void* stream);

/* How many times this process has timed GEMM candidates so far (once per GEMM of a new shape class, see above): a
 * caller that must not block, or that is about to capture a graph, can check that a warm-up call left nothing to tune. */
int64_t hstu_layer_gemm_tunings(void);

/*
 * FP8 around the layer's two projections (paper Section 4.2.2, "Mixed-Precision Training and Inference", and the FP8
 * benchmarks of its appendix).  Format: OCP FP8 E4M3 (largest finite value 448), one fp32 scale per row:
 *   scale = amax / 448 (1 for a row of zeros),  code = nearest E4M3 value, ties to even, of  y * (448 / amax),
 * both divisions and the multiplication in fp32.
 *
 * hstu_norm_quant_fp8: the scaling and quantisation fused behind the norm that precedes a projection (Eq. 1: u = NULL;
 *   Eq. 4: u = the gate).  y = (LayerNorm_D(a) * gamma + beta) * u as hstu_gated_norm_fwd computes it, never written;
 *   q: E4M3 codes [T, D] (8-byte aligned), q_scale: fp32 [T]; mean, rstd: fp32 [T] or NULL.
 *   gamma = NULL: no normalisation, y = a (times u when given): plain row-wise quantisation, e.g. of a weight matrix
 *   [N, K] with one scale per output feature (beta must be NULL then).  a, u: [T, D] contiguous of `dtype`.
 *
 * hstu_fp8_gemm_bias2d: the projection on quantised operands with a two-dimensional additive operand
 *   (D = A B + C with C in R^{m x n}: the post-attention projection accumulated with the residual, Eq. 5):
 *     d[m, n] = a_scale[m] * b_scale[n] * sum_k a_q[m, k] * b_q[n, k]  +  c[m, n]
 *   a_q: codes [M, K]; b_q: codes [N, K] (weights stored [out, in]); c: bf16 [M, N] or NULL; d: bf16 [M, N]; products
 *   exact, fp32 accumulation, one rounding to bf16.  K in {128, 256, 512, 1024}, N a multiple of 64 (else
 *   HSTU_ERR_UNSUPPORTED); all pointers 16-byte aligned.  c may be d (in-place accumulation).
 */
int hstu_norm_quant_fp8(int64_t T, int32_t D, int32_t dtype, const void* a, const void* u, const float* gamma,
                        const float* beta, float eps, void* q, float* q_scale, float* mean, float* rstd, void* stream);
int hstu_fp8_gemm_bias2d(int64_t M, int32_t N, int32_t K, const void* a_q, const float* a_scale, const void* b_q,
                         const float* b_scale, const void* c, void* d, void* stream);

/*
 * Load-Balanced Stochastic Length (paper Section 4.1, "Load-Balanced Stochastic Length", and Alg. 1 of its appendix):
 * the length sampler that keeps the attention load of the ranks of a data-parallel job level.  HOST code on HOST
 * pointers: it deals in sequence lengths, never touches a GPU, and plays all `world_size` ranks in one process (the
 * one number the ranks exchange, a mean load, is a plain mean here).  Load of a sequence of n items: n^gamma; load of a
 * rank: the sum over its batch.
 *
 * Stochastic Length with sampling length sl_len (= L^(alpha/2) in the paper's notation): a sequence of n <= sl_len items
 * is left alone; a longer one stays whole with probability hstu_lbsl_weight(n) = (sl_len / n)^2 and is cut to sl_len
 * items otherwise.  hstu_lbsl_expected_load(n) = w n^gamma + (1 - w) min(n, sl_len)^gamma is the load it leaves on
 * average.
 *
 * hstu_lbsl_step runs one training step of Alg. 1 for every rank.  rank_offsets [world_size + 1] (starting at 0,
 * non-decreasing) delimits the ranks' batches inside lengths [total] (raw lengths >= 0) and uniforms [total] (one number
 * in (0, 1] per sequence, drawn by the caller).  Every rank first adds the expected plain-SL load of its batch to
 * state.rank_load[r].  During the first warmup_steps steps it then applies plain SL (sequence u stays whole iff
 * uniforms[u] < weight).  Afterwards it visits its batch in a weighted random order without replacement (weights = the
 * weights above, drawn with exponential clocks: ascending -ln(uniforms[u]) / weight, ties by index) and leaves u whole
 * while the load so added, n^gamma - min(n, sl_len)^gamma each, stays within state.target minus the load of the batch
 * with every long sequence cut; the rest is cut to sl_len.  Outputs: new_lengths [total], unsampled [total] (1 = left
 * whole), realised_load [world_size] (sum of new_length^gamma; may be NULL).  At the end of step warmup_steps the target
 * becomes the mean of rank_load over ranks and warm-up steps and the accumulators restart; after the warm-up the same
 * happens at every step that is a multiple of recal_interval (mean over ranks and recal_interval steps).
 * hstu_lbsl_init clears a state whose rank_load the caller has pointed at world_size doubles.
 * Errors: HSTU_ERR_NULL, HSTU_ERR_SHAPE (world_size, warmup_steps, recal_interval, sl_len < 1, gamma not positive and
 * finite, offsets not as described, a negative length, a uniform outside (0, 1]); nothing is written then.  The step
 * allocates host memory for its sort; not thread-safe per state.
 *
 * hstu_lbsl_fit_gamma: the exponent that a measured cost curve implies, the least-squares slope of log(times[i]) against
 * log(lengths[i]) over n >= 2 points (all > 0, at least two distinct lengths).
 */
typedef struct hstu_lbsl_config {
  int32_t world_size;      /* R */
  int32_t warmup_steps;    /* T_warm */
  int32_t recal_interval;  /* T_recal */
  int32_t sl_len;          /* l_SL */
  double gamma;            /* load exponent */
} hstu_lbsl_config;
typedef struct hstu_lbsl_state {
  int64_t step;            /* steps done so far */
  double target;           /* the target load; 0 until the warm-up ends */
  double* rank_load;       /* HOST double[world_size], owned by the caller: the accumulators l_r */
} hstu_lbsl_state;
double hstu_lbsl_weight(int32_t n, int32_t sl_len);
double hstu_lbsl_expected_load(int32_t n, int32_t sl_len, double gamma);
int hstu_lbsl_init(const hstu_lbsl_config* cfg, hstu_lbsl_state* state);
int hstu_lbsl_step(const hstu_lbsl_config* cfg, hstu_lbsl_state* state, const int32_t* rank_offsets, const int32_t* lengths,
                   const double* uniforms, int32_t* new_lengths, uint8_t* unsampled, double* realised_load);
int hstu_lbsl_fit_gamma(int32_t n, const double* lengths, const double* times, double* gamma);

/* Human-readable name of a status code (static storage). */
const char* hstu_status_string(int status);

/* Statistics of the last tile schedule written by hstu_attn_fwd/bwd into `workspace`
 * (valid after the stream has been synchronised): HOST out[0] = scheduled row blocks x heads,
 * out[1] = scheduled (row block, column block) tiles x heads, out[2] = tiles a dense L x L
 * grid would have.  Reads device memory with a blocking copy; for reporting only.
 * Returns HSTU_ERR_SHAPE (out[0] = 0) when the scheduler of that call found the DEVICE copies of seq_offsets / num_targets
 * inconsistent with the description (offsets not starting at 0, decreasing, a sequence longer than max_seqlen, an end past
 * total_tokens, a candidate count outside [0, L]): such a call computes nothing and leaves every output untouched, instead of
 * addressing rows outside the tensors (the host cannot see device-side offsets when seq_offsets_host is NULL). */
int hstu_attn_schedule_stats(const hstu_attn_params* p, const void* workspace, int for_backward, int64_t out[3]);

/* Per-kernel timing for benchmarks (not part of the paper's method).  While enabled, every kernel
 * launch made by the entry points above is bracketed by HIP events on its stream (up to 64 launches
 * between two reads).  hstu_profile_read waits for those events and returns the number of entries
 * written: names[i] (static strings: "attn_fwd", "attn_bwd_dq", "attn_bwd_dkdv", "gated_norm_fwd",
 * "gated_norm_bwd" [the latter includes its column-sum kernel], "schedule_fwd", "schedule_bwd" [both backward lists, one launch], "bias_expand", "dbias_zero", "dbias_reduce",
 * "truncate_offsets", "truncate_fwd", "truncate_bwd", and from the layer entry points "layer_norm_fwd",
 * "gemm_uvqk", "silu_fwd", "gemm_out", "gemm_dy", "gemm_dw2", "gemm_dxn", "gemm_dw1", "layer_norm_bwd",
 * and "norm_quant_fp8", "fp8_gemm_bias2d";
 * "attn_bwd_dkdv" includes the kernel that combines the partial sums of cut key blocks) and
 * ms[i] = elapsed milliseconds.  HOST arrays.  Not thread-safe; enable(1) creates the events once. */
int hstu_profile_enable(int on);
int hstu_profile_read(int max_entries, const char** names, float* ms);

#ifdef __cplusplus
}
#endif
#endif /* HSTU_ATTN_H */
