// Plain bf16 GEMMs of the layer's two projections and their backward, through hipBLASLt (library GEMMs: the
// contractions here are ordinary dense products with at most a residual added).  Row-major operands are handed to
// the column-major library as their transposes: D^T = op(B)^T op(A)^T.
// Host code only.  One hipBLASLt handle per device, created on first use; not thread-safe.
//
// Two caches.  The token count of a jagged batch differs from call to call, so what is expensive, choosing the kernel by
// timing the library's candidates on the stream (which waits for them), is done once per SHAPE CLASS: operation, the
// dimensions that do not depend on the batch, leading dimensions, residual, output type, and the token dimension
// rounded up to a power of two.  A class remembers the index of the kernel that won.  A new exact shape of a known
// class only builds its descriptors (host work, nothing is launched or waited for), asks the library whether that
// kernel supports it and otherwise takes the heuristic's first answer untimed.  Exact shapes are kept in a small
// least-recently-made list so that a repeated shape costs a lookup.
#include <hipblaslt/hipblaslt.h>
#include <hipblaslt/hipblaslt-ext.hpp>

#include <vector>

#include "hstu_kernels.h"

namespace hstu {
namespace {

struct Shape {
  int device, op; int64_t M, N, K, lda, ldb, ldc, ldd; bool residual, d_fp32, silu;
};
struct Plan {
  Shape s;
  hipblasLtMatmulDesc_t desc;
  hipblasLtMatrixLayout_t la, lb, lc, ld;
  hipblasLtMatmulAlgo_t algo;
  size_t ws_needed;
};
struct TunedClass {                      // Shape with the token dimension replaced by its power-of-two bucket
  Shape s;
  int algo_index;                        // the library's index of the kernel that won the timing (-1: none usable)
};
constexpr int kMaxPlans = 64, kMaxClasses = 64;
Plan g_plans[kMaxPlans];
int g_nplans = 0;
TunedClass g_classes[kMaxClasses];
int g_nclasses = 0;
long g_tunings = 0;                       // how many times candidates were timed (each one blocks the host)
hipblasLtHandle_t g_handle[64];
bool g_has_handle[64];

constexpr int kCandidates = 16;   // heuristic answers timed when a class is tuned
constexpr int kTrialRuns = 3;

int64_t bucket_of(int64_t n) { int64_t b = 1; while (b < n) b <<= 1; return b; }
// The token count is M for the projections and their input gradients, and the contraction length K for the weight gradients.
Shape class_of(Shape s) {
  if (s.op == kGemmTN) s.K = bucket_of(s.K); else s.M = bucket_of(s.M);
  return s;
}
bool same(const Shape& a, const Shape& b) {
  return a.device == b.device && a.op == b.op && a.M == b.M && a.N == b.N && a.K == b.K && a.lda == b.lda && a.ldb == b.ldb &&
         a.ldd == b.ldd && a.residual == b.residual && (!a.residual || a.ldc == b.ldc) && a.d_fp32 == b.d_fp32 && a.silu == b.silu;
}
void destroy(Plan& pl) {
  if (pl.desc) hipblasLtMatmulDescDestroy(pl.desc);
  if (pl.la) hipblasLtMatrixLayoutDestroy(pl.la);
  if (pl.lb) hipblasLtMatrixLayoutDestroy(pl.lb);
  if (pl.lc) hipblasLtMatrixLayoutDestroy(pl.lc);
  if (pl.ld) hipblasLtMatrixLayoutDestroy(pl.ld);
  pl.desc = nullptr; pl.la = pl.lb = pl.lc = pl.ld = nullptr;
}

// Descriptors of one exact shape.  Column-major problem m = N, n = M: the library's first operand is B, its second is A.
bool describe(Plan& pl) {
  const Shape& s = pl.s;
  hipblasOperation_t ta, tb;
  int64_t a_rows, a_cols, b_rows, b_cols;
  if (s.op == kGemmNT) {        // B row-major [N, K] = col-major K x N -> transposed; A row-major [M, K] = col-major K x M
    ta = HIPBLAS_OP_T; tb = HIPBLAS_OP_N; a_rows = s.K; a_cols = s.N; b_rows = s.K; b_cols = s.M;
  } else if (s.op == kGemmNN) { // B row-major [K, N] = col-major N x K; A as above
    ta = HIPBLAS_OP_N; tb = HIPBLAS_OP_N; a_rows = s.N; a_cols = s.K; b_rows = s.K; b_cols = s.M;
  } else {                      // TN: B row-major [K, N] = col-major N x K; A row-major [K, M] = col-major M x K -> transposed
    ta = HIPBLAS_OP_N; tb = HIPBLAS_OP_T; a_rows = s.N; a_cols = s.K; b_rows = s.M; b_cols = s.K;
  }
  const hipDataType dt = s.d_fp32 ? HIP_R_32F : HIP_R_16BF;
  const hipblasLtEpilogue_t epi = s.silu ? HIPBLASLT_EPILOGUE_SWISH_EXT : HIPBLASLT_EPILOGUE_DEFAULT;   // Swish(x, 1) = x sigmoid(x) = SiLU
  const bool ok =
      hipblasLtMatmulDescCreate(&pl.desc, HIPBLAS_COMPUTE_32F, HIP_R_32F) == HIPBLAS_STATUS_SUCCESS &&
      hipblasLtMatmulDescSetAttribute(pl.desc, HIPBLASLT_MATMUL_DESC_EPILOGUE, &epi, sizeof(epi)) == HIPBLAS_STATUS_SUCCESS &&
      hipblasLtMatmulDescSetAttribute(pl.desc, HIPBLASLT_MATMUL_DESC_TRANSA, &ta, sizeof(ta)) == HIPBLAS_STATUS_SUCCESS &&
      hipblasLtMatmulDescSetAttribute(pl.desc, HIPBLASLT_MATMUL_DESC_TRANSB, &tb, sizeof(tb)) == HIPBLAS_STATUS_SUCCESS &&
      hipblasLtMatrixLayoutCreate(&pl.la, HIP_R_16BF, a_rows, a_cols, s.ldb) == HIPBLAS_STATUS_SUCCESS &&
      hipblasLtMatrixLayoutCreate(&pl.lb, HIP_R_16BF, b_rows, b_cols, s.lda) == HIPBLAS_STATUS_SUCCESS &&
      hipblasLtMatrixLayoutCreate(&pl.lc, dt, s.N, s.M, s.residual ? s.ldc : s.ldd) == HIPBLAS_STATUS_SUCCESS &&
      hipblasLtMatrixLayoutCreate(&pl.ld, dt, s.N, s.M, s.ldd) == HIPBLAS_STATUS_SUCCESS;
  if (!ok) destroy(pl);
  return ok;
}

// The library's candidates for this shape, best guess first.  0 on failure.
int candidates(const Plan& pl, size_t ws_bytes, hipblasLtMatmulHeuristicResult_t* res) {
  hipblasLtMatmulPreference_t pref;
  if (hipblasLtMatmulPreferenceCreate(&pref) != HIPBLAS_STATUS_SUCCESS) return 0;
  int found = 0;
  const bool ok =
      hipblasLtMatmulPreferenceSetAttribute(pref, HIPBLASLT_MATMUL_PREF_MAX_WORKSPACE_BYTES, &ws_bytes, sizeof(ws_bytes)) == HIPBLAS_STATUS_SUCCESS &&
      hipblasLtMatmulAlgoGetHeuristic(g_handle[pl.s.device], pl.desc, pl.la, pl.lb, pl.lc, pl.ld, pref, kCandidates, res, &found) == HIPBLAS_STATUS_SUCCESS;
  hipblasLtMatmulPreferenceDestroy(pref);
  return ok ? found : 0;
}

// Times every candidate on the real operands and returns the position of the fastest (-1: none ran).  The library's
// first answer is not always its fastest kernel for these shapes (the split-K weight-gradient products differ by up to
// 5x between candidates).  The product is written kTrialRuns + 1 times per candidate into D, which the caller is about
// to overwrite anyway.  Blocks the host until the trials are done.
int fastest(const Plan& pl, const hipblasLtMatmulHeuristicResult_t* res, int found, const void* A, const void* B, const void* C, void* D,
            void* ws, size_t ws_bytes, hipStream_t stream) {
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return -1;
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return -1; }
  ++g_tunings;
  const float alpha = 1.0f, beta = pl.s.residual ? 1.0f : 0.0f;
  float best_ms = 0.f;
  int best = -1;
  for (int i = 0; i < found; ++i) {
    if (res[i].workspaceSize > ws_bytes) continue;
    bool ok = true;
    for (int r = 0; r <= kTrialRuns && ok; ++r) {
      if (r == 1) ok = hipEventRecord(e0, stream) == hipSuccess;
      ok = ok && hipblasLtMatmul(g_handle[pl.s.device], pl.desc, &alpha, B, pl.la, A, pl.lb, &beta, pl.s.residual ? C : D, pl.lc, D, pl.ld,
                                 &res[i].algo, ws, ws_bytes, stream) == HIPBLAS_STATUS_SUCCESS;
    }
    ok = ok && hipEventRecord(e1, stream) == hipSuccess && hipEventSynchronize(e1) == hipSuccess;
    float ms = 0.f;
    if (!ok || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) continue;
    if (best < 0 || ms < best_ms) { best_ms = ms; best = i; }
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  return best;
}

// Fills pl.algo / pl.ws_needed for a described shape.  A class seen before contributes its tuned kernel without any
// launch; a new class is tuned now.
int choose_algo(Plan& pl, const void* A, const void* B, const void* C, void* D, void* ws, size_t ws_bytes, hipStream_t stream) {
  const Shape cls = class_of(pl.s);
  TunedClass* tc = nullptr;
  for (int i = 0; i < g_nclasses; ++i)
    if (same(g_classes[i].s, cls)) { tc = &g_classes[i]; break; }
  hipblasLtHandle_t h = g_handle[pl.s.device];
  if (tc && tc->algo_index >= 0) {
    std::vector<int> idx = {tc->algo_index};
    std::vector<hipblasLtMatmulHeuristicResult_t> got;
    const float alpha = 1.0f, beta = pl.s.residual ? 1.0f : 0.0f;
    if (hipblaslt_ext::getAlgosFromIndex(h, idx, got) == HIPBLAS_STATUS_SUCCESS && !got.empty()) {
      size_t need = 0;
      if (hipblaslt_ext::matmulIsAlgoSupported(h, pl.desc, &alpha, pl.la, pl.lb, &beta, pl.lc, pl.ld, got[0].algo, need) == HIPBLAS_STATUS_SUCCESS &&
          need <= ws_bytes) {
        pl.algo = got[0].algo;
        pl.ws_needed = need;
        return 0;
      }
    }
  }
  hipblasLtMatmulHeuristicResult_t res[kCandidates];
  const int found = candidates(pl, ws_bytes, res);
  if (found < 1) return -2;
  int best = 0;
  if (!tc) {                                             // a class met for the first time: time its candidates, remember the winner
    if (found > 1) best = fastest(pl, res, found, A, B, C, D, ws, ws_bytes, stream);
    if (best < 0) return -2;
    if (g_nclasses == kMaxClasses) {                     // drop the oldest class
      for (int i = 1; i < kMaxClasses; ++i) g_classes[i - 1] = g_classes[i];
      --g_nclasses;
    }
    g_classes[g_nclasses++] = {cls, hipblaslt_ext::getIndexFromAlgo(res[best].algo)};
  } else {                                               // tuned kernel unusable for this member: the heuristic's first that fits, untimed
    while (best < found && res[best].workspaceSize > ws_bytes) ++best;
    if (best == found) return -2;
  }
  pl.algo = res[best].algo;
  pl.ws_needed = res[best].workspaceSize;
  return 0;
}

}  // namespace

long gemm_bf16_tunings() { return g_tunings; }

int gemm_bf16(int op, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B, int64_t ldb, const void* C,
              int64_t ldc, void* D, int64_t ldd, bool d_fp32, void* ws, size_t ws_bytes, hipStream_t stream, bool silu) {
  if (M <= 0 || N <= 0 || K <= 0) return -1;
  int device = 0;
  if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= 64) return -1;
  if (!g_has_handle[device]) {
    if (hipblasLtCreate(&g_handle[device]) != HIPBLAS_STATUS_SUCCESS) return -1;
    g_has_handle[device] = true;
  }
  const bool residual = C != nullptr;
  const Shape shape = {device, op, M, N, K, lda, ldb, ldc, ldd, residual, d_fp32, silu};
  Plan* pl = nullptr;
  for (int i = 0; i < g_nplans; ++i)
    if (same(g_plans[i].s, shape) && g_plans[i].ws_needed <= ws_bytes) { pl = &g_plans[i]; break; }
  if (!pl) {
    Plan np = {};
    np.s = shape;
    if (!describe(np)) return -1;
    const int rc = choose_algo(np, A, B, C, D, ws, ws_bytes, stream);
    if (rc != 0) { destroy(np); return rc; }
    if (g_nplans == kMaxPlans) {                       // drop the oldest plan
      destroy(g_plans[0]);
      for (int i = 1; i < kMaxPlans; ++i) g_plans[i - 1] = g_plans[i];
      --g_nplans;
    }
    g_plans[g_nplans] = np;
    pl = &g_plans[g_nplans++];
  }
  const float alpha = 1.0f, beta = residual ? 1.0f : 0.0f;
  const hipblasStatus_t st = hipblasLtMatmul(g_handle[device], pl->desc, &alpha, B, pl->la, A, pl->lb, &beta, residual ? C : D, pl->lc,
                                             D, pl->ld, &pl->algo, ws, ws_bytes, stream);
  return st == HIPBLAS_STATUS_SUCCESS ? 0 : -1;
}

}  // namespace hstu
