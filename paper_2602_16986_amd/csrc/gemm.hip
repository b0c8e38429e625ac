// Plain bf16 GEMMs of the layer's two projections and their backward, through hipBLASLt (library GEMMs: the
// contractions here are ordinary dense products with at most a residual added).  Row-major operands are handed to
// the column-major library as their transposes: D^T = op(B)^T op(A)^T.
// Host code only.  One hipBLASLt handle per device and a small cache of matmul plans, created on first use (making
// a plan times the library's candidate kernels on the stream and waits for them); not thread-safe.
#include <hipblaslt/hipblaslt.h>

#include "hstu_kernels.h"

namespace hstu {
namespace {

struct Plan {
  int device, op; int64_t M, N, K, lda, ldb, ldc, ldd; bool residual, d_fp32;
  hipblasLtMatmulDesc_t desc;
  hipblasLtMatrixLayout_t la, lb, lc, ld;
  hipblasLtMatmulAlgo_t algo;
  size_t ws_needed;
};
constexpr int kMaxPlans = 64;
Plan g_plans[kMaxPlans];
int g_nplans = 0;
hipblasLtHandle_t g_handle[64];
bool g_has_handle[64];

#define LT(x) do { if ((x) != HIPBLAS_STATUS_SUCCESS) return -1; } while (0)

constexpr int kCandidates = 16;   // heuristic answers timed when a plan is made
constexpr int kTrialRuns = 3;

int make_plan(Plan& pl, const void* A, const void* B, const void* C, void* D, void* ws, size_t ws_bytes, hipStream_t stream) {
  hipblasLtHandle_t h = g_handle[pl.device];
  // column-major problem m = N, n = M: first operand is B, second is A
  hipblasOperation_t ta, tb;
  int64_t a_rows, a_cols, b_rows, b_cols;
  if (pl.op == kGemmNT) {        // B row-major [N, K] = col-major K x N -> transposed; A row-major [M, K] = col-major K x M
    ta = HIPBLAS_OP_T; tb = HIPBLAS_OP_N; a_rows = pl.K; a_cols = pl.N; b_rows = pl.K; b_cols = pl.M;
  } else if (pl.op == kGemmNN) { // B row-major [K, N] = col-major N x K; A as above
    ta = HIPBLAS_OP_N; tb = HIPBLAS_OP_N; a_rows = pl.N; a_cols = pl.K; b_rows = pl.K; b_cols = pl.M;
  } else {                       // TN: B row-major [K, N] = col-major N x K; A row-major [K, M] = col-major M x K -> transposed
    ta = HIPBLAS_OP_N; tb = HIPBLAS_OP_T; a_rows = pl.N; a_cols = pl.K; b_rows = pl.M; b_cols = pl.K;
  }
  LT(hipblasLtMatmulDescCreate(&pl.desc, HIPBLAS_COMPUTE_32F, HIP_R_32F));
  LT(hipblasLtMatmulDescSetAttribute(pl.desc, HIPBLASLT_MATMUL_DESC_TRANSA, &ta, sizeof(ta)));
  LT(hipblasLtMatmulDescSetAttribute(pl.desc, HIPBLASLT_MATMUL_DESC_TRANSB, &tb, sizeof(tb)));
  const hipDataType dt = pl.d_fp32 ? HIP_R_32F : HIP_R_16BF;
  LT(hipblasLtMatrixLayoutCreate(&pl.la, HIP_R_16BF, a_rows, a_cols, pl.ldb));
  LT(hipblasLtMatrixLayoutCreate(&pl.lb, HIP_R_16BF, b_rows, b_cols, pl.lda));
  LT(hipblasLtMatrixLayoutCreate(&pl.lc, dt, pl.N, pl.M, pl.residual ? pl.ldc : pl.ldd));
  LT(hipblasLtMatrixLayoutCreate(&pl.ld, dt, pl.N, pl.M, pl.ldd));
  hipblasLtMatmulPreference_t pref;
  LT(hipblasLtMatmulPreferenceCreate(&pref));
  LT(hipblasLtMatmulPreferenceSetAttribute(pref, HIPBLASLT_MATMUL_PREF_MAX_WORKSPACE_BYTES, &ws_bytes, sizeof(ws_bytes)));
  hipblasLtMatmulHeuristicResult_t res[kCandidates];
  int found = 0;
  const hipblasStatus_t st = hipblasLtMatmulAlgoGetHeuristic(h, pl.desc, pl.la, pl.lb, pl.lc, pl.ld, pref, kCandidates, res, &found);
  hipblasLtMatmulPreferenceDestroy(pref);
  if (st != HIPBLAS_STATUS_SUCCESS || found < 1) return -2;
  // The library's first answer is not always its fastest kernel for these shapes (the split-K weight-gradient products
  // differ by up to 5x between candidates): run every candidate on the real operands and keep the fastest.  The
  // product is written kTrialRuns + 1 times per candidate into D, which the caller is about to overwrite anyway.
  int best = 0;
  if (found > 1) {
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return -1;
    const float alpha = 1.0f, beta = pl.residual ? 1.0f : 0.0f;
    float best_ms = 0.f;
    bool have = false;
    for (int i = 0; i < found; ++i) {
      if (res[i].workspaceSize > ws_bytes) continue;
      bool ok = true;
      for (int r = 0; r <= kTrialRuns && ok; ++r) {
        if (r == 1) ok = hipEventRecord(e0, stream) == hipSuccess;
        ok = ok && hipblasLtMatmul(h, pl.desc, &alpha, B, pl.la, A, pl.lb, &beta, pl.residual ? C : D, pl.lc, D, pl.ld, &res[i].algo, ws,
                                   ws_bytes, stream) == HIPBLAS_STATUS_SUCCESS;
      }
      ok = ok && hipEventRecord(e1, stream) == hipSuccess && hipEventSynchronize(e1) == hipSuccess;
      float ms = 0.f;
      if (!ok || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) continue;
      if (!have || ms < best_ms) { have = true; best_ms = ms; best = i; }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (!have) return -2;
  }
  pl.algo = res[best].algo;
  pl.ws_needed = res[best].workspaceSize;
  return 0;
}

}  // namespace

int gemm_bf16(int op, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B, int64_t ldb, const void* C,
              int64_t ldc, void* D, int64_t ldd, bool d_fp32, void* ws, size_t ws_bytes, hipStream_t stream) {
  if (M <= 0 || N <= 0 || K <= 0) return -1;
  int device = 0;
  if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= 64) return -1;
  if (!g_has_handle[device]) {
    if (hipblasLtCreate(&g_handle[device]) != HIPBLAS_STATUS_SUCCESS) return -1;
    g_has_handle[device] = true;
  }
  const bool residual = C != nullptr;
  Plan* pl = nullptr;
  for (int i = 0; i < g_nplans; ++i) {
    Plan& c = g_plans[i];
    if (c.device == device && c.op == op && c.M == M && c.N == N && c.K == K && c.lda == lda && c.ldb == ldb && c.ldd == ldd &&
        c.residual == residual && (!residual || c.ldc == ldc) && c.d_fp32 == d_fp32 && c.ws_needed <= ws_bytes) {
      pl = &c;
      break;
    }
  }
  if (!pl) {
    if (g_nplans == kMaxPlans) {                       // drop the oldest plan
      Plan& o = g_plans[0];
      hipblasLtMatmulDescDestroy(o.desc);
      hipblasLtMatrixLayoutDestroy(o.la); hipblasLtMatrixLayoutDestroy(o.lb);
      hipblasLtMatrixLayoutDestroy(o.lc); hipblasLtMatrixLayoutDestroy(o.ld);
      for (int i = 1; i < kMaxPlans; ++i) g_plans[i - 1] = g_plans[i];
      --g_nplans;
    }
    Plan np = {};
    np.device = device; np.op = op; np.M = M; np.N = N; np.K = K; np.lda = lda; np.ldb = ldb; np.ldc = ldc; np.ldd = ldd;
    np.residual = residual; np.d_fp32 = d_fp32;
    const int rc = make_plan(np, A, B, C, D, ws, ws_bytes, stream);
    if (rc != 0) return rc;
    g_plans[g_nplans] = np;
    pl = &g_plans[g_nplans++];
  }
  const float alpha = 1.0f, beta = residual ? 1.0f : 0.0f;
  const hipblasStatus_t st = hipblasLtMatmul(g_handle[device], pl->desc, &alpha, B, pl->la, A, pl->lb, &beta, residual ? C : D, pl->lc,
                                             D, pl->ld, &pl->algo, ws, ws_bytes, stream);
  return st == HIPBLAS_STATUS_SUCCESS ? 0 : -1;
}

}  // namespace hstu
