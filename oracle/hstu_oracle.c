/*
 * CPU fp64 oracle for the jagged HSTU attention layer.  TEST INFRASTRUCTURE ONLY:
 * it exists to check the HIP kernels; only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it.  It shares no code with the GPU path.
 *
 * Every function is the plain definition written out, in definition order, with
 * no blocking or fusion; OpenMP only distributes independent output rows.
 *
 *   attention   A = ( (SiLU(alpha Q K^T + bias) / N)  (.)  M ) V        (paper Eq. 3,
 *               Section 4.2.1 for the causal and semi-local masks M; the 1/N factor,
 *               the relative-position bias and the target-aware rows are readings
 *               fixed by the benchmark spec, the paper's equations carry none of them)
 *   epilogue    Y = (LayerNorm_D(A) * gamma + beta) (.) U                (paper Eq. 4:
 *               Norm(A) (.) U; Section 4.2.2 calls the Norm a layer normalisation)
 *   backward    the derivatives of the two, with the op signatures of the appendix
 *               pseudocode: attention backward sees only dA, Q, K, V;
 *               gated-norm backward returns dA, dU and the weight gradient.
 *
 * Layout: Q, K, V, A, U, Y and their gradients are [T, H, d] row-major doubles
 * (token, head, feature); seq_offsets is int32[B+1].
 *
 * Mask (ordinary 0-based indexing, query row i, key j, inside one sequence of
 * length L whose last M tokens are candidates and n = L - M are history):
 *   hist(p, j) = j < n  &&  j <= p  &&  (K1 < 0 || p - j < K1 || j < K2)
 *   history row  i < n :  visible(i, j) = hist(i, j)            distance  i - j
 *   candidate row i >= n: visible(i, j) = (j == i) || hist(n, j) distance  (j == i) ? 0 : n - j
 * This is the paper's flipped-index mask (local band  L-K1 <= i+j <= L,  global
 * j <= K2 and j <= L-i) after substituting query time t = L - i, with the
 * diagonal visible, a window of exactly K1 keys including the query itself and a
 * prefix of exactly K2 keys.  K1 < 0 means no local limit (dense causal); K1 = 0
 * with K2 > 0 is the paper's global-only ablation (Section 5.3).
 *
 * Parity pins: see tests/test_oracle_pins.py.  Unpinned against the paper (it
 * gives no definition): the spacing of the bias buckets (they arrive as data),
 * eps and the gamma/beta convention of the layer norm.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double sigmoid(double x) { return 1.0 / (1.0 + exp(-x)); }

/* bucket(delta) = max{ b : bounds[b] <= delta };  bounds[0] == 0 */
static int bucket_of(const int32_t *bounds, int nb, int delta) {
    int b = 0;
    for (int c = 1; c < nb; ++c)
        if (bounds[c] <= delta) b = c;
    return b;
}

/* visibility of key j from query i; writes the bias distance to *delta */
static int visible(int i, int j, int L, int M, int K1, int K2, int *delta) {
    const int n = L - M;
    if (i >= n && j == i) { *delta = 0; return 1; }   /* a candidate sees itself */
    const int p = i < n ? i : n;                        /* effective position */
    if (j >= n || j > p) return 0;
    if (!(K1 < 0 || p - j < K1 || j < K2)) return 0;
    *delta = p - j;
    return 1;
}

typedef struct {
    int B, H, d;
    const int32_t *offsets;      /* [B+1] */
    const int32_t *num_targets;  /* [B] or NULL */
    int K1, K2;
    double alpha, inv_n;
    const double *table;         /* [H, nb] or NULL */
    const int32_t *bounds;       /* [nb] */
    int nb;
} attn_desc;

static double score(const attn_desc *a, const double *Q, const double *K, int64_t tq, int64_t tk, int h, int delta) {
    const int d = a->d, H = a->H;
    const double *q = Q + (tq * H + h) * d, *k = K + (tk * H + h) * d;
    double s = 0.0;
    for (int c = 0; c < d; ++c) s += q[c] * k[c];
    s *= a->alpha;
    if (a->table) s += a->table[(int64_t)h * a->nb + bucket_of(a->bounds, a->nb, delta)];
    return s;
}

/* which sequence holds global token t */
static int seq_of(const attn_desc *a, int64_t t) {
    for (int b = 0; b < a->B; ++b)
        if (t >= a->offsets[b] && t < a->offsets[b + 1]) return b;
    return -1;
}

static void fwd_row(const attn_desc *a, const double *Q, const double *K, const double *V, int b, int i, double *out /* [H,d] */) {
    const int H = a->H, d = a->d;
    const int64_t base = a->offsets[b];
    const int L = a->offsets[b + 1] - a->offsets[b];
    const int M = a->num_targets ? a->num_targets[b] : 0;
    for (int h = 0; h < H; ++h) {
        double *o = out + (int64_t)h * d;
        for (int c = 0; c < d; ++c) o[c] = 0.0;
        for (int j = 0; j < L; ++j) {
            int delta;
            if (!visible(i, j, L, M, a->K1, a->K2, &delta)) continue;
            const double s = score(a, Q, K, base + i, base + j, h, delta);
            const double w = s * sigmoid(s) * a->inv_n;
            const double *v = V + ((base + j) * H + h) * d;
            for (int c = 0; c < d; ++c) o[c] += w * v[c];
        }
    }
}

static attn_desc make_desc(int B, int H, int d, const int32_t *offsets, const int32_t *num_targets, int K1, int K2,
                           double alpha, double inv_n, const double *table, const int32_t *bounds, int nb) {
    attn_desc a = {B, H, d, offsets, num_targets, K1, K2, alpha, inv_n, table, bounds, nb};
    return a;
}

/* Forward for every token.  A is fully overwritten. */
void oracle_attn_fwd(int B, int H, int d, const int32_t *offsets, const int32_t *num_targets, int K1, int K2,
                     double alpha, double inv_n, const double *table, const int32_t *bounds, int nb,
                     const double *Q, const double *K, const double *V, double *A) {
    const attn_desc a = make_desc(B, H, d, offsets, num_targets, K1, K2, alpha, inv_n, table, bounds, nb);
    for (int b = 0; b < B; ++b) {
        const int L = offsets[b + 1] - offsets[b];
#pragma omp parallel for schedule(dynamic, 4)
        for (int i = 0; i < L; ++i)
            fwd_row(&a, Q, K, V, b, i, A + ((int64_t)offsets[b] + i) * H * d);
    }
}

/* Forward for a list of global token rows only: out is [nrows, H, d]. */
void oracle_attn_fwd_rows(int B, int H, int d, const int32_t *offsets, const int32_t *num_targets, int K1, int K2,
                          double alpha, double inv_n, const double *table, const int32_t *bounds, int nb,
                          const double *Q, const double *K, const double *V,
                          int nrows, const int64_t *rows, double *out) {
    const attn_desc a = make_desc(B, H, d, offsets, num_targets, K1, K2, alpha, inv_n, table, bounds, nb);
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < nrows; ++r) {
        const int b = seq_of(&a, rows[r]);
        fwd_row(&a, Q, K, V, b, (int)(rows[r] - offsets[b]), out + (int64_t)r * H * d);
    }
}

/*
 * Backward, per visible pair (i, j), with s the recomputed score and sg = sigmoid(s):
 *   w  = s sg / N                      dV_j += w dA_i
 *   dw = dA_i . V_j                    ds = dw (sg (1 + s (1 - sg))) / N
 *   dQ_i += alpha ds K_j               dK_j += alpha ds Q_i
 */
static void bwd_q_row(const attn_desc *a, const double *Q, const double *K, const double *V, const double *dA,
                      int b, int i, double *dq /* [H,d] */) {
    const int H = a->H, d = a->d;
    const int64_t base = a->offsets[b];
    const int L = a->offsets[b + 1] - a->offsets[b];
    const int M = a->num_targets ? a->num_targets[b] : 0;
    for (int h = 0; h < H; ++h) {
        double *g = dq + (int64_t)h * d;
        for (int c = 0; c < d; ++c) g[c] = 0.0;
        const double *da = dA + ((base + i) * H + h) * d;
        for (int j = 0; j < L; ++j) {
            int delta;
            if (!visible(i, j, L, M, a->K1, a->K2, &delta)) continue;
            const double s = score(a, Q, K, base + i, base + j, h, delta);
            const double sg = sigmoid(s);
            const double *v = V + ((base + j) * H + h) * d, *k = K + ((base + j) * H + h) * d;
            double dw = 0.0;
            for (int c = 0; c < d; ++c) dw += da[c] * v[c];
            const double ds = dw * sg * (1.0 + s * (1.0 - sg)) * a->inv_n;
            for (int c = 0; c < d; ++c) g[c] += a->alpha * ds * k[c];
        }
    }
}

static void bwd_kv_row(const attn_desc *a, const double *Q, const double *K, const double *V, const double *dA,
                       int b, int j, double *dk, double *dv /* [H,d] each */) {
    const int H = a->H, d = a->d;
    const int64_t base = a->offsets[b];
    const int L = a->offsets[b + 1] - a->offsets[b];
    const int M = a->num_targets ? a->num_targets[b] : 0;
    for (int h = 0; h < H; ++h) {
        double *gk = dk + (int64_t)h * d, *gv = dv + (int64_t)h * d;
        for (int c = 0; c < d; ++c) { gk[c] = 0.0; gv[c] = 0.0; }
        const double *v = V + ((base + j) * H + h) * d;
        for (int i = 0; i < L; ++i) {
            int delta;
            if (!visible(i, j, L, M, a->K1, a->K2, &delta)) continue;
            const double s = score(a, Q, K, base + i, base + j, h, delta);
            const double sg = sigmoid(s);
            const double w = s * sg * a->inv_n;
            const double *da = dA + ((base + i) * H + h) * d, *q = Q + ((base + i) * H + h) * d;
            double dw = 0.0;
            for (int c = 0; c < d; ++c) dw += da[c] * v[c];
            const double ds = dw * sg * (1.0 + s * (1.0 - sg)) * a->inv_n;
            for (int c = 0; c < d; ++c) { gv[c] += w * da[c]; gk[c] += a->alpha * ds * q[c]; }
        }
    }
}

/* Backward for every token.  dQ, dK, dV are fully overwritten. */
void oracle_attn_bwd(int B, int H, int d, const int32_t *offsets, const int32_t *num_targets, int K1, int K2,
                     double alpha, double inv_n, const double *table, const int32_t *bounds, int nb,
                     const double *Q, const double *K, const double *V, const double *dA,
                     double *dQ, double *dK, double *dV) {
    const attn_desc a = make_desc(B, H, d, offsets, num_targets, K1, K2, alpha, inv_n, table, bounds, nb);
    for (int b = 0; b < B; ++b) {
        const int L = offsets[b + 1] - offsets[b];
#pragma omp parallel for schedule(dynamic, 4)
        for (int i = 0; i < L; ++i) {
            const int64_t t = (int64_t)offsets[b] + i;
            bwd_q_row(&a, Q, K, V, dA, b, i, dQ + t * H * d);
            bwd_kv_row(&a, Q, K, V, dA, b, i, dK + t * H * d, dV + t * H * d);
        }
    }
}

/* Backward for a list of global token rows only: dq, dk, dv are [nrows, H, d]. */
void oracle_attn_bwd_rows(int B, int H, int d, const int32_t *offsets, const int32_t *num_targets, int K1, int K2,
                          double alpha, double inv_n, const double *table, const int32_t *bounds, int nb,
                          const double *Q, const double *K, const double *V, const double *dA,
                          int nrows, const int64_t *rows, double *dq, double *dk, double *dv) {
    const attn_desc a = make_desc(B, H, d, offsets, num_targets, K1, K2, alpha, inv_n, table, bounds, nb);
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < 2 * nrows; ++r) {
        const int rr = r >> 1;
        const int b = seq_of(&a, rows[rr]);
        const int i = (int)(rows[rr] - offsets[b]);
        if (r & 1) bwd_kv_row(&a, Q, K, V, dA, b, i, dk + (int64_t)rr * H * d, dv + (int64_t)rr * H * d);
        else       bwd_q_row(&a, Q, K, V, dA, b, i, dq + (int64_t)rr * H * d);
    }
}

/*
 * Gradient of the relative-bias table.  The bias enters the score additively, s = alpha q.k + table[h, bucket(dist)],
 * so dL/dtable[h, c] is the sum of ds (as defined above) over the visible pairs of head h whose distance falls in
 * bucket c.  dtable is [H, nb], fully overwritten.  (The paper has no bias; this follows the benchmark spec of the
 * layer, like score().)
 */
void oracle_attn_bwd_bias(int B, int H, int d, const int32_t *offsets, const int32_t *num_targets, int K1, int K2,
                          double alpha, double inv_n, const double *table, const int32_t *bounds, int nb,
                          const double *Q, const double *K, const double *V, const double *dA, double *dtable) {
    const attn_desc a = make_desc(B, H, d, offsets, num_targets, K1, K2, alpha, inv_n, table, bounds, nb);
    for (int64_t x = 0; x < (int64_t)H * nb; ++x) dtable[x] = 0.0;
    if (!table) return;
    for (int b = 0; b < B; ++b) {
        const int64_t base = offsets[b];
        const int L = offsets[b + 1] - offsets[b];
        const int M = num_targets ? num_targets[b] : 0;
#pragma omp parallel
        {
            double *loc = (double *)calloc((size_t)H * nb, sizeof(double));
#pragma omp for schedule(dynamic, 4)
            for (int i = 0; i < L; ++i)
                for (int h = 0; h < H; ++h) {
                    const double *da = dA + ((base + i) * H + h) * d;
                    for (int j = 0; j < L; ++j) {
                        int delta;
                        if (!visible(i, j, L, M, K1, K2, &delta)) continue;
                        const double s = score(&a, Q, K, base + i, base + j, h, delta);
                        const double sg = sigmoid(s);
                        const double *v = V + ((base + j) * H + h) * d;
                        double dw = 0.0;
                        for (int c = 0; c < d; ++c) dw += da[c] * v[c];
                        loc[(int64_t)h * nb + bucket_of(bounds, nb, delta)] += dw * sg * (1.0 + s * (1.0 - sg)) * inv_n;
                    }
                }
#pragma omp critical
            for (int64_t x = 0; x < (int64_t)H * nb; ++x) dtable[x] += loc[x];
            free(loc);
        }
    }
}

/* visible(i, j) for one sequence as a dense L x L byte matrix, plus the distances (for tests). */
void oracle_mask(int L, int M, int K1, int K2, uint8_t *mask, int32_t *dist) {
    for (int i = 0; i < L; ++i)
        for (int j = 0; j < L; ++j) {
            int delta = -1;
            const int vis = visible(i, j, L, M, K1, K2, &delta);
            mask[(int64_t)i * L + j] = (uint8_t)vis;
            dist[(int64_t)i * L + j] = vis ? delta : -1;
        }
}

/* number of visible (query, key) pairs of one sequence */
int64_t oracle_count_pairs(int L, int M, int K1, int K2) {
    int64_t cnt = 0;
    for (int i = 0; i < L; ++i)
        for (int j = 0; j < L; ++j) {
            int delta;
            cnt += visible(i, j, L, M, K1, K2, &delta);
        }
    return cnt;
}

/*
 * Epilogue forward, per token t with a = A[t, :] of D = H d features:
 *   mu = mean(a); var = mean((a - mu)^2); ahat = (a - mu) / sqrt(var + eps)
 *   Y[t] = (ahat gamma + beta) U[t]
 */
void oracle_gated_norm_fwd(int64_t T, int D, const double *A, const double *U, const double *gamma, const double *beta,
                           double eps, double *Y, double *mean, double *rstd) {
#pragma omp parallel for
    for (int64_t t = 0; t < T; ++t) {
        const double *a = A + t * D, *u = U + t * D;
        double mu = 0.0, var = 0.0;
        for (int c = 0; c < D; ++c) mu += a[c];
        mu /= D;
        for (int c = 0; c < D; ++c) var += (a[c] - mu) * (a[c] - mu);
        var /= D;
        const double rs = 1.0 / sqrt(var + eps);
        for (int c = 0; c < D; ++c)
            Y[t * D + c] = ((a[c] - mu) * rs * gamma[c] + (beta ? beta[c] : 0.0)) * u[c];
        if (mean) mean[t] = mu;
        if (rstd) rstd[t] = rs;
    }
}

/*
 * Epilogue backward:
 *   dn = dY U;  dU = dY (ahat gamma + beta);  dgamma = sum_t dn ahat;  dbeta = sum_t dn
 *   dahat = dn gamma;  dA = rstd (dahat - mean(dahat) - ahat mean(dahat ahat))
 */
void oracle_gated_norm_bwd(int64_t T, int D, const double *dY, const double *A, const double *U, const double *gamma,
                           const double *beta, double eps, double *dA, double *dU, double *dgamma, double *dbeta) {
    for (int c = 0; c < D; ++c) { dgamma[c] = 0.0; if (dbeta) dbeta[c] = 0.0; }
    double *ahat = (double *)malloc(sizeof(double) * D), *dahat = (double *)malloc(sizeof(double) * D);
    for (int64_t t = 0; t < T; ++t) {
        const double *a = A + t * D, *u = U + t * D, *dy = dY + t * D;
        double mu = 0.0, var = 0.0;
        for (int c = 0; c < D; ++c) mu += a[c];
        mu /= D;
        for (int c = 0; c < D; ++c) var += (a[c] - mu) * (a[c] - mu);
        var /= D;
        const double rs = 1.0 / sqrt(var + eps);
        double m1 = 0.0, m2 = 0.0;
        for (int c = 0; c < D; ++c) {
            ahat[c] = (a[c] - mu) * rs;
            const double dn = dy[c] * u[c];
            dU[t * D + c] = dy[c] * (ahat[c] * gamma[c] + (beta ? beta[c] : 0.0));
            dgamma[c] += dn * ahat[c];
            if (dbeta) dbeta[c] += dn;
            dahat[c] = dn * gamma[c];
            m1 += dahat[c];
            m2 += dahat[c] * ahat[c];
        }
        m1 /= D; m2 /= D;
        for (int c = 0; c < D; ++c) dA[t * D + c] = rs * (dahat[c] - m1 - ahat[c] * m2);
    }
    free(ahat); free(dahat);
}
