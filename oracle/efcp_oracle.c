/*
 * efcp_oracle.c -- CPU oracle for one EFCP / Sparse M-FAC step.
 *
 * TEST INFRASTRUCTURE ONLY; see efcp_oracle.h.  Plain C, single thread, no
 * blocking, no fusion: every function is the definition (or the paper's
 * recursion) written out so it can be checked against the paper by eye.
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -shared -fPIC
 */
#include "efcp_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

struct eo_state {
    int64_t d, k;
    int32_t m;
    double lambda;
    int values_bf16;    /* stored values are bfloat16 */
    int64_t block;      /* 0: global Top-k; B > 0: Top-k applied in blocks of B coordinates */
    int64_t kb;         /* entries kept per full block (block mode) */
    int ggt;            /* 0: Sparse M-FAC; 1: Sparse GGT (lambda then holds epsilon) */
    int64_t t;          /* steps done */
    float *e;           /* error feedback xi, d */
    int32_t **idx;      /* m row pointers, NULL until the slot is filled */
    float **val;
    double *S;          /* m*m Gram matrix, by slot */
    double *q, *coef;   /* m, by slot */
    float *a;           /* d, accumulator scratch */
    float *dense;       /* d, newest row scattered to dense, scratch */
};

float eo_bf16_round(float a)
{
    uint32_t bits;
    memcpy(&bits, &a, 4);
    bits += 0x7fffu + ((bits >> 16) & 1u);      /* nearest, ties to even */
    bits &= 0xffff0000u;
    float r;
    memcpy(&r, &bits, 4);
    return r;
}

eo_state *eo_create_fmt(int64_t d, int32_t m, int64_t k, double lambda, int values_bf16)
{
    eo_state *st = eo_create(d, m, k, lambda);
    if (st) st->values_bf16 = values_bf16 != 0;
    return st;
}

int64_t eo_block_row_length(int64_t d, int64_t block, int64_t kb)
{
    if (d < 1 || block < 1 || kb < 1 || kb > block) return 0;
    const int64_t full = d / block, tail = d % block;
    /* the ragged last block keeps the same share, rounded up */
    return full * kb + (tail ? (kb * tail + block - 1) / block : 0);
}

eo_state *eo_create_block(int64_t d, int32_t m, int64_t block, int64_t kb, double lambda,
                          int values_bf16)
{
    const int64_t k = eo_block_row_length(d, block, kb);
    if (k < 1) return NULL;
    eo_state *st = eo_create_fmt(d, m, k, lambda, values_bf16);
    if (st) { st->block = block; st->kb = kb; }
    return st;
}

/* Top-k applied in blocks (Section "Sparsity Pattern"): the kb largest magnitudes of every
 * block of B consecutive coordinates, each block on its own; idx ascending overall. */
static int topk_blockwise(const float *a, int64_t d, int64_t block, int64_t kb, int32_t *idx, float *val)
{
    int64_t w = 0;
    for (int64_t lo = 0; lo < d; lo += block) {
        const int64_t len = d - lo < block ? d - lo : block;
        const int64_t keep = len == block ? kb : (kb * len + block - 1) / block;
        if (eo_topk(a + lo, len, keep, idx + w, val + w) != 0) return -1;
        for (int64_t p = 0; p < keep; p++) idx[w + p] += (int32_t)lo;
        w += keep;
    }
    return 0;
}

eo_state *eo_create(int64_t d, int32_t m, int64_t k, double lambda)
{
    if (d < 1 || d >= ((int64_t)1 << 31) || k < 1 || k > d || m < 1 ||
        !(lambda > 0.0) || !isfinite(lambda))
        return NULL;
    eo_state *st = calloc(1, sizeof *st);
    if (!st) return NULL;
    st->d = d; st->k = k; st->m = m; st->lambda = lambda;
    st->e = calloc((size_t)d, sizeof(float));
    st->a = calloc((size_t)d, sizeof(float));
    st->dense = calloc((size_t)d, sizeof(float));
    st->idx = calloc((size_t)m, sizeof(int32_t *));
    st->val = calloc((size_t)m, sizeof(float *));
    st->S = calloc((size_t)m * m, sizeof(double));
    st->q = calloc((size_t)m, sizeof(double));
    st->coef = calloc((size_t)m, sizeof(double));
    if (!st->e || !st->a || !st->dense || !st->idx || !st->val || !st->S ||
        !st->q || !st->coef) {
        eo_destroy(st);
        return NULL;
    }
    return st;
}

void eo_destroy(eo_state *st)
{
    if (!st) return;
    if (st->idx) for (int32_t r = 0; r < st->m; r++) free(st->idx[r]);
    if (st->val) for (int32_t r = 0; r < st->m; r++) free(st->val[r]);
    free(st->idx); free(st->val);
    free(st->e); free(st->a); free(st->dense);
    free(st->S); free(st->q); free(st->coef);
    free(st);
}

int64_t eo_step_count(const eo_state *st) { return st->t; }
int32_t eo_filled(const eo_state *st) { return st->t < st->m ? (int32_t)st->t : st->m; }
const float *eo_error(const eo_state *st) { return st->e; }
const int32_t *eo_row_idx(const eo_state *st, int32_t slot)
{ return (slot >= 0 && slot < st->m) ? st->idx[slot] : NULL; }
const float *eo_row_val(const eo_state *st, int32_t slot)
{ return (slot >= 0 && slot < st->m) ? st->val[slot] : NULL; }
const double *eo_gram(const eo_state *st) { return st->S; }
const double *eo_q(const eo_state *st) { return st->q; }
const double *eo_coef(const eo_state *st) { return st->coef; }

/* ------------------------------------------------------------------ */
/* Top-k (Algorithm 1 line 6 with Compress = Top-k by magnitude).      */
/* Definition: sort all (key_j, j) by key descending, then j ascending; */
/* the first k pairs are the selection.                                */

typedef struct { uint32_t key; int32_t j; } eo_pair;

static int cmp_key_desc_j_asc(const void *pa, const void *pb)
{
    const eo_pair *a = pa, *b = pb;
    if (a->key != b->key) return a->key > b->key ? -1 : 1;
    if (a->j != b->j) return a->j < b->j ? -1 : 1;
    return 0;
}

static int cmp_j_asc(const void *pa, const void *pb)
{
    const eo_pair *a = pa, *b = pb;
    return a->j < b->j ? -1 : (a->j > b->j ? 1 : 0);
}

int eo_topk(const float *a, int64_t d, int64_t k, int32_t *idx, float *val)
{
    eo_pair *p = malloc((size_t)d * sizeof *p);
    if (!p) return -1;
    for (int64_t j = 0; j < d; j++) {
        uint32_t bits;
        memcpy(&bits, &a[j], 4);
        p[j].key = bits & 0x7fffffffu;      /* magnitude as an ordered integer */
        p[j].j = (int32_t)j;
    }
    qsort(p, (size_t)d, sizeof *p, cmp_key_desc_j_asc);
    qsort(p, (size_t)k, sizeof *p, cmp_j_asc);      /* stored rows are index-ascending */
    for (int64_t s = 0; s < k; s++) {
        idx[s] = p[s].j;
        val[s] = a[p[s].j];
    }
    free(p);
    return 0;
}

/* ------------------------------------------------------------------ */
/* Coefficients of eq. (2) by the WSM recursion.                       */
/*                                                                     */
/* Rows c_1..c_n in processing order.  F_0 = lambda*I,                 */
/* F_k = F_{k-1} + (1/m) c_k c_k^T.  With v_k = F_{k-1}^{-1} c_k and   */
/* D_k = m + c_k^T v_k the rank-one inverse update reads               */
/*   F_k^{-1} = F_{k-1}^{-1} - v_k v_k^T / D_k,                        */
/* hence F_n^{-1} x = x/lambda - sum_k v_k (v_k^T x) / D_k.            */
/* Each v_k lies in span(c_1..c_k): v_k = sum_{i<=k} B[k][i] c_i, and  */
/*   v_k = c_k/lambda - sum_{j<k} v_j (v_j^T c_k)/D_j                  */
/* needs only S_ij = c_i^T c_j.  Collecting terms of                   */
/*   sum_k v_k p_k / D_k,  p_k = v_k^T x = sum_i B[k][i] q_i,          */
/* by c_i gives coef_i = sum_{k>=i} B[k][i] p_k / D_k.                 */

int eo_coefficients(const double *S, const double *q, int32_t n, int32_t m,
                    double lambda, double *coef)
{
    if (n == 0) return 0;
    double *B = calloc((size_t)n * n, sizeof(double));
    double *D = calloc((size_t)n, sizeof(double));
    double *p = calloc((size_t)n, sizeof(double));
    if (!B || !D || !p) { free(B); free(D); free(p); return -1; }

    for (int32_t k = 0; k < n; k++) {
        B[(size_t)k * n + k] = 1.0 / lambda;
        for (int32_t j = 0; j < k; j++) {
            double vjck = 0.0;                       /* v_j^T c_k */
            for (int32_t i = 0; i <= j; i++)
                vjck += B[(size_t)j * n + i] * S[(size_t)i * n + k];
            double f = vjck / D[j];
            for (int32_t i = 0; i <= j; i++)
                B[(size_t)k * n + i] -= f * B[(size_t)j * n + i];
        }
        double ckvk = 0.0;                           /* c_k^T v_k */
        for (int32_t i = 0; i <= k; i++)
            ckvk += B[(size_t)k * n + i] * S[(size_t)i * n + k];
        D[k] = (double)m + ckvk;
    }
    for (int32_t k = 0; k < n; k++) {
        double s = 0.0;
        for (int32_t i = 0; i <= k; i++) s += B[(size_t)k * n + i] * q[i];
        p[k] = s;
    }
    for (int32_t i = 0; i < n; i++) {
        double s = 0.0;
        for (int32_t k = i; k < n; k++) s += B[(size_t)k * n + i] * p[k] / D[k];
        coef[i] = s;
    }
    free(B); free(D); free(p);
    return 0;
}

/* ------------------------------------------------------------------ */

/* Place (idx,val) into the slot of step t and refresh row/column of S:
 * S[slot][r] = S[r][slot] = <c_r, c_new> for every filled row r
 * (Section "Scalar Products (SP)": S_{i,:} = S_{:,i} = G g). */
static int insert_row(eo_state *st, const int32_t *idx, const float *val)
{
    const int64_t k = st->k;
    const int32_t m = st->m;
    st->t += 1;
    const int32_t slot = (int32_t)((st->t - 1) % m);
    if (!st->idx[slot]) {
        st->idx[slot] = malloc((size_t)k * sizeof(int32_t));
        st->val[slot] = malloc((size_t)k * sizeof(float));
        if (!st->idx[slot] || !st->val[slot]) return -1;
    }
    memcpy(st->idx[slot], idx, (size_t)k * sizeof(int32_t));
    memcpy(st->val[slot], val, (size_t)k * sizeof(float));

    for (int64_t p = 0; p < k; p++) st->dense[idx[p]] = val[p];
    for (int32_t r = 0; r < m; r++) {
        if (!st->idx[r]) continue;
        double s = 0.0;
        for (int64_t p = 0; p < k; p++)
            s += (double)st->val[r][p] * (double)st->dense[st->idx[r][p]];
        st->S[(size_t)slot * m + r] = s;
        st->S[(size_t)r * m + slot] = s;
    }
    for (int64_t p = 0; p < k; p++) st->dense[idx[p]] = 0.0f;
    return 0;
}

int eo_load_row(eo_state *st, const int32_t *idx, const float *val)
{
    return insert_row(st, idx, val);
}

eo_state *eo_create_ggt(int64_t d, int32_t m, int64_t k, double epsilon, int values_bf16,
                        int64_t block)
{
    eo_state *st = block ? eo_create_block(d, m, block, k, epsilon, values_bf16)
                         : eo_create_fmt(d, m, k, epsilon, values_bf16);
    if (st) st->ggt = 1;
    return st;
}

/* Eigendecomposition of a symmetric n*n matrix by the classical cyclic Jacobi method:
 * sweep over all (p, q), annihilate a_pq with a plane rotation, repeat until a sweep
 * rotates nothing.  On return lam holds the eigenvalues and column i of V (V[r*n+i]) the
 * eigenvector of lam[i]; A is destroyed. */
int eo_jacobi_eigh(double *A, int32_t n, double *lam, double *V)
{
    for (int32_t i = 0; i < n; i++)
        for (int32_t j = 0; j < n; j++) V[(size_t)i * n + j] = i == j ? 1.0 : 0.0;
    for (int sweep = 0; sweep < 100; sweep++) {
        int rotated = 0;
        for (int32_t p = 0; p < n - 1; p++) {
            for (int32_t q = p + 1; q < n; q++) {
                const double apq = A[(size_t)p * n + q];
                const double app = A[(size_t)p * n + p], aqq = A[(size_t)q * n + q];
                if (apq == 0.0 || fabs(apq) <= 0x1p-54 * sqrt(fabs(app) * fabs(aqq))) continue;
                rotated = 1;
                const double tau = (aqq - app) / (2.0 * apq);
                const double t = (tau >= 0.0 ? 1.0 : -1.0) / (fabs(tau) + sqrt(1.0 + tau * tau));
                const double c = 1.0 / sqrt(1.0 + t * t), sn = t * c;
                for (int32_t i = 0; i < n; i++) {            /* A <- A J */
                    const double aip = A[(size_t)i * n + p], aiq = A[(size_t)i * n + q];
                    A[(size_t)i * n + p] = c * aip - sn * aiq;
                    A[(size_t)i * n + q] = sn * aip + c * aiq;
                }
                for (int32_t j = 0; j < n; j++) {            /* A <- J^T A */
                    const double apj = A[(size_t)p * n + j], aqj = A[(size_t)q * n + j];
                    A[(size_t)p * n + j] = c * apj - sn * aqj;
                    A[(size_t)q * n + j] = sn * apj + c * aqj;
                }
                A[(size_t)p * n + q] = A[(size_t)q * n + p] = 0.0;
                for (int32_t i = 0; i < n; i++) {            /* V <- V J */
                    const double vip = V[(size_t)i * n + p], viq = V[(size_t)i * n + q];
                    V[(size_t)i * n + p] = c * vip - sn * viq;
                    V[(size_t)i * n + q] = sn * vip + c * viq;
                }
            }
        }
        if (!rotated) break;
    }
    for (int32_t i = 0; i < n; i++) lam[i] = A[(size_t)i * n + i];
    return 0;
}

/* Sparse GGT direction (Algorithm "Detailed Sparse GGT Implementation"), for the window as it
 * stands: with G (d x n) holding the stored vectors as columns and G^T G = V Sigma^2 V^T,
 *   U = G V Sigma^+,   u = x/eps + U [ (Sigma + eps I)^-1 - I/eps ] U^T x,
 * i.e. u = ((G G^T)^{1/2} + eps I)^-1 x.  Directions with Sigma_i = 0 (up to rounding: Sigma_i^2
 * <= n * 2^-52 * max Sigma^2) are left out by the pseudo-inverse.  q = G^T x is kept for
 * inspection; coef is set to the multiples of the stored vectors that u - x/eps consists of,
 * negated (u = x/eps - sum_r coef_r c_r), so that it reads like eq. (2). */
static int precondition_ggt(eo_state *st, const float *x, double *y)
{
    const int64_t d = st->d, k = st->k;
    const int32_t m = st->m;
    const double eps = st->lambda;
    const int32_t n = eo_filled(st);
    for (int32_t r = 0; r < m; r++) { st->q[r] = 0.0; st->coef[r] = 0.0; }
    for (int64_t j = 0; j < d; j++) y[j] = (double)x[j] / eps;
    if (n == 0) return 0;
    /* filled slots are 0..n-1 (slot order; the result does not depend on the order) */
    double *A = malloc((size_t)n * n * sizeof(double));
    double *V = malloc((size_t)n * n * sizeof(double));
    double *lam = malloc((size_t)n * sizeof(double));
    double *U = calloc((size_t)d * n, sizeof(double));
    double *w = malloc((size_t)n * sizeof(double));
    if (!A || !V || !lam || !U || !w) { free(A); free(V); free(lam); free(U); free(w); return -1; }
    for (int32_t a = 0; a < n; a++)
        for (int32_t b = 0; b < n; b++) A[(size_t)a * n + b] = st->S[(size_t)a * m + b];
    eo_jacobi_eigh(A, n, lam, V);
    double lmax = 0.0;
    for (int32_t i = 0; i < n; i++) if (lam[i] > lmax) lmax = lam[i];
    /* U = G V Sigma^+ : column i = sum_r c_r V[r][i] / sigma_i */
    for (int32_t i = 0; i < n; i++) {
        if (!(lam[i] > (double)n * 0x1p-52 * lmax)) { lam[i] = 0.0; continue; }
        const double sigma = sqrt(lam[i]);
        for (int32_t r = 0; r < n; r++) {
            const double f = V[(size_t)r * n + i] / sigma;
            for (int64_t p = 0; p < k; p++)
                U[(size_t)st->idx[r][p] * n + i] += f * (double)st->val[r][p];
        }
    }
    /* w = [ (Sigma + eps)^-1 - 1/eps ] U^T x ;  u = x/eps + U w */
    for (int32_t i = 0; i < n; i++) {
        double s = 0.0;
        for (int64_t j = 0; j < d; j++) s += U[(size_t)j * n + i] * (double)x[j];
        const double sigma = sqrt(lam[i]);
        w[i] = lam[i] > 0.0 ? (1.0 / (sigma + eps) - 1.0 / eps) * s : 0.0;
    }
    for (int64_t j = 0; j < d; j++) {
        double s = 0.0;
        for (int32_t i = 0; i < n; i++) s += U[(size_t)j * n + i] * w[i];
        y[j] += s;
    }
    /* for inspection only: q = G^T x and the equivalent multiples of the stored vectors */
    for (int32_t r = 0; r < n; r++) {
        double s = 0.0;
        for (int64_t p = 0; p < k; p++) s += (double)st->val[r][p] * (double)x[st->idx[r][p]];
        st->q[r] = s;
        double c = 0.0;
        for (int32_t i = 0; i < n; i++)
            if (lam[i] > 0.0) c += V[(size_t)r * n + i] * w[i] / sqrt(lam[i]);
        st->coef[r] = -c;
    }
    free(A); free(V); free(lam); free(U); free(w);
    return 0;
}

/* q_r = <c_r, x>, coefficients in age order, y = x/lambda - sum_r coef_r c_r
 * for the window as it stands. */
static int precondition(eo_state *st, const float *x, double *y)
{
    if (st->ggt) return precondition_ggt(st, x, y);
    const int64_t d = st->d, k = st->k;
    const int32_t m = st->m;
    for (int32_t r = 0; r < m; r++) {
        st->q[r] = 0.0;
        st->coef[r] = 0.0;
        if (!st->idx[r]) continue;
        double s = 0.0;
        for (int64_t p = 0; p < k; p++)
            s += (double)st->val[r][p] * (double)x[st->idx[r][p]];
        st->q[r] = s;
    }
    const int32_t n = eo_filled(st);
    if (n > 0) {
        const int32_t newest = (int32_t)((st->t - 1) % m);
        int32_t *order = malloc((size_t)n * sizeof(int32_t));
        double *Sn = malloc((size_t)n * n * sizeof(double));
        double *qn = malloc((size_t)n * sizeof(double));
        double *cn = malloc((size_t)n * sizeof(double));
        if (!order || !Sn || !qn || !cn) { free(order); free(Sn); free(qn); free(cn); return -1; }
        for (int32_t a = 0; a < n; a++)          /* age a: 0 = oldest, n-1 = newest */
            order[a] = (int32_t)(((int64_t)newest - (n - 1) + a + (int64_t)m * 2) % m);
        for (int32_t a = 0; a < n; a++) {
            qn[a] = st->q[order[a]];
            for (int32_t b = 0; b < n; b++)
                Sn[(size_t)a * n + b] = st->S[(size_t)order[a] * m + order[b]];
        }
        const int rc = eo_coefficients(Sn, qn, n, m, st->lambda, cn);
        for (int32_t a = 0; a < n; a++) st->coef[order[a]] = cn[a];
        free(order); free(Sn); free(qn); free(cn);
        if (rc != 0) return -1;
    }
    /* eq. (2): y = x/lambda - sum_r coef_r c_r. */
    for (int64_t j = 0; j < d; j++) y[j] = (double)x[j] / st->lambda;
    for (int32_t r = 0; r < m; r++) {
        if (!st->idx[r]) continue;
        const double c = st->coef[r];
        for (int64_t p = 0; p < k; p++)
            y[st->idx[r][p]] -= c * (double)st->val[r][p];
    }
    return 0;
}

int eo_apply(eo_state *st, const float *x, double *y) { return precondition(st, x, y); }

/* Lines 5-7 of Algorithm 1 and the window update; on return idx/val of the
 * newest slot hold c_t. */
static int compress_and_insert(eo_state *st, const float *g)
{
    const int64_t d = st->d, k = st->k;

    /* Algorithm 1 line 5: a = xi + g (fp32). */
    for (int64_t j = 0; j < d; j++) st->a[j] = st->e[j] + g[j];

    /* line 6: c = TopK(a). */
    int32_t *idx = malloc((size_t)k * sizeof(int32_t));
    float *val = malloc((size_t)k * sizeof(float));
    if (!idx || !val) { free(idx); free(val); return -1; }
    const int rc_sel = st->block ? topk_blockwise(st->a, d, st->block, st->kb, idx, val)
                                 : eo_topk(st->a, d, k, idx, val);
    if (rc_sel != 0) { free(idx); free(val); return -1; }

    /* bfloat16 window: c holds the rounded values. */
    if (st->values_bf16)
        for (int64_t p = 0; p < k; p++) val[p] = eo_bf16_round(val[p]);

    /* line 7: xi = a - c. */
    memcpy(st->e, st->a, (size_t)d * sizeof(float));
    for (int64_t p = 0; p < k; p++) st->e[idx[p]] = st->a[idx[p]] - val[p];

    /* line 8, first half: update G (ring buffer) and S. */
    const int rc = insert_row(st, idx, val);
    free(idx); free(val);
    return rc;
}

int eo_step_no_output(eo_state *st, const float *g)
{
    return compress_and_insert(st, g);
}

int eo_step(eo_state *st, const float *g, const float *x, double *y)
{
    if (compress_and_insert(st, g) != 0) return -1;
    return precondition(st, x ? x : g, y);
}

int eo_step_compressed(eo_state *st, const float *g, double *y)
{
    if (compress_and_insert(st, g) != 0) return -1;
    const int32_t slot = (int32_t)((st->t - 1) % st->m);
    float *x = calloc((size_t)st->d, sizeof(float));            /* c_t scattered to dense */
    if (!x) return -1;
    for (int64_t p = 0; p < st->k; p++) x[st->idx[slot][p]] = st->val[slot][p];
    const int rc = precondition(st, x, y);
    free(x);
    return rc;
}

void eo_param_update(float *theta, const double *u, int64_t d, double lr, double weight_decay)
{
    const double decay = 1.0 - lr * weight_decay;
    for (int64_t j = 0; j < d; j++)
        theta[j] = (float)(decay * (double)theta[j] - lr * u[j]);
}
