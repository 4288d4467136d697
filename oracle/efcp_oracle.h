/*
 * efcp_oracle.h -- CPU oracle for one EFCP / Sparse M-FAC step.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the plain, slow, single-threaded
 * reference that the GPU library is checked against.  It shares no code,
 * header, table or helper with the HIP path and must never be called from
 * the product path; only tests, the smoke check and the benchmark's
 * cpu_baseline leg load it.
 *
 * What it computes, per step t = 1, 2, ... (paper: Algorithm 1, lines 5-8;
 * Section "Efficient Full-Matrix Preconditioners", the WSM recursion and
 * eq. (2); Section "Compressing Preconditioners via Sparsity"):
 *
 *   a   = e + g                          fp32, one rounding per element
 *   c   = TopK(a)                        k largest |a_j|, ties -> lower index
 *   e   = a - c                          +0 on selected entries, a_j elsewhere
 *   slot (t-1) mod m of the window G=(I,V) <- c    (oldest row overwritten)
 *   S[slot][r] = S[r][slot] = <c_r, c>   for every filled row r, fp64
 *   q[r]   = <c_r, x>                    fp64
 *   coef   = coefficients of eq. (2) obtained from the WSM recursion, fp64
 *   y      = x/lambda - sum_r coef[r] * c_r                        fp64
 *
 * so that y = F^{-1} x with F = lambda*I + (1/m) * sum_r c_r c_r^T over the
 * filled rows (unfilled slots count as zero rows; the divisor stays m).
 *
 * Parity pins live in tests/test_oracle_*.py (dense inversion, brute-force
 * Top-k, EF telescoping, closed forms).  No worked numerical example is
 * printed in the paper, so parity against paper-printed values is unpinned;
 * every function below is pinned by mathematics instead.
 */
#ifndef EFCP_ORACLE_H
#define EFCP_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct eo_state eo_state;

/* Returns NULL on invalid arguments or allocation failure.
 * Requires 1 <= k <= d < 2^31, m >= 1, lambda > 0. */
eo_state *eo_create(int64_t d, int32_t m, int64_t k, double lambda);

/* Same with the stored values V kept in bfloat16 (Section "Format for V"):
 * values_bf16 != 0 makes the compressed vector c hold bf16(a_j) (round to
 * nearest even on the upper 16 bits) at the selected positions, and, as
 * xi = a - c says, the error keeps the rounding remainder a_j - bf16(a_j) there
 * instead of 0.  Selection itself is done on the fp32 accumulator. */
eo_state *eo_create_fmt(int64_t d, int32_t m, int64_t k, double lambda, int values_bf16);

/* Top-k applied in blocks of `block` consecutive coordinates (Section "Sparsity Pattern"):
 * every full block keeps exactly kb entries, its kb largest magnitudes (ties -> lower index);
 * a ragged last block of len coordinates keeps ceil(kb*len/block).  The row length k is
 * eo_block_row_length(d, block, kb).  Requires 1 <= kb <= block. */
eo_state *eo_create_block(int64_t d, int32_t m, int64_t block, int64_t kb, double lambda,
                          int values_bf16);
int64_t eo_block_row_length(int64_t d, int64_t block, int64_t kb);

/* Sparse GGT instead of Sparse M-FAC on the same error feedback, Top-k and window (Appendix
 * "Sparse GGT", Algorithm "Detailed Sparse GGT Implementation"): eo_step / eo_step_compressed /
 * eo_apply then return u = ((G G^T)^{1/2} + epsilon I)^-1 x, G = the stored vectors as columns.
 * The paper's algorithm preconditions the compressed accumulator (eo_step_compressed).
 * block = 0: global Top-k of k; block = B: Top-k in blocks of B, k per block. */
eo_state *eo_create_ggt(int64_t d, int32_t m, int64_t k, double epsilon, int values_bf16,
                        int64_t block);

/* Symmetric eigendecomposition by cyclic Jacobi: A (n*n, destroyed) = V diag(lam) V^T,
 * eigenvector i in column i of V (V[r*n+i]). */
int eo_jacobi_eigh(double *A, int32_t n, double *lam, double *V);

/* Round an fp32 value to bfloat16 (nearest, ties to even), returned as fp32. */
float eo_bf16_round(float a);
void eo_destroy(eo_state *st);

/* One full step.  g: d floats (gradient).  x: d floats to precondition, or
 * NULL meaning x = g.  y: d doubles, receives F^{-1} x.  Returns 0, or -1 on
 * allocation failure. */
int eo_step(eo_state *st, const float *g, const float *x, double *y);

/* Lines 5-7 of Algorithm 1 and the window update of line 8 only (a = e + g, c = TopK(a),
 * e = a - c, c into the ring, its row and column of S): exactly what eo_step does before it
 * preconditions, so the state afterwards is the state eo_step leaves, bit for bit; q and coef
 * keep their previous contents.  For filling a window without paying for F^-1 x. */
int eo_step_no_output(eo_state *st, const float *g);

/* Algorithm 1 line 8 as printed: the vector preconditioned is the compressed
 * accumulator itself, u = A(c_t), i.e. x = c_t scattered to dense.  Otherwise
 * identical to eo_step. */
int eo_step_compressed(eo_state *st, const float *g, double *y);

/* y = F^{-1} x for the window as it stands (eq. (2)); the state is not changed
 * except for the q / coef views below. */
int eo_apply(eo_state *st, const float *x, double *y);

/* Algorithm 1 line 9 with decoupled weight decay (the AdamW-style decay the paper's
 * experiments use): theta_j <- fp32( (1 - lr*weight_decay)*theta_j - lr*u_j ), in fp64. */
void eo_param_update(float *theta, const double *u, int64_t d, double lr, double weight_decay);

/* Read-only views of the state after the last step. */
int64_t eo_step_count(const eo_state *st);          /* t */
int32_t eo_filled(const eo_state *st);              /* n_t = min(t, m) */
const float *eo_error(const eo_state *st);          /* e, d floats */
const int32_t *eo_row_idx(const eo_state *st, int32_t slot);   /* k, ascending; NULL if unfilled */
const float *eo_row_val(const eo_state *st, int32_t slot);     /* k */
const double *eo_gram(const eo_state *st);          /* S, m*m row-major, zeros for unfilled */
const double *eo_q(const eo_state *st);             /* q, m (by slot) */
const double *eo_coef(const eo_state *st);          /* coef, m (by slot) */

/* Overwrite one window slot directly (used to preload a window when timing
 * the oracle on a full window).  idx ascending, distinct, in [0,d).  The slot
 * becomes the newest row: step count advances by one and the Gram row/column
 * is recomputed exactly as eo_step does.  Returns 0 or -1. */
int eo_load_row(eo_state *st, const int32_t *idx, const float *val);

/* ---- the individual pieces, exposed so each can be pinned on its own ---- */

/* Top-k by magnitude.  Order: key_j = bits(a_j) & 0x7fffffff descending, then
 * j ascending.  Writes idx (ascending) and val[p] = a[idx[p]].  Returns 0/-1. */
int eo_topk(const float *a, int64_t d, int64_t k, int32_t *idx, float *val);

/* Coefficients of eq. (2) from scalar products only.
 * S: n*n row-major Gram matrix of the rows in processing order, q: n scalar
 * products with x, m: window size in the 1/m factor, lambda: damping.
 * coef: n outputs.  Literal rank-one (WSM) recursion, O(n^3).  Returns 0/-1. */
int eo_coefficients(const double *S, const double *q, int32_t n, int32_t m,
                    double lambda, double *coef);

#ifdef __cplusplus
}
#endif
#endif
