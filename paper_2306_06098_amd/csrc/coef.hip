// coef.hip -- the m x m part of the step: coefficients of eq. (2),
//   coef = (1/lambda) (m*lambda*I + S)^-1 q,
// which is what the WSM recursion of Section "Efficient Full-Matrix
// Preconditioners" produces (Woodbury identity applied to
// F = lambda*I + (1/m) sum_r c_r c_r^T).
//
// One workgroup of 1024 threads, fp64 throughout, O(m^2) work per step:
// thread p owns window slot p.  The Cholesky factor L of A = m*lambda*I + S
// is kept in age order (oldest row first) and stored by slot, so sliding the
// window never moves data:
//   * evicting the oldest row deletes the first row/column of A; the factor
//     of what remains is the rank-one *update* chol(L22 L22^T + l l^T) with
//     l the deleted column (an update, never a downdate: unconditionally
//     stable);
//   * appending the newest row is one forward substitution L z = s with the
//     new Gram column s, and a new diagonal sqrt(A_nn - z^T z);
//   * coef needs L w = q (forward, done in the same sweep) and L^T c = w
//     (backward).
// The update rotations and both forward substitutions share one sweep over
// the columns in age order (one barrier per column); the backward sweep
// walks each thread's own column downwards in 64-byte pieces.
#include "efcp_internal.h"

namespace efcp {

struct ColMsg {      // published by the thread that owns the diagonal of a column
    double ic, s, c;     // rotation: inverse cosine-like factor, sine-like factor, c
    double z, w;         // forward-substitution results for the two right-hand sides
};

__device__ __forceinline__ double block_sum_fixed(double v, double *buf /*1024*/)
{
    // Fixed-shape tree over 1024 slots: same order every run.
    buf[threadIdx.x] = v;
    __syncthreads();
    for (int o = 512; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) buf[threadIdx.x] += buf[threadIdx.x + o];
        __syncthreads();
    }
    const double r = buf[0];
    __syncthreads();
    return r;
}

__global__ __launch_bounds__(1024) void k_coef(int32_t m, int32_t ldm, int32_t n, int32_t slot,
                                               int32_t evict, double lambda,
                                               const double2 *__restrict__ partial2, int32_t n_groups,
                                               double *__restrict__ S, double *__restrict__ L,
                                               double *__restrict__ q_out, double *__restrict__ coef_out,
                                               const uint32_t *__restrict__ rowmax,
                                               LcgParams *__restrict__ lcg, uint32_t *__restrict__ status)
{
    __shared__ ColMsg msg[2];
    __shared__ double red[1024];
    __shared__ double bc[2];

    const int p = threadIdx.x;
    // Rows present besides the new one: every other slot when the window was
    // already full (evict), else slots 0..slot-1.
    const bool is_new = (p == slot);
    const bool is_old = (p < m) && !is_new && (evict ? true : (p < slot));
    // Age among the old rows after the eviction: 0 = oldest.
    const int age = evict ? ((p - slot - 1 + m) % m) : p;

    // ---- finish the fixed-order reduction over slice groups ----
    double qv = 0.0, sv = 0.0;
    if (p < m && (is_old || is_new)) {
        for (int g = 0; g < n_groups; g++) {
            const double2 t = partial2[(int64_t)g * m + p];
            qv += t.x;
            sv += t.y;
        }
    }
    if (p < m) {
        q_out[p] = qv;
        if (is_old || is_new) {
            S[(int64_t)slot * m + p] = sv;
            S[(int64_t)p * m + slot] = sv;
        }
    }
    const double mlam = (double)m * lambda;
    const double a_nn = sv + mlam;       // meaningful on the thread that owns the new row
    const double q_nn = qv;

    // ---- sweep over the old columns in age order ----
    // w_upd: the deleted column l (only when evicting); rhs_s / rhs_q: right-hand sides.
    double w_upd = (evict && is_old) ? L[(int64_t)slot * ldm + p] : 0.0;
    double rhs_s = sv, rhs_q = qv;
    double z_own = 0.0, w_own = 0.0, diag = 1.0;

    int step = 0;
    // two physical segments in ascending age: [slot+1, m-1] (only when evicting), then [0, slot-1]
    for (int seg = evict ? 0 : 1; seg < 2; seg++) {
        const int lo = seg == 0 ? slot + 1 : 0;
        const int hi = seg == 0 ? m - 1 : slot - 1;
        for (int kb = lo & ~7; kb <= hi; kb += 8) {
            double v[8];
#pragma unroll
            for (int r = 0; r < 8; r++) {
                const int kp = kb + r;
                const int ak = evict ? ((kp - slot - 1 + m) % m) : kp;
                v[r] = (kp >= lo && kp <= hi && is_old && age >= ak) ? L[(int64_t)kp * ldm + p] : 0.0;
            }
#pragma unroll
            for (int r = 0; r < 8; r++) {
                const int kp = kb + r;
                if (kp < lo || kp > hi) continue;          // uniform
                const int ak = evict ? ((kp - slot - 1 + m) % m) : kp;
                ColMsg *mm = &msg[step & 1];
                if (p == kp) {
                    double lkk = v[r];
                    double ic = 1.0, sn = 0.0, cs = 1.0;
                    if (evict) {
                        const double rr = sqrt(lkk * lkk + w_upd * w_upd);
                        cs = rr / lkk;
                        sn = w_upd / lkk;
                        ic = lkk / rr;
                        lkk = rr;
                        L[(int64_t)kp * ldm + p] = lkk;
                    }
                    diag = lkk;
                    z_own = rhs_s / lkk;
                    w_own = rhs_q / lkk;
                    mm->ic = ic; mm->s = sn; mm->c = cs; mm->z = z_own; mm->w = w_own;
                    L[(int64_t)kp * ldm + slot] = z_own;       // new row of the factor
                }
                __syncthreads();
                if (is_old && age > ak) {
                    double lv = v[r];
                    if (evict) {
                        lv = (lv + mm->s * w_upd) * mm->ic;
                        w_upd = mm->c * w_upd - mm->s * lv;
                        L[(int64_t)kp * ldm + p] = lv;
                    }
                    rhs_s -= lv * mm->z;
                    rhs_q -= lv * mm->w;
                }
                step++;
            }
        }
    }
    __syncthreads();

    // ---- diagonal of the new row and its forward-substitution entry ----
    const double zz = block_sum_fixed(is_old ? z_own * z_own : 0.0, red);
    const double zw = block_sum_fixed(is_old ? z_own * w_own : 0.0, red);
    if (is_new) {
        double piv = a_nn - zz;
        if (!(piv >= mlam)) {        // the exact Schur complement is >= m*lambda
            piv = mlam;
            atomicOr(status, kStatusPivot);
        }
        diag = sqrt(piv);
        w_own = (q_nn - zw) / diag;
        L[(int64_t)slot * ldm + slot] = diag;
    }

    // ---- backward substitution L^T c = w, newest row first ----
    double csol = 0.0;       // this thread's solution entry once its turn has come
    if (is_new) { csol = w_own / diag; bc[0] = csol; }
    __syncthreads();
    if (is_old) w_own -= z_own * bc[0];      // row `slot` of L is z
    step = 1;
    // descending age: [slot-1 .. 0], then [m-1 .. slot+1] (only when evicting)
    for (int seg = 0; seg < (evict ? 2 : 1); seg++) {
        const int lo = seg == 0 ? 0 : slot + 1;
        const int hi = seg == 0 ? slot - 1 : m - 1;
        if (hi < lo) continue;
        for (int kb = hi & ~7; kb >= (lo & ~7); kb -= 8) {
            double v[8];
            // rows kb..kb+7 of this thread's own column: one 64-byte piece
            const bool any = is_old;
#pragma unroll
            for (int r = 0; r < 8; r++) {
                const int kp = kb + r;
                const int ak = evict ? ((kp - slot - 1 + m) % m) : kp;
                v[r] = (any && kp >= lo && kp <= hi && ak > age) ? L[(int64_t)p * ldm + kp] : 0.0;
            }
#pragma unroll
            for (int r = 7; r >= 0; r--) {
                const int kp = kb + r;
                if (kp < lo || kp > hi) continue;          // uniform
                const int ak = evict ? ((kp - slot - 1 + m) % m) : kp;
                if (p == kp) { csol = w_own / diag; bc[step & 1] = csol; }
                __syncthreads();
                if (is_old && age < ak) w_own -= v[r] * bc[step & 1];
                step++;
            }
        }
    }
    __syncthreads();

    const double coef = (is_old || is_new) ? csol / lambda : 0.0;
    if (p < m) coef_out[p] = coef;

    // ---- fixed-point scale for the LCG accumulator ----
    const double vmax = (p < m && (is_old || is_new)) ? (double)__uint_as_float(rowmax[p]) : 0.0;
    const double bound = block_sum_fixed(fabs(coef) * vmax, red);
    if (p == 0) {
        int ex = 0;
        if (bound > 0.0 && bound < 1.0e300) {
            ex = ilogb(bound) + 1;
            ex = ex < -900 ? -900 : (ex > 900 ? 900 : ex);
        } else if (bound != 0.0) {
            atomicOr(status, kStatusRange);
        }
        lcg->unit = ldexp(1.0, ex - 50);
        lcg->magic = ldexp(1.5, ex + 2);      // 1.5 * 2^52 * unit
    }
}

hipError_t launch_coef(const Geometry &g, const DevicePtrs &p, int32_t n_filled, int32_t slot,
                       int32_t evict, double lambda, hipStream_t stream)
{
    hipLaunchKernelGGL(k_coef, dim3(1), dim3(1024), 0, stream, g.m, g.ldm, n_filled, slot, evict, lambda,
                       p.partial2, g.n_groups, p.S, p.L, p.q, p.coef, p.rowmax, p.lcg, p.status);
    return hipGetLastError();
}

}  // namespace efcp
