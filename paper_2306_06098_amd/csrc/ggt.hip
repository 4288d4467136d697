// ggt.hip -- the m x m part of Sparse GGT (Appendix "Sparse GGT", Algorithm "Detailed Sparse GGT
// Implementation"): with G the stored vectors as columns and G^T G = V Sigma^2 V^T,
//   u = x/eps + U [ (Sigma + eps I)^-1 - I/eps ] U^T x,   U = G V Sigma^+,
// which in terms of q = G^T x (the SP pass) is  u = x/eps - sum_r coef_r c_r  with
//   coef = V diag( 1 / (eps sigma_i (sigma_i + eps)) ) V^T q      (sigma_i = 0 left out),
// so the SP and LCG passes of Sparse M-FAC serve unchanged and only the coefficients differ.
//
// The eigendecomposition is a parallel two-sided Jacobi method in one workgroup: the matrix lives
// in LDS, every stage applies n/2 disjoint plane rotations chosen by a round-robin schedule, and
// a sweep is n-1 stages.  V is never formed: the rotations are logged, V^T q is the log applied
// forwards to q and V z the log applied backwards, each rotation touching two numbers.  A later
// efcp_apply on the same window replays the log with its own q.
#include "efcp_internal.h"

namespace efcp {

namespace {

constexpr int kGgtLd = kGgtMaxM + 1;          // padded row length of the matrix in LDS

// Pair j of stage r in a round-robin over N (even) players: everybody meets everybody once in
// N-1 stages.  Returns p < q.
__device__ __forceinline__ void rr_pair(int32_t N, int32_t r, int32_t j, int32_t &p, int32_t &q)
{
    int32_t a, b;
    if (j == 0) {
        a = N - 1;
        b = r;
    } else {
        // r < N-1 and j < N/2: one conditional step replaces the division of a modulo
        a = r + j;
        if (a >= N - 1) a -= N - 1;
        b = r - j;
        if (b < 0) b += N - 1;
    }
    p = a < b ? a : b;
    q = a < b ? b : a;
}

}  // namespace

// One workgroup of 1024 threads.  update != 0: first write the new Gram row and column (sq[].y)
// into S and q (sq[].x) into q_out.  Then diagonalise S[0..n)[0..n).  Outputs: lam[m]
// (eigenvalues, 0 beyond n), the rotation log rot[stage][64] = (c, s) and *n_stages.
// The slot written last and the number of filled rows n come from the step state ("after").
__global__ __launch_bounds__(1024) void k_ggt_eig(int32_t m, const StepState *__restrict__ step, int32_t update,
                                                  double *__restrict__ S, const double2 *__restrict__ sq,
                                                  double *__restrict__ q_out, double *__restrict__ lam,
                                                  double2 *__restrict__ rot, int32_t *__restrict__ n_stages,
                                                  int32_t max_sweeps, double *__restrict__ vtq)
{
    extern __shared__ __align__(16) unsigned char smem[];
    double *A = reinterpret_cast<double *>(smem);                          // [kGgtMaxM][kGgtLd]
    double2 *cs = reinterpret_cast<double2 *>(A + kGgtMaxM * kGgtLd);      // [64]
    int32_t *n_rot = reinterpret_cast<int32_t *>(cs + 64);                 // [1] rotations of this sweep
    double *yv = reinterpret_cast<double *>(n_rot + 4);                    // [kGgtMaxM + 2] V^T q as it forms (update)

    const StepView sv = step_view(step, m, kAfter);
    const int32_t n = sv.n_filled, slot = sv.slot;
    const int tid = threadIdx.x;
    if (update) {
        if (tid < m) {
            const double2 t = sq[tid];
            S[(int64_t)slot * m + tid] = t.y;
            S[(int64_t)tid * m + slot] = t.y;
            q_out[tid] = t.x;
        }
        __syncthreads();                      // the row and column are read back below
    }
    const int32_t N = (n + 1) & ~1;           // even; index n is a dummy player when n is odd
    const int32_t half = N >> 1;
    for (int32_t e = tid; e < kGgtMaxM * kGgtLd; e += 1024) {
        const int32_t i = e / kGgtLd, j = e - i * kGgtLd;
        A[e] = (i < n && j < n) ? S[(int64_t)i * m + j] : 0.0;
    }
    if (tid == 0) *n_rot = 0;
    // With update, q is known: every rotation is applied to it as it is found (by the thread that
    // found it: the pairs of a stage are disjoint), which is V^T q for the coefficients at no cost;
    // the replay kernel then only goes backwards through the log.
    if (tid < kGgtMaxM + 2) yv[tid] = (update && tid < n) ? sq[tid].x : 0.0;
    __syncthreads();

    // The 2x2 blocks a thread updates are the same pairs of pairs (k1 <= k2) in every stage; found
    // once, which keeps integer divisions out of the stages.  Only the blocks on and above the
    // diagonal of the pair grid are computed: A stays symmetric, the block (k2, k1) is the
    // transpose of (k1, k2) and is written along with it.  What limits a stage is LDS traffic,
    // and this way a pair of blocks costs 4 reads and 8 writes instead of 8 and 8, with one
    // fetch of the two rotations instead of two.
    constexpr int kPairsMax = kGgtMaxM / 2;
    constexpr int kBlocksPerThread = (kPairsMax * (kPairsMax + 1) / 2 + 1023) / 1024;
    int32_t bk1[kBlocksPerThread], bk2[kBlocksPerThread];
#pragma unroll
    for (int i = 0; i < kBlocksPerThread; i++) {
        int32_t rem = tid + i * 1024, k1 = 0;
        bk1[i] = -1;
        bk2[i] = 0;
        if (rem < half * (half + 1) / 2) {
            while (rem >= half - k1) {        // row k1 of the triangle holds half - k1 blocks
                rem -= half - k1;
                k1++;
            }
            bk1[i] = k1;
            bk2[i] = k1 + rem;
        }
    }

    int32_t stage_out = 0;
    for (int32_t sweep = 0; sweep < max_sweeps; sweep++) {
        for (int32_t r = 0; r < N - 1; r++) {
            if (tid < 64) {
                double c = 1.0, s = 0.0;
                int32_t p = 0, q = 0;
                if (tid < half) {
                    rr_pair(N, r, tid, p, q);
                    if (q < n) {
                        const double apq = A[p * kGgtLd + q];
                        const double app = A[p * kGgtLd + p], aqq = A[q * kGgtLd + q];
                        // Scaled by a power of two so that the largest of the two diagonal entries is in
                        // [1, 2): squares below neither overflow nor lose a pair that matters.
                        const double dmax = fmax(fabs(app), fabs(aqq));
                        if (apq != 0.0 && dmax > 0.0 && dmax < 1.0e300) {
                            const int ex = ilogb(dmax);
                            const double as = ldexp(apq, -ex), ps = ldexp(app, -ex), qs = ldexp(aqq, -ex);
                            // at rest when |apq| <= 2^-54 sqrt(|app aqq|), compared in squares
                            if (as * as > 0x1p-108 * fabs(ps * qs)) {
                                // t = tan of the rotation angle, the smaller root of t^2 + 2 tau t - 1 = 0,
                                // tau = (aqq - app) / (2 apq): t = sign(tau) / (|tau| + sqrt(1 + tau^2))
                                //     = apq sign(h) / (|h| + sqrt(h^2 + apq^2)),  h = (aqq - app) / 2
                                // (one square root and one division; h = 0 gives t = +-1)
                                const double h = 0.5 * (qs - ps);
                                const double hy = sqrt(h * h + as * as);
                                const double t = (h >= 0.0 ? as : -as) / (fabs(h) + hy);
                                c = rsqrt(1.0 + t * t);
                                s = t * c;
                                // A sweep whose rotations all have |t| <= 2^-27 leaves off-diagonal entries
                                // of relative size 2^-54 (each is annihilated once and then only moved by
                                // other angles of that size times entries of that size): such a sweep is the
                                // last one, and only larger rotations are counted.
                                if (t * t > 0x1p-54) atomicAdd(n_rot, 1);
                            }
                        }
                    }
                }
                cs[tid] = make_double2(c, s);
                rot[(int64_t)stage_out * 64 + tid] = make_double2(c, s);
                if (s != 0.0) {
                    const double yp = yv[p], yq = yv[q];
                    yv[p] = c * yp - s * yq;
                    yv[q] = s * yp + c * yq;
                }
            }
            __syncthreads();
            // A <- J^T A J, one 2x2 block per (row pair, column pair) and its mirror image; all
            // blocks are disjoint.  The pairs are recomputed rather than fetched from LDS.
#pragma unroll
            for (int i = 0; i < kBlocksPerThread; i++) {
                const int32_t k1 = bk1[i], k2 = bk2[i];
                if (k1 < 0) continue;
                int32_t p1, q1, p2, q2;
                rr_pair(N, r, k1, p1, q1);
                rr_pair(N, r, k2, p2, q2);
                const double2 r1 = cs[k1], r2 = cs[k2];
                if (r1.y == 0.0 && r2.y == 0.0) continue;   // both pairs at rest (late sweeps): block unchanged
                const double b00 = A[p1 * kGgtLd + p2], b01 = A[p1 * kGgtLd + q2];
                const double b10 = A[q1 * kGgtLd + p2], b11 = A[q1 * kGgtLd + q2];
                const double t00 = r2.x * b00 - r2.y * b01, t01 = r2.y * b00 + r2.x * b01;
                const double t10 = r2.x * b10 - r2.y * b11, t11 = r2.y * b10 + r2.x * b11;
                double n00 = r1.x * t00 - r1.y * t10, n01 = r1.x * t01 - r1.y * t11;
                double n10 = r1.y * t00 + r1.x * t10, n11 = r1.y * t01 + r1.x * t11;
                if (k1 == k2 && r1.y != 0.0) { n01 = 0.0; n10 = 0.0; }      // the annihilated entry
                A[p1 * kGgtLd + p2] = n00;
                A[p1 * kGgtLd + q2] = n01;
                A[q1 * kGgtLd + p2] = n10;
                A[q1 * kGgtLd + q2] = n11;
                if (k1 != k2) {
                    A[p2 * kGgtLd + p1] = n00;
                    A[q2 * kGgtLd + p1] = n01;
                    A[p2 * kGgtLd + q1] = n10;
                    A[q2 * kGgtLd + q1] = n11;
                }
            }
            __syncthreads();
            stage_out++;
        }
        const int32_t done = *n_rot == 0;     // read by all before it is cleared
        __syncthreads();
        if (tid == 0) *n_rot = 0;
        __syncthreads();
        if (done) break;                      // uniform: a whole sweep without a rotation that counts
    }
    if (tid < m) lam[tid] = tid < n ? A[tid * kGgtLd + tid] : 0.0;
    if (update && tid < m) vtq[tid] = yv[tid];
    if (tid == 0) *n_stages = stage_out;
}

// One wave.  y = V^T q by the logged rotations in order, z_i = y_i / (eps sigma_i (sigma_i + eps)),
// coef = V z by the log backwards.  q is sq[].x; coef of slots >= n is 0.
// have_y != 0: coef_out holds V^T q already (left there by k_ggt_eig in the same step), the forward
// pass is skipped.
__global__ __launch_bounds__(64) void k_ggt_coef(int32_t m, const StepState *__restrict__ step, double eps,
                                                 int32_t have_y,
                                                 const double2 *__restrict__ sq,
                                                 const double *__restrict__ lam,
                                                 const double2 *__restrict__ rot,
                                                 const int32_t *__restrict__ n_stages,
                                                 double *__restrict__ q_out, double *__restrict__ coef_out)
{
    __shared__ double y[kGgtMaxM + 2];
    const int lane = threadIdx.x;
    const int32_t n = step_view(step, m, kAfter).n_filled;
    const int32_t N = (n + 1) & ~1, half = N >> 1;
    const int32_t stages = *n_stages;
    double lmax = 0.0;
    for (int32_t i = lane; i < kGgtMaxM + 2; i += 64) {
        const double qi = i < n ? sq[i].x : 0.0;
        y[i] = (have_y && i < n) ? coef_out[i] : qi;
        if (i < m) q_out[i] = i < n ? qi : 0.0;
        if (i < n) lmax = fmax(lmax, lam[i]);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) lmax = fmax(lmax, __shfl_xor(lmax, o, 64));
    __syncthreads();

    // The log is read kLogAhead stages ahead of its use (a stage is one LDS round trip long, a
    // load of the log many): loads unconditional and clamped, stages past the end are identities.
    constexpr int kLogAhead = 8;
    auto fetch = [&](int32_t st0, int32_t dir, double2 (&b)[kLogAhead]) {
#pragma unroll
        for (int u = 0; u < kLogAhead; u++) {
            const int32_t st = st0 + dir * u;
            const double2 t = rot[(int64_t)min(max(st, 0), max(stages - 1, 0)) * 64 + lane];
            b[u] = (st >= 0 && st < stages) ? t : make_double2(1.0, 0.0);
        }
    };
    double2 ahead[kLogAhead];
    int32_t r = 0;
    if (!have_y) fetch(0, 1, ahead);
    for (int32_t st0 = 0; st0 < (have_y ? 0 : stages); st0 += kLogAhead) {
        double2 cur[kLogAhead];
#pragma unroll
        for (int u = 0; u < kLogAhead; u++) cur[u] = ahead[u];
        fetch(st0 + kLogAhead, 1, ahead);
#pragma unroll
        for (int u = 0; u < kLogAhead; u++) {
            if (lane < half && cur[u].y != 0.0) {          // (an identity past the end moves nothing)
                int32_t p, q;
                rr_pair(N, r, lane, p, q);
                const double yp = y[p], yq = y[q];
                y[p] = cur[u].x * yp - cur[u].y * yq;
                y[q] = cur[u].y * yp + cur[u].x * yq;
            }
            __syncthreads();
            r = r + 1 == N - 1 ? 0 : r + 1;
        }
    }
    const double cut = (double)n * 0x1p-52 * lmax;
    for (int32_t i = lane; i < n; i += 64) {
        const double l = lam[i];
        double z = 0.0;
        if (l > cut) {
            const double sg = sqrt(l);
            z = y[i] / (eps * sg * (sg + eps));
        }
        y[i] = z;
    }
    __syncthreads();
    // backwards: stage st used r = st mod (N-1)
    int32_t rb = stages > 0 ? (stages - 1) % (N - 1) : 0;
    fetch(stages - 1, -1, ahead);
    for (int32_t st0 = stages - 1; st0 >= 0; st0 -= kLogAhead) {
        double2 cur[kLogAhead];
#pragma unroll
        for (int u = 0; u < kLogAhead; u++) cur[u] = ahead[u];
        fetch(st0 - kLogAhead, -1, ahead);
#pragma unroll
        for (int u = 0; u < kLogAhead; u++) {
            if (lane < half && cur[u].y != 0.0) {
                int32_t p, q;
                rr_pair(N, rb, lane, p, q);
                const double zp = y[p], zq = y[q];
                y[p] = cur[u].x * zp + cur[u].y * zq;
                y[q] = -cur[u].y * zp + cur[u].x * zq;
            }
            __syncthreads();
            rb = rb == 0 ? N - 2 : rb - 1;
        }
    }
    for (int32_t i = lane; i < m; i += 64) coef_out[i] = i < n ? y[i] : 0.0;
}

size_t ggt_eig_lds_bytes()
{
    return (size_t)kGgtMaxM * kGgtLd * sizeof(double) + 64 * sizeof(double2) + 16 + (kGgtMaxM + 2) * sizeof(double);
}

hipError_t configure_ggt()
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(k_ggt_eig),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)ggt_eig_lds_bytes());
}

// Coefficients of the step: new Gram row/column, eigendecomposition, coefficients for q.
hipError_t launch_ggt_step(const Geometry &g, const DevicePtrs &p, double eps, hipStream_t stream)
{
    hipLaunchKernelGGL(k_ggt_eig, dim3(1), dim3(1024), ggt_eig_lds_bytes(), stream, g.m, p.step, 1, p.S,
                       p.sq, p.q, p.lam, p.rot, p.n_stages, kGgtMaxSweeps, p.coef);
    hipLaunchKernelGGL(k_ggt_coef, dim3(1), dim3(64), 0, stream, g.m, p.step, eps, 1, p.sq, p.lam, p.rot,
                       p.n_stages, p.q, p.coef);
    return hipGetLastError();
}

// Decomposition of S as it stands (after a state import), without touching S or q.
hipError_t launch_ggt_refresh(const Geometry &g, const DevicePtrs &p, hipStream_t stream)
{
    hipLaunchKernelGGL(k_ggt_eig, dim3(1), dim3(1024), ggt_eig_lds_bytes(), stream, g.m, p.step, 0, p.S,
                       p.sq, p.q, p.lam, p.rot, p.n_stages, kGgtMaxSweeps, p.coef);
    return hipGetLastError();
}

// Coefficients for another x on the window as it stands: the decomposition of the last step is reused.
hipError_t launch_ggt_apply(const Geometry &g, const DevicePtrs &p, double eps, hipStream_t stream)
{
    hipLaunchKernelGGL(k_ggt_coef, dim3(1), dim3(64), 0, stream, g.m, p.step, eps, 0, p.sq, p.lam, p.rot,
                       p.n_stages, p.q, p.coef);
    return hipGetLastError();
}

}  // namespace efcp
