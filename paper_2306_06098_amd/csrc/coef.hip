// coef.hip -- the m x m part of the step: coefficients of eq. (2),
//   coef = (1/lambda) (m*lambda*I + S)^-1 q,
// which is what the WSM recursion of Section "Efficient Full-Matrix
// Preconditioners" produces (Woodbury identity applied to
// F = lambda*I + (1/m) sum_r c_r c_r^T).  fp64 throughout, O(m^2) per step.
//
// State: W = L^-1, the inverse of the Cholesky factor of A = m*lambda*I + S
// with rows in age order (oldest first), so A^-1 = W^T W.  W is stored
// row-major by window slot (W(i,j) at W[i*ldm + j]); entries above the
// diagonal *in age order*, and rows/columns of unfilled slots, are kept at
// exactly zero, so every product below may run over full rows and columns.
// Keeping the inverse factor instead of the factor turns the two triangular
// solves of a step (a chain of m dependent column steps each) into plain
// matrix-vector products that many workgroups share:
//
//   evict     (window already full; evict.h, run by the first selection kernel or by k_evict)
//             delete the oldest row/column of A.
//             If A = [[a11, a^T], [a, A22]], L = [[l11, 0], [l, L22]] then
//             A22 = L22 (I + p p^T) L22^T with p = L22^-1 l, and with the
//             Cholesky factor K of I + p p^T (closed form, below) the new
//             inverse factor is K^-1 W22.  K is "diagonal plus rank-one
//             below the diagonal", so K^-1 W22 is one running sum per column:
//             columns are independent and need no barrier.  p comes from the
//             first column of W itself: p = -W(:,old) / W(old,old).
//   k_fwd     z = W s and w = W q for the new Gram column s and for q.
//   k_bwd     new diagonal l = sqrt(a_nn - z^T z), w_n = (q_n - z^T w)/l,
//             coef = (1/lambda) [W^T (w - z w_n/l) ; w_n/l], and the new last
//             row of W: [-(W^T z)/l , 1/l].
//
// All reductions have a fixed shape, so results do not depend on scheduling.
#include "efcp_internal.h"
#include "evict.h"

namespace efcp {

__device__ __forceinline__ double wave_sum_f64(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// Two sums over the 1024 threads of a block at once, each in a fixed order.  buf: 32 doubles.
__device__ __forceinline__ void block_sum2_f64_1024(double &a, double &b, double *buf)
{
    a = wave_sum_f64(a);
    b = wave_sum_f64(b);
    if ((threadIdx.x & 63) == 0) {
        buf[threadIdx.x >> 6] = a;
        buf[16 + (threadIdx.x >> 6)] = b;
    }
    __syncthreads();
    double ra = 0.0, rb = 0.0;
#pragma unroll
    for (int i = 0; i < 16; i++) {
        ra += buf[i];
        rb += buf[16 + i];
    }
    __syncthreads();
    a = ra;
    b = rb;
}

// ------------------------------------------------------------------
// Delete the oldest row from the inverse factor (evict.h) as a kernel of its own: the step with
// Top-k in blocks, which has no selection kernels to carry it.  It is part of every such step
// and returns at once while the window is not yet full.
__global__ __launch_bounds__(1024) void k_evict(int32_t m, int32_t ldm, const StepState *__restrict__ step,
                                                double *__restrict__ W)
{
    const StepView sv = step_view(step, m, kBefore);
    if (!sv.evict) return;                    // uniform: nothing is replaced by this step
    evict_block(blockIdx.x, m, ldm, sv.slot, W);
}

// ------------------------------------------------------------------
// z = W s, w = W q.  One wave per row; sq[j] = (q_j, s_j).  The entry of the
// slot being (re)written is excluded on both sides.
// whole != 0 (efcp_apply): no slot is being rewritten, the product runs over the whole factor.
__global__ __launch_bounds__(256) void k_fwd(int32_t m, int32_t ldm, const StepState *__restrict__ step,
                                             int32_t whole, const double *__restrict__ W,
                                             const double2 *__restrict__ sq,
                                             double2 *__restrict__ zw)
{
    __shared__ double2 s_sq[kMaxM];
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // The row of W is requested first, before anything is known about the step: all its loads at
    // once (m <= 1024: at most 16 per lane); a column past the end is read again from the last
    // one and meets an exact zero in s_sq, a row past the end is the last row and is dropped.
    double v[kMaxM / 64];
    {
        const double *wr = W + (int64_t)min(row, m - 1) * ldm;
#pragma unroll
        for (int u = 0; u < kMaxM / 64; u++) v[u] = wr[min(lane + 64 * u, m - 1)];
    }
    // ... and so is (q, s): unconditional loads (clamped), masked once the slot is known, so that
    // the kernel waits for memory once
    double2 t_sq[kMaxM / 256];
#pragma unroll
    for (int u = 0; u < kMaxM / 256; u++) t_sq[u] = sq[min((int)threadIdx.x + 256 * u, m - 1)];
    const int32_t slot = whole ? -1 : step_view(step, m, kAfter).slot;
#pragma unroll
    for (int u = 0; u < kMaxM / 256; u++) {
        const int j = threadIdx.x + 256 * u;
        s_sq[j] = (j < m && j != slot) ? t_sq[u] : make_double2(0.0, 0.0);
    }
    __syncthreads();
    if (row >= m) return;
    double az = 0.0, aw = 0.0;
    if (row != slot) {
#pragma unroll
        for (int u = 0; u < kMaxM / 64; u++) {
            const double2 t = s_sq[lane + 64 * u];
            aw = fma(v[u], t.x, aw);
            az = fma(v[u], t.y, az);
        }
    }
    az = wave_sum_f64(az);
    aw = wave_sum_f64(aw);
    if (lane == 0) zw[row] = make_double2(az, aw);
}

// ------------------------------------------------------------------
// Block b owns the kBwdCols columns [16b, 16b+16); thread (rg, cl) adds rows rg, rg+64, ... of
// column cl, so 64 blocks share the one pass over W and a thread waits for 16 loads, not 64.
constexpr int kBwdCols = 16;

__global__ __launch_bounds__(1024) void k_bwd(int32_t m, int32_t ldm, const StepState *__restrict__ step,
                                              double lambda, double *__restrict__ W,
                                              const double2 *__restrict__ sq,
                                              const double2 *__restrict__ zw,
                                              double *__restrict__ S, double *__restrict__ q_out,
                                              double *__restrict__ coef_out,
                                              uint32_t *__restrict__ status)
{
    __shared__ double s_z[kMaxM], s_r[kMaxM];
    __shared__ double2 s_sq[kMaxM];
    __shared__ double buf[32];
    __shared__ double2 red[64][kBwdCols];

    const int tid = threadIdx.x;
    const int cl = tid & (kBwdCols - 1), rg = tid >> 4;          // 16 columns x 64 row groups
    const int col = blockIdx.x * kBwdCols + cl;
    const int colc = min(col, m - 1);
    // This thread's 16 entries of W are requested first (they depend on nothing): rows past the
    // end are read again from the last one and meet exact zeros below.
    double wv[kMaxM / 64];
#pragma unroll
    for (int u = 0; u < kMaxM / 64; u++) wv[u] = W[(int64_t)min(rg + 64 * u, m - 1) * ldm + colc];
    // ... and with them everything else the block reads, whatever the slot turns out to be: the
    // kernel waits for memory once
    const double2 t_zw = zw[min(tid, m - 1)];
    const double2 t_sq = sq[min(tid, m - 1)];
    const double2 sqc = sq[colc];
    const int32_t slot = step_view(step, m, kAfter).slot;         // the slot written by this step
    s_sq[tid] = t_sq;
    double z = 0.0, w = 0.0;
    if (tid < m && tid != slot) {
        z = t_zw.x;
        w = t_zw.y;
    }
    double zz = z * z, zwd = z * w;
    block_sum2_f64_1024(zz, zwd, buf);               // (its barrier also publishes s_sq)
    const double2 sqn = s_sq[slot];                  // (q_n, s_nn)
    const double mlam = (double)m * lambda;
    double piv = sqn.y + mlam - zz;
    if (!(piv >= mlam)) {                            // the exact Schur complement is >= m*lambda
        piv = mlam;
        if (blockIdx.x == 0 && tid == 0) atomicOr(status, kStatusPivot);
    }
    const double l = sqrt(piv);
    const double wn = (sqn.x - zwd) / l;
    const double f = wn / l;
    s_z[tid] = z;
    s_r[tid] = (tid < m && tid != slot) ? (w - z * f) : 0.0;
    __syncthreads();

    double ac = 0.0, ay = 0.0;
    // row `slot` needs no skip: s_r[slot] = s_z[slot] = 0 and the row holds finite values
#pragma unroll
    for (int u = 0; u < kMaxM / 64; u++) {
        ac = fma(wv[u], s_r[rg + 64 * u], ac);
        ay = fma(wv[u], s_z[rg + 64 * u], ay);
    }
    red[rg][cl] = make_double2(ac, ay);
    __syncthreads();
    if (col < m && col == slot) {
        // column of the slot that was rewritten: nothing older may refer to it
        for (int i = rg; i < m; i += 64)
            if (i != slot) W[(int64_t)i * ldm + col] = 0.0;
    }
    if (rg == 0 && col < m) {
        double c = 0.0, y = 0.0;
        for (int i = 0; i < 64; i++) {               // fixed order
            c += red[i][cl].x;
            y += red[i][cl].y;
        }
        double coef;
        if (col == slot) {
            coef = f / lambda;
            W[(int64_t)slot * ldm + slot] = 1.0 / l;
        } else {
            coef = c / lambda;
            W[(int64_t)slot * ldm + col] = -y / l;
        }
        coef_out[col] = coef;
        q_out[col] = sqc.x;
        S[(int64_t)slot * m + col] = sqc.y;
        S[(int64_t)col * m + slot] = sqc.y;
    }
}

// ------------------------------------------------------------------
// Coefficients for a vector applied to the window as it stands: with w = W q over all rows,
// coef = (1/lambda) W^T w.  Block b owns columns [64b, 64b+64); its 16 waves split the rows.
__global__ __launch_bounds__(1024) void k_apply_bwd(int32_t m, int32_t ldm, double lambda,
                                                    const double *__restrict__ W,
                                                    const double2 *__restrict__ sq,
                                                    const double2 *__restrict__ zw,
                                                    double *__restrict__ q_out,
                                                    double *__restrict__ coef_out)
{
    __shared__ double s_w[kMaxM];
    __shared__ double red[16][64];
    const int tid = threadIdx.x;
    s_w[tid] = tid < m ? zw[tid].y : 0.0;
    __syncthreads();
    const int lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = blockIdx.x * 64 + lane;
    const int colc = min(col, m - 1);
    double ac = 0.0;
    for (int i = wv; i < m; i += 16) ac = fma(W[(int64_t)i * ldm + colc], s_w[i], ac);
    red[wv][lane] = ac;
    __syncthreads();
    if (wv == 0 && col < m) {
        double c = 0.0;
#pragma unroll
        for (int i = 0; i < 16; i++) c += red[i][lane];
        coef_out[col] = c / lambda;
        q_out[col] = sq[col].x;
    }
}

hipError_t launch_evict(const Geometry &g, const DevicePtrs &p, hipStream_t stream)
{
    hipLaunchKernelGGL(k_evict, dim3(evict_blocks(g.m)), dim3(1024), 0, stream, g.m, g.ldm, p.step, p.W);
    return hipGetLastError();
}

hipError_t launch_coef(const Geometry &g, const DevicePtrs &p, double lambda, hipStream_t stream)
{
    hipLaunchKernelGGL(k_fwd, dim3((g.m + 3) / 4), dim3(256), 0, stream, g.m, g.ldm, p.step, 0, p.W, p.sq,
                       p.zw);
    hipLaunchKernelGGL(k_bwd, dim3((g.m + kBwdCols - 1) / kBwdCols), dim3(1024), 0, stream, g.m, g.ldm, p.step,
                       lambda, p.W, p.sq, p.zw, p.S, p.q, p.coef, p.status);
    return hipGetLastError();
}

hipError_t launch_coef_apply(const Geometry &g, const DevicePtrs &p, double lambda, hipStream_t stream)
{
    // no row is left out; unfilled rows and columns of W are exact zeros
    hipLaunchKernelGGL(k_fwd, dim3((g.m + 3) / 4), dim3(256), 0, stream, g.m, g.ldm, p.step, 1, p.W, p.sq, p.zw);
    hipLaunchKernelGGL(k_apply_bwd, dim3((g.m + 63) / 64), dim3(1024), 0, stream, g.m, g.ldm, lambda, p.W,
                       p.sq, p.zw, p.q, p.coef);
    return hipGetLastError();
}

}  // namespace efcp
