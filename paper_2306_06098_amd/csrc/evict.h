// evict.h -- deleting the oldest row from the inverse factor W = L^-1 of the coefficient step
// (see coef.hip for the factor and the other two kernels), as a function one workgroup of 1024
// threads runs per 16 columns: it is part of the kernel that opens the selection of the global
// Top-k (the machine is nearly idle there) and a kernel of its own otherwise.
#pragma once
#include "efcp_internal.h"

namespace efcp {

// ------------------------------------------------------------------
// Delete the oldest row (slot `old`) from the inverse factor.
// Ages a = 0..m-2 of the surviving rows map to slots (old + 1 + a) mod m.
// With sigma_a = 1 + sum_{b<a} p_b^2:
//   K_aa = sqrt(sigma_{a+1}/sigma_a),  K_ab = p_a p_b / sqrt(sigma_b sigma_{b+1})  (a > b)
// and Y = K^-1 W22 row by row:  Y_a = (W_a - p_a R_a) / K_aa,
//   R_{a+1} = R_a + p_a / sqrt(sigma_a sigma_{a+1}) * Y_a,  R_0 = 0.
// The recurrence is affine in R: R_{a+1} = (sigma_a/sigma_{a+1}) R_a + (...) W_a.  A block owns
// 16 columns and splits the rows into 64 chunks of 16 ages: a thread loads its 16 entries of one
// column once (all loads independent of every other chunk), runs them from R = 0, the chunk
// results are chained through LDS with the closed-form factor sigma_start/sigma_end (one thread per
// column walks the chunks), and the
// thread runs its 16 entries again, from registers, with the right starting value and stores
// them.  Memory is thus waited for three times in all (first column, entries, nothing after the
// stores), which keeps the kernel short also while a d-sized pass saturates the memory system
// beside it.  Column `old` is left alone (k_bwd clears it).
constexpr int kEvictCols = 16, kEvictAges = 16, kEvictChunks = kMaxM / kEvictAges;
__host__ __device__ constexpr int32_t evict_blocks(int32_t m) { return (m + kEvictCols - 1) / kEvictCols; }

// blk: which 16 columns (0 .. evict_blocks(m) - 1); every thread of the workgroup must call it.
__device__ __forceinline__ void evict_block(int32_t blk, int32_t m, int32_t ldm, int32_t old,
                                            double *__restrict__ W)
{
    __shared__ double s_p[kMaxM], s_ik[kMaxM], s_g[kMaxM], s_sig[kMaxM + 1];
    __shared__ double s_wave[16];
    __shared__ double s_ratio[kEvictChunks];
    __shared__ double s_B[kEvictChunks][kEvictCols];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform
    const int n = m - 1;                      // surviving rows
    auto slot_of = [&](int a) {               // age a (< m) of the surviving rows -> slot
        const int r = old + 1 + a;
        return r >= m ? r - m : r;
    };

    // this thread's entries, requested before anything else: column cl of the block, ages
    // a_lo .. a_lo + 15 (loads unconditional and clamped, values masked: conditional loads
    // would be waited for one by one)
    const int cl = tid & (kEvictCols - 1), ch = tid >> 4;
    const int col = blk * kEvictCols + cl;
    const bool live = (col < m) && (col != old);
    const int colc = min(col, m - 1);
    const int a_lo = ch * kEvictAges;
    double v[kEvictAges];
#pragma unroll
    for (int u = 0; u < kEvictAges; u++)
        v[u] = W[(int64_t)slot_of(min(a_lo + u, n)) * ldm + colc];
    const double w00 = W[(int64_t)old * ldm + old];
    const double wp = W[(int64_t)slot_of(min(tid, n)) * ldm + old];
#pragma unroll
    for (int u = 0; u < kEvictAges; u++)
        if (!(live && a_lo + u < n)) v[u] = 0.0;

    // thread a: p_a, then sigma by an exclusive scan of p^2 in age order
    const double p = tid < n ? -wp * (1.0 / w00) : 0.0;
    const double p2 = p * p;
    double incl = p2;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const double t = __shfl_up(incl, o, 64);
        if (lane >= o) incl += t;
    }
    if (lane == 63) s_wave[wv] = incl;
    __syncthreads();
    double before = 1.0;                      // sigma_0 = 1
#pragma unroll
    for (int i = 0; i < 16; i++) before += i < wv ? s_wave[i] : 0.0;     // (all 16 reads at once)
    const double sigma = before + (incl - p2);
    const double nxt = sigma + p2;
    const double rs = 1.0 / sqrt(sigma * nxt);    // 1/K_aa = sqrt(sigma/nxt) = sigma * rs
    s_p[tid] = p;
    s_ik[tid] = sigma * rs;
    s_g[tid] = p * rs;
    s_sig[tid] = sigma;
    if (tid == 1023) s_sig[1024] = nxt;
    __syncthreads();
    if (tid < kEvictChunks) s_ratio[tid] = s_sig[tid * kEvictAges] / s_sig[tid * kEvictAges + kEvictAges];

    // sweep 1: this thread's ages starting from R = 0
    double R = 0.0;
#pragma unroll
    for (int u = 0; u < kEvictAges; u++) {
        const int a = a_lo + u;
        const double y = (v[u] - s_p[a] * R) * s_ik[a];
        R = fma(s_g[a], y, R);
    }
    s_B[ch][cl] = R;
    __syncthreads();
    // chain the chunks: the value a chunk starts from is R_in(c+1) = R_in(c) * sigma_start(c)/sigma_end(c)
    // + B_c, R_in(0) = 0.  One thread per column walks the 64 chunks and leaves R_in in place of B
    // (every thread doing the walk for itself is 1 MB of LDS reads per workgroup, a quarter of the
    // whole update's time).
    if (tid < kEvictCols) {
        double Rin = 0.0;
#pragma unroll 8
        for (int c = 0; c < kEvictChunks; c++) {
            const double t = s_B[c][tid];
            s_B[c][tid] = Rin;
            Rin = fma(Rin, s_ratio[c], t);
        }
    }
    __syncthreads();
    R = s_B[ch][cl];

    // sweep 2: the same entries with the right start, stored
#pragma unroll
    for (int u = 0; u < kEvictAges; u++) {
        const int a = a_lo + u;
        const double y = (v[u] - s_p[a] * R) * s_ik[a];
        R = fma(s_g[a], y, R);
        if (live && a < n) W[(int64_t)slot_of(a) * ldm + col] = y;
    }
}

}  // namespace efcp
