// sp.hip -- scalar products of every window row with the dense vector x and
// with the newest row: q_r = <c_r, x> and the Gram row S[slot][r] = <c_r, c_new>
// (Section "Scalar Products (SP)", Section "Sparse Scalar Products").
//
// Traversal is by d-slice, not by row: one workgroup stages x[slice] and the
// newest row scattered to dense in LDS (interleaved float2, one 8-byte LDS
// gather serves both products), then streams the index/value runs of all
// filled rows that fall in the slice.  x is read from HBM once and every
// gather is an LDS access.  A 16-lane group owns one row at a time and reads
// its run with 16-byte loads; products of two fp32 values are exact in fp64
// and are accumulated in fp64.  Per-(slice,row) partial sums go to a scratch
// array and are added in a fixed order by k_sp_reduce, so the result does not
// depend on scheduling.
#include "efcp_internal.h"

namespace efcp {

// Slice handled by a workgroup: consecutive slices share an XCD (workgroups
// are dealt to the 8 XCDs round-robin), so the cache line that straddles two
// neighbouring runs of a row is fetched into one L2 only.
__device__ __forceinline__ int32_t slice_of_block(int32_t nsl)
{
    const int32_t per = (nsl + 7) >> 3;
    const int32_t xcd = blockIdx.x & 7, i = blockIdx.x >> 3;
    const int32_t s = xcd * per + i;
    return (i < per && s < nsl) ? s : -1;
}

__global__ __launch_bounds__(1024) void k_sp(const float *__restrict__ x, int64_t d, int32_t m,
                                             int32_t n_filled, int32_t slot, int64_t row_stride,
                                             int32_t slice_log2, int32_t nsl,
                                             const int32_t *__restrict__ ring_idx,
                                             const float *__restrict__ ring_val,
                                             const int32_t *__restrict__ offT,
                                             double2 *__restrict__ partial)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int32_t slice = 1 << slice_log2;
    float2 *xc = reinterpret_cast<float2 *>(smem);                 // [slice]: (x_j, c_new_j)
    int32_t *off0 = reinterpret_cast<int32_t *>(xc + slice);       // [1024]
    int32_t *off1 = off0 + kMaxM;                                  // [1024]

    const int32_t s = slice_of_block(nsl);
    if (s < 0) return;
    const int64_t base = (int64_t)s << slice_log2;
    const int32_t len = (int32_t)min((int64_t)slice, d - base);
    const int tid = threadIdx.x;

    for (int32_t i = tid * 4; i < slice; i += 4096) {
        float4 xv;
        if (i + 3 < len) {
            xv = *reinterpret_cast<const float4 *>(x + base + i);
        } else {
            xv.x = (i + 0 < len) ? x[base + i + 0] : 0.0f;
            xv.y = (i + 1 < len) ? x[base + i + 1] : 0.0f;
            xv.z = (i + 2 < len) ? x[base + i + 2] : 0.0f;
            xv.w = (i + 3 < len) ? x[base + i + 3] : 0.0f;
        }
        xc[i + 0] = make_float2(xv.x, 0.0f);
        xc[i + 1] = make_float2(xv.y, 0.0f);
        xc[i + 2] = make_float2(xv.z, 0.0f);
        xc[i + 3] = make_float2(xv.w, 0.0f);
    }
    for (int32_t r = tid; r < m; r += 1024) {
        off0[r] = offT[(int64_t)s * m + r];
        off1[r] = offT[(int64_t)(s + 1) * m + r];
    }
    __syncthreads();
    {   // scatter the newest row's entries of this slice next to x
        const int64_t rb = (int64_t)slot * row_stride;
        const int32_t p1 = off1[slot];
        for (int32_t p = off0[slot] + tid; p < p1; p += 1024) {
            const int32_t li = (ring_idx[rb + p] - (int32_t)base) & (slice - 1);
            xc[li].y = ring_val[rb + p];
        }
    }
    __syncthreads();

    const int grp = tid >> 4, gl = tid & 15;
    for (int32_t r = grp; r < n_filled; r += kRowGroups) {
        const int64_t rb = (int64_t)r * row_stride;
        const int32_t p0 = off0[r], p1 = off1[r];
        double aq = 0.0, ag = 0.0;
        for (int32_t pc = (p0 & ~3) + gl * 4; pc < p1; pc += 64) {
            const int4 iv = *reinterpret_cast<const int4 *>(ring_idx + rb + pc);
            const float4 vv = *reinterpret_cast<const float4 *>(ring_val + rb + pc);
            const int32_t ii[4] = {iv.x, iv.y, iv.z, iv.w};
            const float fv[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
            for (int c = 0; c < 4; c++) {
                const int32_t p = pc + c;
                const bool ok = (p >= p0) && (p < p1);
                const int32_t li = ok ? ((ii[c] - (int32_t)base) & (slice - 1)) : 0;
                const double v = ok ? (double)fv[c] : 0.0;
                const float2 t = xc[li];
                aq = fma(v, (double)t.x, aq);
                ag = fma(v, (double)t.y, ag);
            }
        }
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) {
            aq += __shfl_xor(aq, o, 16);
            ag += __shfl_xor(ag, o, 16);
        }
        if (gl == 0) partial[(int64_t)s * m + r] = make_double2(aq, ag);
    }
}

// First level of the fixed-order reduction over slices: block (bx, by) adds
// the partial sums of 64 rows over slice group by.
__global__ __launch_bounds__(1024) void k_sp_reduce(const double2 *__restrict__ partial, int32_t m,
                                                    int32_t n_filled, int32_t nsl, int32_t per_group,
                                                    double2 *__restrict__ partial2)
{
    __shared__ double2 sh[16][64];
    const int rl = threadIdx.x & 63, sl = threadIdx.x >> 6;
    const int32_t r = blockIdx.x * 64 + rl;
    const int32_t s0 = blockIdx.y * per_group, s1 = min(nsl, s0 + per_group);
    double ax = 0.0, ay = 0.0;
    if (r < n_filled) {
        for (int32_t s = s0 + sl; s < s1; s += 16) {
            const double2 t = partial[(int64_t)s * m + r];
            ax += t.x;
            ay += t.y;
        }
    }
    sh[sl][rl] = make_double2(ax, ay);
    __syncthreads();
    if (sl == 0 && r < m) {
        double sx = 0.0, sy = 0.0;
#pragma unroll
        for (int i = 0; i < 16; i++) {
            sx += sh[i][rl].x;
            sy += sh[i][rl].y;
        }
        partial2[(int64_t)blockIdx.y * m + r] = make_double2(sx, sy);
    }
}

hipError_t launch_sp(const Geometry &g, const DevicePtrs &p, const float *x, int32_t n_filled,
                     int32_t slot, hipStream_t stream)
{
    const int32_t per = (g.n_slices + 7) / 8;
    hipLaunchKernelGGL(k_sp, dim3(per * 8), dim3(1024), g.lds_sp, stream, x, g.d, g.m, n_filled, slot,
                       g.row_stride, g.slice_log2, g.n_slices, p.ring_idx, p.ring_val, p.offT, p.partial);
    return hipGetLastError();
}

hipError_t launch_sp_reduce(const Geometry &g, const DevicePtrs &p, int32_t n_filled, hipStream_t stream)
{
    const int32_t per_group = (g.n_slices + g.n_groups - 1) / g.n_groups;
    hipLaunchKernelGGL(k_sp_reduce, dim3((g.m + 63) / 64, g.n_groups), dim3(1024), 0, stream, p.partial,
                       g.m, n_filled, g.n_slices, per_group, p.partial2);
    return hipGetLastError();
}

hipError_t configure_sp(const Geometry &g)
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(k_sp),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)g.lds_sp);
}

}  // namespace efcp
