// lcg.hip -- linear combination of the window rows and the output of eq. (2):
//   out_j = x_j / lambda - sum_r coef_r * c_r[j]
// (Section "Linear Combination of Gradients (LCG)", Section "Sparse LCG").
//
// Segmented by d-slice: one workgroup owns the coordinates of a slice and
// keeps their accumulators in LDS, so no global-memory atomics exist and two
// workgroups never touch the same output.  Inside the workgroup all 64
// 16-lane groups stream different rows at once; to make the sum independent
// of the order in which they arrive, every product coef_r * v is converted to
// a 64-bit fixed-point integer (unit chosen per step from sum_r |coef_r| max|c_r|
// so that the whole sum fits in 51 bits) and added with integer LDS
// atomics.  Integer addition is associative, hence the result is bit-stable
// from run to run, and the fixed-point grid (2^-50 of the largest possible
// sum) is far finer than the fp32 output.
#include "efcp_internal.h"

namespace efcp {

__device__ __forceinline__ int32_t lcg_slice_of_block(int32_t nsl)
{
    const int32_t per = (nsl + 7) >> 3;
    const int32_t xcd = blockIdx.x & 7, i = blockIdx.x >> 3;
    const int32_t s = xcd * per + i;
    return (i < per && s < nsl) ? s : -1;
}

constexpr int kLcgChunksAhead = 3;

struct LcgBatch {
    int4 iv[kLcgChunksAhead];
    float4 vv[kLcgChunksAhead];
    int32_t p0, p1;
    double c;
};

__device__ __forceinline__ void lcg_issue(const int32_t *__restrict__ idx_row,
                                          const float *__restrict__ val_row, int32_t p0, int32_t p1,
                                          double c, int gl, LcgBatch &b)
{
    b.p0 = p0;
    b.p1 = p1;
    b.c = c;
#pragma unroll
    for (int q = 0; q < kLcgChunksAhead; q++) {
        // always load (from the row start when the chunk lies past the run) so that the
        // number of loads in flight is known and later waits need not drain the prefetch
        const int32_t pc = (p0 & ~3) + gl * 4 + q * 64;
        const int32_t pcs = pc < p1 ? pc : 0;
        b.iv[q] = *reinterpret_cast<const int4 *>(idx_row + pcs);
        b.vv[q] = *reinterpret_cast<const float4 *>(val_row + pcs);
    }
}

// round(c*v / unit) as an integer: the magic constant puts the product's
// units digit at the last mantissa bit; integer LDS atomics add it.
__device__ __forceinline__ void lcg_scatter(const int4 &iv, const float4 &vv, int32_t pc, int32_t p0,
                                            int32_t p1, int32_t base, int32_t mask, double c,
                                            double magic, long long magic_bits,
                                            unsigned long long *__restrict__ acc)
{
    const int32_t ii[4] = {iv.x, iv.y, iv.z, iv.w};
    const float fv[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
    for (int q = 0; q < 4; q++) {
        const int32_t p = pc + q;
        if (p >= p0 && p < p1) {
            const int32_t li = (ii[q] - base) & mask;
            const double t = fma(c, (double)fv[q], magic);
            const long long cnt = __double_as_longlong(t) - magic_bits;
            atomicAdd(&acc[li], (unsigned long long)cnt);
        }
    }
}

__global__ __launch_bounds__(1024) void k_lcg(const float *__restrict__ x, float *__restrict__ out,
                                              int64_t d, int32_t m, int32_t n_filled, int64_t row_stride,
                                              int32_t slice_log2, int32_t nsl,
                                              const int32_t *__restrict__ ring_idx,
                                              const float *__restrict__ ring_val,
                                              const int32_t *__restrict__ offT,
                                              const double *__restrict__ coef,
                                              const uint32_t *__restrict__ rowmax,
                                              uint32_t *__restrict__ status, double inv_lambda)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int32_t slice = 1 << slice_log2;
    unsigned long long *acc = reinterpret_cast<unsigned long long *>(smem);   // [slice]
    double *cf = reinterpret_cast<double *>(acc + slice);                     // [1024]
    int32_t *off0 = reinterpret_cast<int32_t *>(cf + kMaxM);                  // [1024]
    int32_t *off1 = off0 + kMaxM;                                             // [1024]
    __shared__ double wsum[16];

    const int32_t s = lcg_slice_of_block(nsl);
    if (s < 0) return;
    const int64_t base64 = (int64_t)s << slice_log2;
    const int32_t base = (int32_t)base64;
    const int32_t len = (int32_t)min((int64_t)slice, d - base64);
    const int32_t mask = slice - 1;
    const int tid = threadIdx.x;

    for (int32_t i = tid; i < slice; i += 1024) acc[i] = 0ull;
    double cabs = 0.0;
    if (tid < m) {
        off0[tid] = offT[(int64_t)s * m + tid];
        off1[tid] = offT[(int64_t)(s + 1) * m + tid];
        const double c = tid < n_filled ? coef[tid] : 0.0;
        cf[tid] = c;
        // |coef_r| * (upper bound of the largest |value| of row r)
        cabs = fabs(c) * (double)__uint_as_float(tid < n_filled ? rowmax[tid] : 0u);
    }
    // Fixed-point unit: bound = sum_r |coef_r| max|c_r| >= |any partial sum|; 2^ex >= bound,
    // unit = 2^(ex-50), so every sum fits in 51 bits.  Same reduction order in every workgroup.
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) cabs += __shfl_xor(cabs, o, 64);
    if ((tid & 63) == 0) wsum[tid >> 6] = cabs;
    __syncthreads();
    double bound = 0.0;
#pragma unroll
    for (int i = 0; i < 16; i++) bound += wsum[i];
    int ex = 0;
    if (bound > 0.0 && bound < 1.0e300) {
        ex = ilogb(bound) + 1;
        ex = ex < -900 ? -900 : (ex > 900 ? 900 : ex);
    } else if (bound != 0.0) {
        if (tid == 0 && blockIdx.x == 0) atomicOr(status, kStatusRange);
    }
    const double unit = ldexp(1.0, ex - 50);
    const double magic = ldexp(1.5, ex + 2);          // 1.5 * 2^52 * unit
    const long long magic_bits = __double_as_longlong(magic);

    const int grp = tid >> 4, gl = tid & 15;
    int32_t r = grp;
    LcgBatch cur, nxt;
    {
        const int32_t rc = min(r, n_filled - 1);
        lcg_issue(ring_idx + (int64_t)rc * row_stride, ring_val + (int64_t)rc * row_stride, off0[rc],
                  off1[rc], cf[rc], gl, cur);
    }
    while (r < n_filled) {
        const int32_t rn = r + kRowGroups;
        {   // prefetch the next row of this group (a harmless repeat of the last row at the end)
            const int32_t rc = min(rn, n_filled - 1);
            lcg_issue(ring_idx + (int64_t)rc * row_stride, ring_val + (int64_t)rc * row_stride,
                      off0[rc], off1[rc], cf[rc], gl, nxt);
        }
        const int32_t pc0 = (cur.p0 & ~3) + gl * 4;
#pragma unroll
        for (int q = 0; q < kLcgChunksAhead; q++)
            lcg_scatter(cur.iv[q], cur.vv[q], pc0 + q * 64, cur.p0, cur.p1, base, mask, cur.c, magic,
                        magic_bits, acc);
        for (int32_t pc = pc0 + kLcgChunksAhead * 64; pc < cur.p1; pc += 64) {
            const int64_t rb = (int64_t)r * row_stride;
            const int4 iv = *reinterpret_cast<const int4 *>(ring_idx + rb + pc);
            const float4 vv = *reinterpret_cast<const float4 *>(ring_val + rb + pc);
            lcg_scatter(iv, vv, pc, cur.p0, cur.p1, base, mask, cur.c, magic, magic_bits, acc);
        }
        cur = nxt;
        r = rn;
    }
    __syncthreads();

    for (int32_t i = tid * 4; i < slice; i += 4096) {
        if (i >= len) break;
        float o[4];
        float xv[4];
        if (i + 3 < len) {
            const float4 t = *reinterpret_cast<const float4 *>(x + base64 + i);
            xv[0] = t.x; xv[1] = t.y; xv[2] = t.z; xv[3] = t.w;
        } else {
#pragma unroll
            for (int q = 0; q < 4; q++) xv[q] = (i + q < len) ? x[base64 + i + q] : 0.0f;
        }
#pragma unroll
        for (int q = 0; q < 4; q++) {
            const double sum = (double)(long long)acc[i + q] * unit;
            o[q] = (float)((double)xv[q] * inv_lambda - sum);
        }
        if (i + 3 < len) {
            *reinterpret_cast<float4 *>(out + base64 + i) = make_float4(o[0], o[1], o[2], o[3]);
        } else {
#pragma unroll
            for (int q = 0; q < 4; q++)
                if (i + q < len) out[base64 + i + q] = o[q];
        }
    }
}

hipError_t launch_lcg(const Geometry &g, const DevicePtrs &p, const float *x, float *out,
                      int32_t n_filled, double lambda, hipStream_t stream)
{
    const int32_t per = (g.n_slices + 7) / 8;
    hipLaunchKernelGGL(k_lcg, dim3(per * 8), dim3(1024), g.lds_lcg, stream, x, out, g.d, g.m, n_filled,
                       g.row_stride, g.slice_log2, g.n_slices, p.ring_idx, p.ring_val, p.offT, p.coef,
                       p.rowmax, p.status, 1.0 / lambda);
    return hipGetLastError();
}

hipError_t configure_lcg(const Geometry &g)
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(k_lcg),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)g.lds_lcg);
}

}  // namespace efcp
