// lcg.hip -- linear combination of the window rows and the output of eq. (2):
//   out_j = x_j / lambda - sum_r coef_r * c_r[j]
// (Section "Linear Combination of Gradients (LCG)", Section "Sparse LCG").
//
// Segmented by d-slice: one workgroup owns the coordinates of a slice and
// keeps their accumulators in LDS, so no global-memory atomics exist and two
// workgroups never touch the same output.  Inside the workgroup all 64
// 16-lane groups (256 4-lane groups where a row has few entries per slice)
// stream different rows at once; to make the sum independent
// of the order in which they arrive, every product coef_r * v is converted to
// a 64-bit fixed-point integer (unit chosen per step from sum_r |coef_r| max|c_r|
// so that the whole sum fits in 51 bits) and added with integer LDS
// atomics.  Integer addition is associative, hence the result is bit-stable
// from run to run, and the fixed-point grid (2^-50 of the largest possible
// sum) is far finer than the fp32 output.
#include "efcp_internal.h"

#include <type_traits>

namespace efcp {

// One batch = up to kBatch chunks of one row's run in the slice (see the SP pass).  A run
// longer than a batch is continued by the next batch (same row, pcs advanced), so the row
// loop has a single shape and the number of loads in flight is always known.
template <int FMT>
struct LcgBatch {
    typename Fmt<FMT>::iraw_t iv[Fmt<FMT>::kBatch];
    int4 vv[Fmt<FMT>::kBatch];
    int32_t r;          // row (may be >= n_filled: then nothing is valid)
    int32_t pcs;        // position of chunk 0, lane 0 (multiple of EPL)
    int32_t p0, p1;     // the row's run in this slice
    double c;
};

// round(c*v / unit) as an integer: the magic constant puts the product's
// units digit at the last mantissa bit; integer LDS atomics add it.
template <int FMT>
__device__ __forceinline__ void lcg_scatter(const typename Fmt<FMT>::iraw_t &iv, const int4 &vv, int32_t pc,
                                            int32_t p0, int32_t p1, int32_t mask, double c,
                                            double magic, long long magic_bits,
                                            unsigned long long *__restrict__ acc)
{
    const uint32_t len = (uint32_t)(p1 - p0);          // pc+q in [p0, p1) as one unsigned compare
    const uint32_t rel = (uint32_t)(pc - p0);
    const int32_t magic_hi = (int32_t)(magic_bits >> 32);     // the low word of 1.5 * 2^k is zero
#pragma unroll
    for (int q = 0; q < Fmt<FMT>::EPL; q++) {
        // The arithmetic is done for all lanes, outside the branch, so that the entries of a
        // chunk overlap; lanes outside the run only sit out the atomic (LDS atomic throughput
        // is what this kernel runs out of next to HBM, so they must not issue one).
        const bool ok = rel + (uint32_t)q < len;
        const int32_t li = entry_pos<FMT>(iv, q, mask);
        const double t = fma(c, (double)entry_val<FMT>(vv, q), magic);
        const uint32_t lo = (uint32_t)__double2loint(t);
        uint32_t hi = (uint32_t)(__double2hiint(t) - magic_hi);
        asm volatile("" : "+v"(hi));          // pins the arithmetic here, subtraction in the high word only
        if (ok) atomicAdd(&acc[li], ((unsigned long long)hi << 32) | lo);
    }
}

// Persistent: workgroup b sits on XCD b%8 and is the (b/8)-th of `cpx` workgroups there; XCD x owns the
// contiguous slice range [x*per, (x+1)*per) and its workgroups work on neighbouring slices at any
// moment (same mapping as the SP pass).  While a slice's rows stream, the x values of its epilogue and
// the row offsets of the workgroup's next slice are already on their way in registers.
//
// XDENSE = false: x is the window row written last (x = c_t, Algorithm 1 line 8 as printed).  Then
// x/lambda is one more multiple of a stored row, out = -sum_r (coef_r - [r = that row]/lambda) c_r,
// and no dense x is read at all.
// The number of filled rows and the row written last come from the step state ("after": the
// step has been counted by the time this kernel runs).  With an empty window (efcp_apply before
// the first step) no row streams and the epilogue writes x/lambda.
// UPDATE = true: `out` holds the parameters and receives the optimizer step with decoupled
// weight decay, theta <- decay*theta - lr*(x/lambda - sum) (Algorithm 1 line 9), instead of
// the preconditioned vector.
template <int FMT, bool XDENSE, bool UPDATE, int GW>
__global__ __launch_bounds__(1024) void k_lcg(const float *__restrict__ x, float *__restrict__ out,
                                              int64_t d, int32_t m, const StepState *__restrict__ step,
                                              int64_t row_stride,
                                              int32_t slice, int32_t nsl, int32_t cpx,
                                              const uint8_t *__restrict__ ring,
                                              const int32_t *__restrict__ offT,
                                              const double *__restrict__ coef,
                                              const uint32_t *__restrict__ rowmax,
                                              uint32_t *__restrict__ status, double inv_lambda,
                                              double decay, double lr)
{
    const StepView sv = step_view(step, m, kAfter);
    const int32_t n_filled = sv.n_filled, x_row = sv.slot;
    const int32_t r_last = max(n_filled, 1) - 1;      // rows past the end repeat this one
    constexpr int EPL = Fmt<FMT>::EPL, kChunk = GW * EPL, kBatch = Fmt<FMT>::kBatch;
    constexpr int kRowGroups = 1024 / GW;                // rows the workgroup works on at once
    extern __shared__ __align__(16) unsigned char smem[];
    // `slice` coordinates (a multiple of 64, at most kCandBlock) are live; the LDS layout is that
    // of the widest slice
    unsigned long long *acc = reinterpret_cast<unsigned long long *>(smem);   // [kCandBlock]
    double *cf = reinterpret_cast<double *>(acc + kCandBlock);                // [1024]
    int32_t *offs = reinterpret_cast<int32_t *>(cf + kMaxM);                  // [2 buffers][2][1024]
    __shared__ double wsum[16];

    const int tid = threadIdx.x;
    const int grp = tid / GW, gl = tid % GW;
    const int32_t per = (nsl + 7) >> 3;
    const int32_t xcd = blockIdx.x & 7, cu = blockIdx.x >> 3;
    const SliceList sl(xcd * per, min(nsl, (xcd + 1) * per), cu, cpx);
    const int32_t mask = kCandBlock - 1;
    if (sl.count == 0) return;                // uniform: this workgroup has no slice
    int32_t it = 0;
    int32_t s = sl.at(0);
    const int32_t trow = min(tid, m - 1);     // row whose offsets this thread fetches

    for (int32_t i = tid; i < kCandBlock; i += 1024) acc[i] = 0ull;
    double cabs = 0.0;
    {
        offs[tid] = offT[(int64_t)s * m + trow];
        offs[kMaxM + tid] = offT[(int64_t)(s + 1) * m + trow];
        double c = tid < n_filled ? coef[tid] : 0.0;
        if (!XDENSE && tid == x_row) c -= inv_lambda;
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
    const double magic = ldexp(1.5, ex + 2);          // 1.5 * 2^52 * unit, unit = 2^(ex-50)
    const long long magic_bits = __double_as_longlong(magic);

    // Batches: two register sets used alternately (no copies between them): while one batch
    // is scattered, the loads of the group's next batch are in flight.
    const int32_t *off0 = offs, *off1 = offs + kMaxM;             // offsets of the current slice
    auto first = [&](LcgBatch<FMT> &b) {
        b.r = grp;
        const int32_t rc = min(b.r, r_last);
        b.p0 = off0[rc]; b.p1 = off1[rc]; b.c = cf[rc];
        b.pcs = b.p0 & ~(EPL - 1);
    };
    auto advance = [&](const LcgBatch<FMT> &a, LcgBatch<FMT> &b) {   // b = the batch after a
        const int32_t cont = a.pcs + kBatch * kChunk;
        const bool same = cont < a.p1;
        b.r = same ? a.r : a.r + kRowGroups;
        const int32_t rc = min(b.r, r_last);                      // past the end: repeat of the last row
        const int32_t q0 = off0[rc], q1 = off1[rc];
        b.p0 = same ? a.p0 : q0;
        b.p1 = same ? a.p1 : q1;
        b.c = cf[rc];
        b.pcs = same ? cont : (q0 & ~(EPL - 1));
    };
    auto load = [&](LcgBatch<FMT> &b) {
        const int32_t rc = min(b.r, r_last);
        const uint8_t *row =
            ring + (uint64_t)(uint32_t)rc * (uint32_t)row_stride * (uint64_t)Fmt<FMT>::kEntryBytes;
#pragma unroll
        for (int q = 0; q < kBatch; q++) {
            // always load (from the row start when the chunk lies past the run)
            const int32_t pc = b.pcs + gl * EPL + q * kChunk;
            const uint32_t pcl = pc < b.p1 ? (uint32_t)pc : 0u;
            load_group<FMT>(row, pcl, b.iv[q], b.vv[q]);
        }
    };

    LcgBatch<FMT> ba, bb;
    first(ba);
    load(ba);                                 // first batch of the first slice
    int buf = 0;
    // One slice.  FULL: all its coordinates exist, so x and out move as 16-byte accesses, the
    // loads unconditional (past a narrow slice's end the last four coordinates are read again and
    // the result is not stored), and the compiler can keep exact counts of the loads in flight.
    // The ragged last slice of the vector (at most one, and the last one of its workgroup) takes
    // the guarded path.
    auto do_slice = [&](auto full_tag) {
        constexpr bool FULL = decltype(full_tag)::value;
        const int64_t base64 = (int64_t)s * slice;
        const int32_t len = FULL ? slice : (int32_t)(d - base64);
        const int32_t snx = it + 1 < sl.count ? sl.at(it + 1) : s;     // this workgroup's next slice
        auto consume = [&](const LcgBatch<FMT> &b) {
            const int32_t hi = b.r < n_filled ? b.p1 : b.p0;       // rows past the end: an empty run
#pragma unroll
            for (int q = 0; q < kBatch; q++)
                lcg_scatter<FMT>(b.iv[q], b.vv[q], b.pcs + gl * EPL + q * kChunk, b.p0, hi, mask, b.c, magic,
                                 magic_bits, acc);
        };

        // on their way while the rows stream: x of this slice (for the epilogue) and the row
        // offsets of this workgroup's next slice
        float4 xr[4];
        if (FULL && XDENSE) {
#pragma unroll
            for (int u = 0; u < 4; u++)
                xr[u] = load_stream_f4(x + base64 + min(tid * 4 + u * 4096, slice - 4));
        }
        const int32_t o0 = offT[(int64_t)snx * m + trow];
        const int32_t o1 = offT[(int64_t)(snx + 1) * m + trow];
        int32_t *offn = offs + (buf ^ 1) * 2 * kMaxM;

        // Two batches per trip and no way out in the middle: a batch past the last row is an
        // empty run read from the last row again.  (With an exit between the two halves the
        // compiler sees a path on which the batch just requested is never waited for before its
        // registers are written again, and answers with a wait for everything at the top of
        // every trip: then the next batch is only requested once the current one has arrived.
        // Without it the waits count: a batch is scattered piece by piece as it arrives while
        // the next one stays in flight.  k_lcg 1.347 -> 1.331 ms at d = 110M.)
        while (__any(ba.r < n_filled)) {
            advance(ba, bb);
            load(bb);
            __builtin_amdgcn_sched_barrier(0);    // request first, then wait: nothing of consume() moves up
            consume(ba);
            advance(bb, ba);
            load(ba);
            __builtin_amdgcn_sched_barrier(0);
            consume(bb);
        }
        offn[tid] = o0;             // offsets of the next slice into the other LDS buffer
        offn[kMaxM + tid] = o1;
        float4 th[4];               // parameters of this slice: requested before the barrier
        if (FULL && UPDATE) {
#pragma unroll
            for (int u = 0; u < 4; u++)
                th[u] = load_stream_f4(out + base64 + min(tid * 4 + u * 4096, slice - 4));
        }
        __syncthreads();            // all rows of this slice are in the accumulators; offn visible

        off0 = offn;
        off1 = offn + kMaxM;
        buf ^= 1;
        // first batch of the next slice: in flight during the epilogue (after the last slice
        // this re-reads the current one: unconditional, so the waits below can leave it in flight)
        first(ba);
        load(ba);

        // out = x/lambda - sum (or the parameter update); accumulators back to zero for the next slice
        auto result = [&](float xj, float thj, unsigned long long a) {
            // a units of `unit`, exactly: magic + a*unit is the double whose bits are bits(magic) + a
            // (the sum stays inside magic's binade), and subtracting magic from it is exact
            const double sum = __longlong_as_double((long long)a + magic_bits) - magic;
            const double y = XDENSE ? (double)xj * inv_lambda - sum : -sum;
            return UPDATE ? (float)((double)thj * decay - lr * y) : (float)y;
        };
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const int32_t i = tid * 4 + u * 4096;
            float o[4];
            if (FULL) {
                const float xv[4] = {XDENSE ? xr[u].x : 0.f, XDENSE ? xr[u].y : 0.f, XDENSE ? xr[u].z : 0.f,
                                     XDENSE ? xr[u].w : 0.f};
                const float tv[4] = {UPDATE ? th[u].x : 0.f, UPDATE ? th[u].y : 0.f, UPDATE ? th[u].z : 0.f,
                                     UPDATE ? th[u].w : 0.f};
#pragma unroll
                for (int q = 0; q < 4; q++) o[q] = result(xv[q], tv[q], acc[i + q]);
                if (i < slice)                // whole 16-byte pieces: the slice is a multiple of 4
                    store_stream_f4(out + base64 + i, make_float4(o[0], o[1], o[2], o[3]));
            } else {
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    if (i + q < len) {
                        const float xj = XDENSE ? x[base64 + i + q] : 0.f;
                        const float tj = UPDATE ? out[base64 + i + q] : 0.f;
                        out[base64 + i + q] = result(xj, tj, acc[i + q]);
                    }
                }
            }
#pragma unroll
            for (int q = 0; q < 4; q++) acc[i + q] = 0ull;
        }
        __syncthreads();            // accumulators are zero before the next slice scatters
    };

    const int32_t n_full = (int32_t)(d / slice);                  // slices with all coordinates
    // the ragged slice, if this workgroup has it, is the last of its list
    const int32_t n_mine_full = sl.count - (sl.at(sl.count - 1) >= n_full ? 1 : 0);
    for (; it < n_mine_full; it++) {
        s = sl.at(it);
        do_slice(std::true_type{});
    }
    if (it < sl.count) {                                          // uniform
        s = sl.at(it);
        do_slice(std::false_type{});
    }
}

namespace {

template <int FMT, bool XDENSE, bool UPDATE, int GW>
void launch_lcg_gw(const Geometry &g, const DevicePtrs &p, const float *x, float *out, double lambda,
                   const LcgMode &md, hipStream_t stream)
{
    hipLaunchKernelGGL((k_lcg<FMT, XDENSE, UPDATE, GW>), dim3(g.sp_grid), dim3(1024), g.lds_lcg, stream, x, out,
                       g.d, g.m, p.step, g.row_stride, g.slice, g.n_slices, g.sp_grid / 8,
                       p.ring, p.offT,
                       p.coef, p.rowmax, p.status, 1.0 / lambda, md.decay, md.lr);
}

template <int FMT, bool XDENSE, bool UPDATE>
void launch_lcg_as(const Geometry &g, const DevicePtrs &p, const float *x, float *out, double lambda,
                   const LcgMode &md, hipStream_t stream)
{
    if (g.row_lanes == 4) launch_lcg_gw<FMT, XDENSE, UPDATE, 4>(g, p, x, out, lambda, md, stream);
    else launch_lcg_gw<FMT, XDENSE, UPDATE, 16>(g, p, x, out, lambda, md, stream);
}

template <int FMT>
void launch_lcg_fmt(const Geometry &g, const DevicePtrs &p, const float *x, float *out, double lambda,
                    const LcgMode &md, hipStream_t stream)
{
    const bool dense = !md.x_is_newest_row;
    if (dense && !md.update) launch_lcg_as<FMT, true, false>(g, p, x, out, lambda, md, stream);
    else if (dense) launch_lcg_as<FMT, true, true>(g, p, x, out, lambda, md, stream);
    else if (!md.update) launch_lcg_as<FMT, false, false>(g, p, x, out, lambda, md, stream);
    else launch_lcg_as<FMT, false, true>(g, p, x, out, lambda, md, stream);
}

template <int FMT, bool XDENSE, bool UPDATE>
hipError_t set_lds_lcg(const Geometry &g)
{
    hipError_t rc = hipFuncSetAttribute(reinterpret_cast<const void *>(k_lcg<FMT, XDENSE, UPDATE, 16>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)g.lds_lcg);
    if (rc == hipSuccess)
        rc = hipFuncSetAttribute(reinterpret_cast<const void *>(k_lcg<FMT, XDENSE, UPDATE, 4>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)g.lds_lcg);
    return rc;
}

template <int FMT>
hipError_t set_lds_lcg_fmt(const Geometry &g)
{
    hipError_t rc = set_lds_lcg<FMT, true, false>(g);
    if (rc == hipSuccess) rc = set_lds_lcg<FMT, true, true>(g);
    if (rc == hipSuccess) rc = set_lds_lcg<FMT, false, false>(g);
    if (rc == hipSuccess) rc = set_lds_lcg<FMT, false, true>(g);
    return rc;
}

}  // namespace

// `out` receives x/lambda - sum_r coef_r c_r, or (md.update) is the parameter vector updated in
// place.  md.x_is_newest_row: x is the window row written last and the pointer x is not read.
hipError_t launch_lcg(const Geometry &g, const DevicePtrs &p, const float *x, float *out, double lambda,
                      const LcgMode &md, hipStream_t stream)
{
    if (g.fmt == kFmtBf16) launch_lcg_fmt<kFmtBf16>(g, p, x, out, lambda, md, stream);
    else launch_lcg_fmt<kFmtF32>(g, p, x, out, lambda, md, stream);
    return hipGetLastError();
}

hipError_t configure_lcg(const Geometry &g)
{
    hipError_t rc = set_lds_lcg_fmt<kFmtF32>(g);
    if (rc == hipSuccess) rc = set_lds_lcg_fmt<kFmtBf16>(g);
    return rc;
}

}  // namespace efcp
