// sp.hip -- scalar products of every window row with the dense vector x and
// with the newest row: q_r = <c_r, x> and the Gram row S[slot][r] = <c_r, c_new>
// (Section "Scalar Products (SP)", Section "Sparse Scalar Products").
//
// Traversal is by d-slice, not by row: a workgroup stages x[slice] and the
// newest row scattered to dense in LDS (interleaved float2, one 8-byte LDS
// gather serves both products), then streams the index/value runs of all
// filled rows that fall in the slice.  x is read from HBM once and every
// gather is an LDS access.  A group of GW lanes (16; 4 where a row has only a
// few entries per slice, so that the workgroup works on 256 rows at once
// instead of 64) owns one row at a time and reads its run chunk by chunk (per
// lane four 16-bit positions and four fp32 or bfloat16 values), one batch of chunks being
// consumed while the next is in flight; products of two fp32 values are exact
// in fp64 and are accumulated in fp64.
//
// Workgroups are persistent: each walks a fixed list of slices and keeps one
// (q, Gram) accumulator per row in LDS, so the partial sums that reach memory
// are one per (workgroup, row); k_sp_reduce adds them in a fixed order.  The
// slice lists are static, which makes the sums independent of scheduling.
#include "efcp_internal.h"

#include <type_traits>

namespace efcp {

// One batch = up to kBatch chunks of one row's run in the slice: lane gl of the row's group
// reads entries [pc, pc+EPL), pc = pcs + EPL*gl + kChunk*c.  A run longer than a batch is
// continued by the next batch (same row, pcs advanced), so the row loop has a single shape
// and the number of loads in flight is always known.
template <int FMT>
struct RunBatch {
    typename Fmt<FMT>::iraw_t iv[Fmt<FMT>::kBatch];
    int4 vv[Fmt<FMT>::kBatch];
    int32_t r;          // row (may be >= n_filled: then nothing is valid)
    int32_t pcs;        // position of chunk 0, lane 0 (multiple of EPL)
    int32_t p0, p1;     // the row's run in this slice
};

template <int FMT>
__device__ __forceinline__ void sp_accumulate(const typename Fmt<FMT>::iraw_t &iv, const int4 &vv,
                                              int32_t pc, int32_t p0, int32_t p1, int32_t mask,
                                              const float2 *__restrict__ xc, double &aq, double &ag)
{
    // entry pc+c belongs to the run iff 0 <= pc+c-p0 < p1-p0 (one unsigned compare); an entry
    // outside gathers the pair of zeros kept behind the slice instead of being zeroed itself
    const uint32_t len = (uint32_t)(p1 - p0);
    const uint32_t rel = (uint32_t)(pc - p0);
#pragma unroll
    for (int c = 0; c < Fmt<FMT>::EPL; c++) {
        const bool ok = rel + (uint32_t)c < len;
        const int32_t li = ok ? entry_pos<FMT>(iv, c, mask) : mask + 1;
        const double v = (double)entry_val<FMT>(vv, c);
        const float2 t = xc[li];
        aq = fma(v, (double)t.x, aq);
        ag = fma(v, (double)t.y, ag);
    }
}

constexpr int kMaxSlicesPerWg = 512;     // ceil(2^31 / 16384 / 8 / 32); narrower slices: checked at creation

// What the staged pair (x_j, c_new_j) holds:
//   kXDense    x from memory, newest row scattered next to it      (step with x = gradient)
//   kXNewest   x IS the newest row: nothing dense is read, the scatter fills both halves,
//              and q equals the Gram row                          (step with x = c_t)
//   kXOnly     x from memory, no newest row: only q is meaningful  (apply on a fixed window)
enum : int { kXDense = 0, kXNewest = 1, kXOnly = 2 };

// Workgroup b sits on XCD b%8 (workgroups are dealt to the 8 XCDs round-robin)
// and is the (b/8)-th of `cpx` workgroups there.  XCD x owns the contiguous
// slice range [x*per, (x+1)*per); at any time its workgroups work on
// neighbouring slices (see SliceList), so a cache line straddling two runs of
// a row is wanted by two CUs of the same L2 at about the same time.
//
// While the rows of one slice stream, everything the next slice needs first is
// already on its way in registers: its x values, its row offsets and the
// newest row's entries that fall into it.  The switch between slices is then
// three barriers and LDS traffic, with the first batch of ring loads of the
// new slice issued before the last two.
template <int FMT, int XM, int GW>
__global__ __launch_bounds__(1024) void k_sp(const float *__restrict__ x, int64_t d, int32_t m,
                                             const StepState *__restrict__ step, int64_t row_stride,
                                             int64_t k, int32_t slice, int32_t nsl, int32_t cpx,
                                             const uint8_t *__restrict__ ring,
                                             const int32_t *__restrict__ offT,
                                             double2 *__restrict__ partial)
{
    // a step's SP pass runs before the step is counted, efcp_apply's on the window as it stands
    const StepView sv = step_view(step, m, XM == kXOnly ? kAfter : kBefore);
    const int32_t n_filled = sv.n_filled, slot = sv.slot;
    const int32_t r_last = max(n_filled, 1) - 1;      // rows past the end repeat this one (row 0 of an empty window)
    using idx_t = typename Fmt<FMT>::idx_t;
    using val_t = typename Fmt<FMT>::val_t;
    constexpr int EPL = Fmt<FMT>::EPL, kChunk = GW * EPL, kBatch = Fmt<FMT>::kBatch;
    constexpr int kRowGroups = 1024 / GW;                // rows the workgroup works on at once
    extern __shared__ __align__(16) unsigned char smem[];
    // `slice` coordinates (a multiple of 64, at most kCandBlock) are live; the LDS layout is that
    // of the widest slice
    float2 *xc = reinterpret_cast<float2 *>(smem);       // [kCandBlock]: (x_j, c_new_j); [kCandBlock] = (0, 0)
    double2 *racc = reinterpret_cast<double2 *>(xc + kCandBlock + 2);   // [1024] per-row sums
    int32_t *off0 = reinterpret_cast<int32_t *>(racc + kMaxM);     // [1024]
    int32_t *off1 = off0 + kMaxM;                                  // [1024]
    int32_t *np0 = off1 + kMaxM;                                   // [kMaxSlicesPerWg] newest row's run
    int32_t *np1 = np0 + kMaxSlicesPerWg;                          //   in each slice of this workgroup

    const int tid = threadIdx.x;
    const int grp = tid / GW, gl = tid % GW;
    const int32_t per = (nsl + 7) >> 3;
    const int32_t xcd = blockIdx.x & 7, cu = blockIdx.x >> 3;
    const SliceList sl(xcd * per, min(nsl, (xcd + 1) * per), cu, cpx);
    const int32_t mask = kCandBlock - 1;
    const int32_t trow = min(tid, m - 1);
    constexpr int64_t kEntryBytes = Fmt<FMT>::kEntryBytes;
    uint8_t *nrow = const_cast<uint8_t *>(ring) + (int64_t)slot * row_stride * kEntryBytes;   // newest row (read only)
    auto nidx = [&](int32_t p) { return *entry_idx_ptr<FMT>(nrow, (uint32_t)p); };
    auto nval = [&](int32_t p) { return *entry_val_ptr<FMT>(nrow, (uint32_t)p); };
    const int32_t klast = (int32_t)(k - 1);

    racc[tid] = make_double2(0.0, 0.0);
    if (tid == 0) xc[kCandBlock] = make_float2(0.0f, 0.0f);        // what entries outside a run gather
    if (sl.count == 0) {                      // uniform: no slice for this workgroup
        if (tid < m) partial[(int64_t)blockIdx.x * m + tid] = make_double2(0.0, 0.0);
        return;
    }
    if (XM != kXOnly) {
        for (int32_t i = tid; i < sl.count; i += 1024) {
            const int32_t si = sl.at(i);
            np0[i] = offT[(int64_t)si * m + slot];
            np1[i] = offT[(int64_t)(si + 1) * m + slot];
        }
    }

    // state carried from one slice to the next (prefetched while the previous one streams)
    float4 xr[4];
    int32_t o0, o1;
    idx_t di = 0;
    val_t dv = 0;
    int32_t it = 0;                           // index of the current slice in this workgroup's list
    int32_t s = sl.at(0);

    auto prefetch = [&](int32_t sp, int32_t ip, auto full_tag) {
        constexpr bool FULL = decltype(full_tag)::value;
        const int64_t b64 = (int64_t)sp * slice;
        if (XM == kXNewest) {
#pragma unroll
            for (int u = 0; u < 4; u++) xr[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        } else if (FULL) {
            // unconditional; past a narrow slice's end the last four coordinates are read again
            // into LDS positions that no entry of the slice points at
#pragma unroll
            for (int u = 0; u < 4; u++) xr[u] = load_stream_f4(x + b64 + min(tid * 4 + u * 4096, slice - 4));
        } else {
            const int32_t len = (int32_t)(d - b64);
#pragma unroll
            for (int u = 0; u < 4; u++) {
                const int32_t i = tid * 4 + u * 4096;
                xr[u].x = (i + 0 < len) ? x[b64 + i + 0] : 0.0f;
                xr[u].y = (i + 1 < len) ? x[b64 + i + 1] : 0.0f;
                xr[u].z = (i + 2 < len) ? x[b64 + i + 2] : 0.0f;
                xr[u].w = (i + 3 < len) ? x[b64 + i + 3] : 0.0f;
            }
        }
        o0 = offT[(int64_t)sp * m + trow];
        o1 = offT[(int64_t)(sp + 1) * m + trow];
        if (XM != kXOnly) {
            const int32_t p = min(np0[ip] + tid, klast);     // clamped: always a valid entry
            di = nidx(p);
            dv = nval(p);
        }
    };

    const int32_t n_full = (int32_t)(d / slice);                 // slices with all coordinates
    __syncthreads();                          // np0/np1 visible, racc zeroed
    if (s < n_full) prefetch(s, 0, std::true_type{}); else prefetch(s, 0, std::false_type{});

    RunBatch<FMT> ba, bb;
    auto first = [&](RunBatch<FMT> &b) {
        b.r = grp;
        const int32_t rc = min(b.r, r_last);
        b.p0 = off0[rc]; b.p1 = off1[rc];
        b.pcs = b.p0 & ~(EPL - 1);
    };
    auto advance = [&](const RunBatch<FMT> &a, RunBatch<FMT> &b) {   // b = the batch after a
        const int32_t cont = a.pcs + kBatch * kChunk;
        const bool same = cont < a.p1;
        b.r = same ? a.r : a.r + kRowGroups;
        const int32_t rc = min(b.r, r_last);                      // past the end: repeat of the last row
        const int32_t q0 = off0[rc], q1 = off1[rc];
        b.p0 = same ? a.p0 : q0;
        b.p1 = same ? a.p1 : q1;
        b.pcs = same ? cont : (q0 & ~(EPL - 1));
    };
    auto load = [&](RunBatch<FMT> &b) {
        const int32_t rc = min(b.r, r_last);
        const uint8_t *row = ring + (uint64_t)(uint32_t)rc * (uint32_t)row_stride * (uint64_t)kEntryBytes;
#pragma unroll
        for (int c = 0; c < kBatch; c++) {
            // always load (from the row start when the chunk lies past the run)
            const int32_t pc = b.pcs + gl * EPL + c * kChunk;
            const uint32_t pcl = pc < b.p1 ? (uint32_t)pc : 0u;
            load_group<FMT>(row, pcl, b.iv[c], b.vv[c]);
        }
    };

    for (; it < sl.count; it++) {
        s = sl.at(it);
        // ---- switch to slice s: everything comes from registers ----
        __syncthreads();            // previous slice fully consumed
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const int32_t i = tid * 4 + u * 4096;
            xc[i + 0] = make_float2(xr[u].x, 0.0f);
            xc[i + 1] = make_float2(xr[u].y, 0.0f);
            xc[i + 2] = make_float2(xr[u].z, 0.0f);
            xc[i + 3] = make_float2(xr[u].w, 0.0f);
        }
        off0[tid] = o0;
        off1[tid] = o1;
        const int32_t q0 = XM != kXOnly ? np0[it] : 0, q1 = XM != kXOnly ? np1[it] : 0;
        __syncthreads();            // x and offsets of slice s in LDS
        first(ba);
        load(ba);                   // first ring batch in flight during the scatter below
        if (XM != kXOnly) {
            auto put = [&](idx_t i, val_t v) {                     // newest row next to x (or as x)
                const float f = stored_val(v);
                if (XM == kXNewest) xc[stored_pos(i, mask)] = make_float2(f, f);
                else xc[stored_pos(i, mask)].y = f;
            };
            if (q0 + tid < q1) put(di, dv);
            for (int32_t p = q0 + 1024 + tid; p < q1; p += 1024)   // runs longer than 1024 entries
                put(nidx(p), nval(p));
        }
        __syncthreads();

        // ---- prefetch for the next slice of this workgroup ----
        if (it + 1 < sl.count) {    // uniform
            const int32_t sn = sl.at(it + 1);
            if (sn < n_full) prefetch(sn, it + 1, std::true_type{});
            else prefetch(sn, it + 1, std::false_type{});
        }

        // ---- stream the rows: two register batches used alternately ----
        auto consume = [&](const RunBatch<FMT> &b) {
            double aq = 0.0, ag = 0.0;
            const int32_t hi = b.r < n_filled ? b.p1 : b.p0;       // rows past the end: an empty run
#pragma unroll
            for (int c = 0; c < kBatch; c++)
                sp_accumulate<FMT>(b.iv[c], b.vv[c], b.pcs + gl * EPL + c * kChunk, b.p0, hi, mask, xc, aq, ag);
            const double sum = row_sum2_f64<GW>(aq, ag);           // lower half of the group: q part, upper: Gram part
            if ((gl & (GW / 2 - 1)) == 0 && b.r < n_filled)        // row r belongs to this group only: no race
                reinterpret_cast<double *>(racc)[2 * b.r + gl / (GW / 2)] += sum;
        };
        while (__any(ba.r < n_filled)) {
            advance(ba, bb);
            load(bb);
            consume(ba);
            if (!__any(bb.r < n_filled)) break;
            advance(bb, ba);
            load(ba);
            consume(bb);
        }
    }
    __syncthreads();
    if (tid < m)
        partial[(int64_t)blockIdx.x * m + tid] = tid < n_filled ? racc[tid] : make_double2(0.0, 0.0);
}

// sq[r] = sum over workgroups of partial[b][r], in a fixed order: block bx
// owns 64 rows; thread (bl, rl) adds workgroups bl, bl+16, ...; the 16
// partial sums are then added in order.  Unfilled rows give exactly 0.
// commit != 0: the "before" part of a step ends here (every kernel that needed t_done = t - 1 has
// finished: they precede this one on the stream, and where the eviction update runs on the side
// stream it has been joined), so one thread counts the step: t_done = t, and with the global Top-k the new row
// becomes the one whose entries are still to be taken out of e.
__global__ __launch_bounds__(1024) void k_sp_reduce(const double2 *__restrict__ partial, int32_t m,
                                                    int32_t nwg, double2 *__restrict__ sq,
                                                    StepState *__restrict__ step, int32_t commit,
                                                    int32_t pend_rows)
{
    if (commit && blockIdx.x == 0 && threadIdx.x == 0) {
        const long long td = step->t_done;
        step->pend_slot = pend_rows ? (int32_t)(td % m) : -1;
        step->t_done = td + 1;
    }
    __shared__ double2 sh[16][64];
    const int rl = threadIdx.x & 63, bl = threadIdx.x >> 6;
    const int32_t r = blockIdx.x * 64 + rl;
    double ax = 0.0, ay = 0.0;
    if (r < m) {
        // at most kMaxWgs / 16 = 16 partial sums per thread, all requested at once
        double2 t[kMaxWgs / 16];
#pragma unroll
        for (int u = 0; u < kMaxWgs / 16; u++) t[u] = partial[(int64_t)min(bl + 16 * u, nwg - 1) * m + r];
#pragma unroll
        for (int u = 0; u < kMaxWgs / 16; u++) {
            const bool in = bl + 16 * u < nwg;
            ax += in ? t[u].x : 0.0;
            ay += in ? t[u].y : 0.0;
        }
    }
    sh[bl][rl] = make_double2(ax, ay);
    __syncthreads();
    if (bl == 0 && r < m) {
        double sx = 0.0, sy = 0.0;
#pragma unroll
        for (int i = 0; i < 16; i++) {
            sx += sh[i][rl].x;
            sy += sh[i][rl].y;
        }
        sq[r] = make_double2(sx, sy);
    }
}

namespace {

template <int FMT, int XM, int GW>
void launch_sp_gw(const Geometry &g, const DevicePtrs &p, const float *x, hipStream_t stream)
{
    hipLaunchKernelGGL((k_sp<FMT, XM, GW>), dim3(g.sp_grid), dim3(1024), g.lds_sp, stream, x, g.d, g.m, p.step,
                       g.row_stride, g.k, g.slice, g.n_slices, g.sp_grid / 8,
                       p.ring, p.offT, p.partial);
}

template <int FMT, int XM>
void launch_sp_as(const Geometry &g, const DevicePtrs &p, const float *x, hipStream_t stream)
{
    if (g.row_lanes == 4) launch_sp_gw<FMT, XM, 4>(g, p, x, stream);
    else launch_sp_gw<FMT, XM, 16>(g, p, x, stream);
}

template <int FMT>
void launch_sp_fmt(const Geometry &g, const DevicePtrs &p, const float *x, int32_t xmode, hipStream_t stream)
{
    if (xmode == kXNewest) launch_sp_as<FMT, kXNewest>(g, p, x, stream);
    else if (xmode == kXOnly) launch_sp_as<FMT, kXOnly>(g, p, x, stream);
    else launch_sp_as<FMT, kXDense>(g, p, x, stream);
}

template <int FMT, int XM>
hipError_t set_lds_sp(const Geometry &g)
{
    hipError_t rc = hipFuncSetAttribute(reinterpret_cast<const void *>(k_sp<FMT, XM, 16>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)g.lds_sp);
    if (rc == hipSuccess)
        rc = hipFuncSetAttribute(reinterpret_cast<const void *>(k_sp<FMT, XM, 4>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)g.lds_sp);
    return rc;
}

}  // namespace

// x_source: 0 = dense x plus the newest row, 1 = the newest row is x (x unused),
// 2 = dense x only, window as it stands (the Gram half of the result is meaningless).
hipError_t launch_sp(const Geometry &g, const DevicePtrs &p, const float *x, int32_t x_source,
                     hipStream_t stream)
{
    if (g.fmt == kFmtBf16) launch_sp_fmt<kFmtBf16>(g, p, x, x_source, stream);
    else launch_sp_fmt<kFmtF32>(g, p, x, x_source, stream);
    return hipGetLastError();
}

hipError_t launch_sp_reduce(const Geometry &g, const DevicePtrs &p, bool commit, hipStream_t stream)
{
    hipLaunchKernelGGL(k_sp_reduce, dim3((g.m + 63) / 64), dim3(1024), 0, stream, p.partial, g.m,
                       g.sp_grid, p.sq, p.step, commit ? 1 : 0, g.kb ? 0 : 1);
    return hipGetLastError();
}

hipError_t configure_sp(const Geometry &g)
{
    hipError_t rc = set_lds_sp<kFmtF32, kXDense>(g);
    if (rc == hipSuccess) rc = set_lds_sp<kFmtF32, kXNewest>(g);
    if (rc == hipSuccess) rc = set_lds_sp<kFmtF32, kXOnly>(g);
    if (rc == hipSuccess) rc = set_lds_sp<kFmtBf16, kXDense>(g);
    if (rc == hipSuccess) rc = set_lds_sp<kFmtBf16, kXNewest>(g);
    if (rc == hipSuccess) rc = set_lds_sp<kFmtBf16, kXOnly>(g);
    return rc;
}

}  // namespace efcp
