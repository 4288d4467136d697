// select.hip -- error feedback and exact Top-k of one step (Algorithm 1,
// lines 5-7, with Compress = Top-k by magnitude, ties to the lower index).
//
// The magnitude of a float is ordered by the integer key = bits & 0x7fffffff.
// A three-digit radix select (11 + 10 + 10 bits, most significant first)
// finds the key tau of the k-th largest magnitude with LDS histograms merged
// by integer atomics (order independent, hence deterministic).  The selected
// set is {key > tau} plus the first `quota` elements with key == tau in index
// order.  An ordered compaction (per-block counts -> exclusive scan ->
// ballot-free wave prefix sums) writes the row with ascending indices and
// zeroes the selected entries of the error buffer.
//
// All kernels are bound by HBM traffic; none uses floating-point arithmetic
// beyond the one fp32 addition a = e + g per element.
#include "efcp_internal.h"

namespace efcp {

// ------------------------------------------------------------------
// a = e + g (written over e) and histogram of key bits 30..20.
__global__ __launch_bounds__(kSelThreads) void k_ef_hist(const float *__restrict__ g,
                                                         float *__restrict__ e, int64_t d,
                                                         uint32_t *__restrict__ hist)
{
    __shared__ uint32_t lh[kBins1];
    for (int i = threadIdx.x; i < kBins1; i += kSelThreads) lh[i] = 0;
    __syncthreads();

    const int64_t n4 = d >> 2;
    const float4 *g4 = reinterpret_cast<const float4 *>(g);
    float4 *e4 = reinterpret_cast<float4 *>(e);
    const int64_t stride = (int64_t)gridDim.x * kSelThreads;
    for (int64_t i = (int64_t)blockIdx.x * kSelThreads + threadIdx.x; i < n4; i += stride) {
        const float4 gv = g4[i];
        const float4 ev = e4[i];
        float4 a;
        a.x = ev.x + gv.x;
        a.y = ev.y + gv.y;
        a.z = ev.z + gv.z;
        a.w = ev.w + gv.w;
        e4[i] = a;
        atomicAdd(&lh[mag_key(a.x) >> 20], 1u);
        atomicAdd(&lh[mag_key(a.y) >> 20], 1u);
        atomicAdd(&lh[mag_key(a.z) >> 20], 1u);
        atomicAdd(&lh[mag_key(a.w) >> 20], 1u);
    }
    if (blockIdx.x == 0 && threadIdx.x < (d & 3)) {
        const int64_t j = (n4 << 2) + threadIdx.x;
        const float a = e[j] + g[j];
        e[j] = a;
        atomicAdd(&lh[mag_key(a) >> 20], 1u);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kBins1; i += kSelThreads) {
        const uint32_t c = lh[i];
        if (c) atomicAdd(&hist[i], c);
    }
}

// ------------------------------------------------------------------
// Histogram of the next 10-bit digit over the elements whose higher key bits
// equal the prefix found so far.  shift_hi: bits to drop to compare with the
// prefix; shift_lo: position of the digit.
__global__ __launch_bounds__(kSelThreads) void k_hist_digit(const float *__restrict__ a, int64_t d,
                                                            const SelState *__restrict__ sel,
                                                            uint32_t *__restrict__ hist,
                                                            int shift_hi, int shift_lo)
{
    __shared__ uint32_t lh[kBins2];
    for (int i = threadIdx.x; i < kBins2; i += kSelThreads) lh[i] = 0;
    __syncthreads();
    const uint32_t prefix = sel->prefix;

    const int64_t n4 = d >> 2;
    const float4 *a4 = reinterpret_cast<const float4 *>(a);
    const int64_t stride = (int64_t)gridDim.x * kSelThreads;
    for (int64_t i = (int64_t)blockIdx.x * kSelThreads + threadIdx.x; i < n4; i += stride) {
        const float4 v = a4[i];
        const uint32_t k0 = mag_key(v.x), k1 = mag_key(v.y), k2 = mag_key(v.z), k3 = mag_key(v.w);
        if ((k0 >> shift_hi) == prefix) atomicAdd(&lh[(k0 >> shift_lo) & (kBins2 - 1)], 1u);
        if ((k1 >> shift_hi) == prefix) atomicAdd(&lh[(k1 >> shift_lo) & (kBins2 - 1)], 1u);
        if ((k2 >> shift_hi) == prefix) atomicAdd(&lh[(k2 >> shift_lo) & (kBins2 - 1)], 1u);
        if ((k3 >> shift_hi) == prefix) atomicAdd(&lh[(k3 >> shift_lo) & (kBins2 - 1)], 1u);
    }
    if (blockIdx.x == 0 && threadIdx.x < (d & 3)) {
        const uint32_t kk = mag_key(a[(n4 << 2) + threadIdx.x]);
        if ((kk >> shift_hi) == prefix) atomicAdd(&lh[(kk >> shift_lo) & (kBins2 - 1)], 1u);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kBins2; i += kSelThreads) {
        const uint32_t c = lh[i];
        if (c) atomicAdd(&hist[i], c);
    }
}

// ------------------------------------------------------------------
// One workgroup: locate the digit in which the kr-th largest remaining key
// falls, update the select state, and clear the histogram for the next step.
// pass 0: 2048 bins (bits 30..20); pass 1, 2: 1024 bins.
template <int NB>
__global__ __launch_bounds__(1024) void k_pick_digit(uint32_t *__restrict__ hist,
                                                     SelState *__restrict__ sel, int pass,
                                                     uint32_t k)
{
    __shared__ uint32_t tmp[33];
    constexpr int PER = NB / 1024;
    const uint32_t kr = (pass == 0) ? k : sel->kr;
    const uint32_t prefix = (pass == 0) ? 0u : sel->prefix;

    // Walk the bins from the largest digit down: rb = NB-1-bin.
    uint32_t c[PER];
    uint32_t local = 0;
#pragma unroll
    for (int i = 0; i < PER; i++) {
        const int bin = NB - 1 - (threadIdx.x * PER + i);
        c[i] = hist[bin];
        hist[bin] = 0;
        local += c[i];
    }
    uint32_t total;
    uint32_t above = block_excl_scan_u32(local, tmp, &total);   // count in larger digits
#pragma unroll
    for (int i = 0; i < PER; i++) {
        const int bin = NB - 1 - (threadIdx.x * PER + i);
        if (above < kr && kr <= above + c[i]) {
            const uint32_t np = (pass == 0) ? (uint32_t)bin : ((prefix << 10) | (uint32_t)bin);
            sel->prefix = np;
            sel->kr = kr - above;
            if (pass == 2) {
                sel->tau = np;
                sel->quota = kr - above;
                sel->n_gt = k - (kr - above);
            }
        }
        above += c[i];
    }
}

// ------------------------------------------------------------------
// Block b owns coordinates [b*kSelChunk, (b+1)*kSelChunk).  Wave w of the
// block owns 1024 consecutive coordinates, read as 4 float4 per lane:
// element (it, lane, c) is coordinate wave_base + it*256 + lane*4 + c.  The
// count kernel and the compaction kernel use this same order.
struct Chunk16 {
    float v[4][4];
    uint32_t gt, eq;      // 16-bit masks, bit it*4+c
};

__device__ __forceinline__ void load_chunk(const float *__restrict__ a, int64_t d, int64_t wave_base,
                                           uint32_t tau, Chunk16 &ch)
{
    const int lane = threadIdx.x & 63;
    ch.gt = 0;
    ch.eq = 0;
#pragma unroll
    for (int it = 0; it < 4; it++) {
        const int64_t j0 = wave_base + it * 256 + lane * 4;
        if (j0 + 3 < d) {
            const float4 t = *reinterpret_cast<const float4 *>(a + j0);
            ch.v[it][0] = t.x; ch.v[it][1] = t.y; ch.v[it][2] = t.z; ch.v[it][3] = t.w;
        } else {
#pragma unroll
            for (int c = 0; c < 4; c++) ch.v[it][c] = (j0 + c < d) ? a[j0 + c] : 0.0f;
        }
#pragma unroll
        for (int c = 0; c < 4; c++) {
            if (j0 + c < d) {
                const uint32_t key = mag_key(ch.v[it][c]);
                if (key > tau) ch.gt |= 1u << (it * 4 + c);
                else if (key == tau) ch.eq |= 1u << (it * 4 + c);
            }
        }
    }
}

__global__ __launch_bounds__(kSelThreads) void k_count(const float *__restrict__ a, int64_t d,
                                                       const SelState *__restrict__ sel,
                                                       uint32_t *__restrict__ cnt_gt,
                                                       uint32_t *__restrict__ cnt_eq)
{
    __shared__ uint32_t s_gt[4], s_eq[4];
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const uint32_t tau = sel->tau;
    Chunk16 ch;
    load_chunk(a, d, (int64_t)blockIdx.x * kSelChunk + w * 1024, tau, ch);
    const uint32_t g = wave_sum_u32(__popc(ch.gt));
    const uint32_t q = wave_sum_u32(__popc(ch.eq));
    if (lane == 0) { s_gt[w] = g; s_eq[w] = q; }
    __syncthreads();
    if (threadIdx.x == 0) {
        cnt_gt[blockIdx.x] = s_gt[0] + s_gt[1] + s_gt[2] + s_gt[3];
        cnt_eq[blockIdx.x] = s_eq[0] + s_eq[1] + s_eq[2] + s_eq[3];
    }
}

// ------------------------------------------------------------------
// One workgroup: exclusive scans over the compaction blocks.
//   eq_before[b] = number of keys == tau in blocks before b
//   sel_off[b]   = number of selected entries in blocks before b
// and the slice offsets of the new row: offT[s][slot] = sel_off[first block of slice s].
__global__ __launch_bounds__(1024) void k_scan_blocks(const uint32_t *__restrict__ cnt_gt,
                                                      const uint32_t *__restrict__ cnt_eq,
                                                      uint32_t *__restrict__ sel_off,
                                                      uint32_t *__restrict__ eq_before,
                                                      SelState *__restrict__ sel, int32_t nb,
                                                      int32_t blocks_per_slice, int32_t n_slices,
                                                      int32_t m, int32_t slot,
                                                      int32_t *__restrict__ offT,
                                                      uint32_t *__restrict__ rowmax, uint32_t k,
                                                      uint32_t *__restrict__ status)
{
    __shared__ uint32_t tmp[33];
    const int32_t per = (nb + 1023) / 1024;
    const int32_t b0 = min(nb, (int32_t)threadIdx.x * per), b1 = min(nb, b0 + per);
    const uint32_t quota = sel->quota;

    uint32_t local = 0;
    for (int32_t b = b0; b < b1; b++) local += cnt_eq[b];
    uint32_t total;
    uint32_t run = block_excl_scan_u32(local, tmp, &total);
    uint32_t lsel = 0;
    for (int32_t b = b0; b < b1; b++) {
        const uint32_t ce = cnt_eq[b];
        eq_before[b] = run;
        const uint32_t take = run >= quota ? 0u : min(quota - run, ce);
        const uint32_t sc = cnt_gt[b] + take;
        sel_off[b] = sc;            // count for now, offset after the second scan
        lsel += sc;
        run += ce;
    }
    run = block_excl_scan_u32(lsel, tmp, &total);
    for (int32_t b = b0; b < b1; b++) {
        const uint32_t sc = sel_off[b];
        sel_off[b] = run;
        if (b % blocks_per_slice == 0) offT[(int64_t)(b / blocks_per_slice) * m + slot] = (int32_t)run;
        run += sc;
    }
    if (threadIdx.x == 0) {
        offT[(int64_t)n_slices * m + slot] = (int32_t)total;
        sel->total = total;
        rowmax[slot] = 0;
        if (total != k) atomicOr(status, kStatusCount);
    }
}

// ------------------------------------------------------------------
// Ordered compaction of the selected entries of block b into the ring row,
// and e = a - c: selected entries of the error buffer become +0.
__global__ __launch_bounds__(kSelThreads) void k_compact(float *__restrict__ e, int64_t d,
                                                         const SelState *__restrict__ sel,
                                                         const uint32_t *__restrict__ sel_off,
                                                         const uint32_t *__restrict__ eq_before,
                                                         int32_t *__restrict__ row_idx,
                                                         float *__restrict__ row_val,
                                                         uint32_t *__restrict__ rowmax_slot)
{
    __shared__ uint32_t s_eq[4], s_sel[4];
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const uint32_t tau = sel->tau, quota = sel->quota;
    const int64_t wave_base = (int64_t)blockIdx.x * kSelChunk + w * 1024;
    Chunk16 ch;
    load_chunk(e, d, wave_base, tau, ch);

    const uint32_t wave_eq = wave_sum_u32(__popc(ch.eq));
    if (lane == 0) s_eq[w] = wave_eq;
    __syncthreads();

    uint32_t selm = ch.gt;
    if (wave_eq != 0) {          // uniform over the wave
        uint32_t run = eq_before[blockIdx.x];
        for (int i = 0; i < w; i++) run += s_eq[i];
        if (run < quota) {       // uniform: some ties of this wave may still be taken
#pragma unroll
            for (int it = 0; it < 4; it++) {
                const uint32_t m4 = (ch.eq >> (it * 4)) & 15u;
                const uint32_t cnt = __popc(m4);
                const uint32_t incl = wave_incl_scan_u32(cnt);
                uint32_t rank = run + incl - cnt;
#pragma unroll
                for (int c = 0; c < 4; c++) {
                    if ((m4 >> c) & 1u) {
                        if (rank < quota) selm |= 1u << (it * 4 + c);
                        rank++;
                    }
                }
                run += __shfl(incl, 63, 64);
            }
        }
    }

    const uint32_t wave_sel = wave_sum_u32(__popc(selm));
    if (lane == 0) s_sel[w] = wave_sel;
    __syncthreads();
    if (wave_sel == 0) return;   // uniform over the wave; no barrier follows

    uint32_t run = sel_off[blockIdx.x];
    for (int i = 0; i < w; i++) run += s_sel[i];
    uint32_t kmax = 0;
#pragma unroll
    for (int it = 0; it < 4; it++) {
        const uint32_t m4 = (selm >> (it * 4)) & 15u;
        const uint32_t cnt = __popc(m4);
        const uint32_t incl = wave_incl_scan_u32(cnt);
        uint32_t pos = run + incl - cnt;
        const int64_t j0 = wave_base + it * 256 + lane * 4;
        if (m4) {
#pragma unroll
            for (int c = 0; c < 4; c++) {
                if ((m4 >> c) & 1u) {
                    row_idx[pos] = (int32_t)(j0 + c);
                    row_val[pos] = ch.v[it][c];
                    kmax = max(kmax, mag_key(ch.v[it][c]));
                    ch.v[it][c] = 0.0f;
                    pos++;
                }
            }
            if (j0 + 3 < d) {
                *reinterpret_cast<float4 *>(e + j0) =
                    make_float4(ch.v[it][0], ch.v[it][1], ch.v[it][2], ch.v[it][3]);
            } else {
#pragma unroll
                for (int c = 0; c < 4; c++)
                    if ((m4 >> c) & 1u) e[j0 + c] = 0.0f;
            }
        }
        run += __shfl(incl, 63, 64);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) kmax = max(kmax, (uint32_t)__shfl_xor(kmax, o, 64));
    if (lane == 0) atomicMax(rowmax_slot, kmax);
}

// ------------------------------------------------------------------

static int select_grid(int64_t d)
{
    const int64_t n4 = (d >> 2) + 1;
    const int64_t want = (n4 + kSelThreads - 1) / kSelThreads;
    return (int)(want < 2048 ? want : 2048);
}

hipError_t launch_ef_hist(const Geometry &g, const DevicePtrs &p, const float *grad, hipStream_t stream)
{
    hipLaunchKernelGGL(k_ef_hist, dim3(select_grid(g.d)), dim3(kSelThreads), 0, stream, grad, p.e, g.d,
                       p.hist1);
    return hipGetLastError();
}

hipError_t launch_select(const Geometry &g, const DevicePtrs &p, int32_t slot, hipStream_t stream)
{
    const int grid = select_grid(g.d);
    hipLaunchKernelGGL(k_pick_digit<kBins1>, dim3(1), dim3(1024), 0, stream, p.hist1, p.sel, 0,
                       (uint32_t)g.k);
    hipLaunchKernelGGL(k_hist_digit, dim3(grid), dim3(kSelThreads), 0, stream, p.e, g.d, p.sel, p.hist2,
                       20, 10);
    hipLaunchKernelGGL(k_pick_digit<kBins2>, dim3(1), dim3(1024), 0, stream, p.hist2, p.sel, 1,
                       (uint32_t)g.k);
    hipLaunchKernelGGL(k_hist_digit, dim3(grid), dim3(kSelThreads), 0, stream, p.e, g.d, p.sel, p.hist3,
                       10, 0);
    hipLaunchKernelGGL(k_pick_digit<kBins2>, dim3(1), dim3(1024), 0, stream, p.hist3, p.sel, 2,
                       (uint32_t)g.k);
    hipLaunchKernelGGL(k_count, dim3(g.n_sel_blocks), dim3(kSelThreads), 0, stream, p.e, g.d, p.sel,
                       p.cnt_gt, p.cnt_eq);
    hipLaunchKernelGGL(k_scan_blocks, dim3(1), dim3(1024), 0, stream, p.cnt_gt, p.cnt_eq, p.sel_off,
                       p.eq_before, p.sel, g.n_sel_blocks, g.slice / kSelChunk, g.n_slices, g.m, slot,
                       p.offT, p.rowmax, (uint32_t)g.k, p.status);
    return hipGetLastError();
}

hipError_t launch_compact(const Geometry &g, const DevicePtrs &p, int32_t slot, hipStream_t stream)
{
    hipLaunchKernelGGL(k_compact, dim3(g.n_sel_blocks), dim3(kSelThreads), 0, stream, p.e, g.d, p.sel,
                       p.sel_off, p.eq_before, p.ring_idx + (int64_t)slot * g.row_stride,
                       p.ring_val + (int64_t)slot * g.row_stride, p.rowmax + slot);
    return hipGetLastError();
}

}  // namespace efcp
