// blocktopk.hip -- error feedback and Top-k applied in blocks (Algorithm 1 lines 5-7 with the
// selection rule of Section "Sparsity Pattern"): every block of 16,384 consecutive coordinates
// keeps exactly kb entries, its kb largest |a_j| (ties -> lower index); a ragged last block of
// len coordinates keeps ceil(kb*len/16384).
//
// The block is the d-slice the SP and LCG kernels stage in LDS, so a selected index is a
// position inside one slice and the slice offsets of a row are simply s*kb.  One workgroup owns
// one block from load to store: a = e + g stays in registers (16 values per thread), an exact
// three-digit radix select (11 + 10 + 10 key bits) runs on LDS histograms, and an ordered
// compaction writes the kb entries and e = a - c.  HBM traffic is the minimum: g and e read once,
// e written once, the row written once; nothing is re-read and nothing crosses workgroups.
#include "efcp_internal.h"

namespace efcp {

namespace {

constexpr int kBlk = kCandBlock;         // coordinates per block == slice width
constexpr int kBlkThreads = 1024;
constexpr int kPerThread = kBlk / kBlkThreads;   // 16 = 4 groups of 4 consecutive coordinates

// Among the keys counted in hist[NB], find the bin that holds the kr-th largest one.
// Thread t looks at the bins NB-1-(t*PER+j): thread 0 owns the highest bins, so an exclusive
// prefix sum over threads counts the keys in higher bins.  res[0] = bin, res[1] = keys above
// it, res[2] = keys counted in total.  Every thread calls; ends with a barrier.
template <int NB>
__device__ __forceinline__ void pick_bin(const uint32_t *hist, uint32_t kr, uint32_t *tmp, uint32_t *res)
{
    constexpr int PER = NB / kBlkThreads;
    uint32_t c[PER], tot = 0;
#pragma unroll
    for (int j = 0; j < PER; j++) {
        c[j] = hist[NB - 1 - ((int)threadIdx.x * PER + j)];
        tot += c[j];
    }
    uint32_t total;
    uint32_t above = block_excl_scan_u32(tot, tmp, &total);
#pragma unroll
    for (int j = 0; j < PER; j++) {
        if (above < kr && kr <= above + c[j]) {
            res[0] = (uint32_t)(NB - 1 - ((int)threadIdx.x * PER + j));
            res[1] = above;
        }
        above += c[j];
    }
    if (threadIdx.x == 0) res[2] = total;
    __syncthreads();
}

}  // namespace

template <int FMT>
__global__ __launch_bounds__(kBlkThreads, 8) void k_block_topk(
    const float *__restrict__ g, float *__restrict__ e, int64_t d, int32_t m,
    const StepState *__restrict__ step, int64_t row_stride, int64_t k, int32_t kb, int32_t nsl,
    uint8_t *__restrict__ ring, int32_t *__restrict__ offT, uint32_t *__restrict__ blk_max, uint32_t *__restrict__ blk_tlo)
{
    const int32_t slot = step_view(step, m, kBefore).slot;           // the slot this step writes
    __shared__ uint32_t hist[kBins1];
    __shared__ uint32_t tmp[40];
    __shared__ uint32_t res[4];
    __shared__ uint32_t wtot[64], wbase[64];
    __shared__ uint32_t wmax[16];

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int32_t s = blockIdx.x;
    const int64_t base64 = (int64_t)s << 14;
    const int32_t len = (int32_t)((d - base64) < (int64_t)kBlk ? (d - base64) : (int64_t)kBlk);
    const bool full = len == kBlk;                                   // uniform
    const uint32_t keep = full ? (uint32_t)kb : (uint32_t)(((int64_t)kb * len + kBlk - 1) >> 14);

    // a = e + g, one fp32 rounding per element; coordinates past d act as +0 (they sit at the
    // highest indices of the block, so the tie rule never prefers them to a real coordinate)
    float a[kPerThread];
    if (full) {
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const int64_t at = base64 + u * 4096 + tid * 4;
            const float4 gv = load_stream_f4(g + at);
            const float4 ev = load_stream_f4(e + at);
            a[u * 4 + 0] = ev.x + gv.x;
            a[u * 4 + 1] = ev.y + gv.y;
            a[u * 4 + 2] = ev.z + gv.z;
            a[u * 4 + 3] = ev.w + gv.w;
        }
    } else {
#pragma unroll
        for (int u = 0; u < 4; u++)
#pragma unroll
            for (int c = 0; c < 4; c++) {
                const int32_t i = u * 4096 + tid * 4 + c;
                a[u * 4 + c] = i < len ? e[base64 + i] + g[base64 + i] : 0.0f;
            }
    }

    // largest key of the block (for the scale of the LCG sums)
    uint32_t mx = 0;
#pragma unroll
    for (int i = 0; i < kPerThread; i++) mx = max(mx, mag_key(a[i]));
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = max(mx, (uint32_t)__shfl_xor((int)mx, o, 64));
    if (lane == 0) wmax[wv] = mx;

    // ---- digit 1: key bits 30..20.  Only keys from two bins below this block's previous
    // threshold are counted (the threshold moves little from step to step); when they turn out
    // to be fewer than `keep`, everything is counted.  The result is the same either way.
    uint32_t tlo = blk_tlo[s];
    for (;;) {
        hist[tid] = 0u;
        hist[tid + 1024] = 0u;
        __syncthreads();
#pragma unroll
        for (int i = 0; i < kPerThread; i++) {
            const uint32_t key = mag_key(a[i]);
            if (key >= tlo) atomicAdd(&hist[key >> 20], 1u);
        }
        __syncthreads();
        pick_bin<kBins1>(hist, keep, tmp, res);
        if (res[2] >= keep) break;               // uniform; always true once tlo == 0
        tlo = 0u;
        __syncthreads();                         // res is rewritten by the next round
    }
    const uint32_t bin1 = res[0];
    uint32_t kr = keep - res[1];
    if (tid == 0) {
        blk_tlo[s] = (bin1 >= 2u ? bin1 - 2u : 0u) << 20;
        uint32_t bm = 0;
#pragma unroll
        for (int i = 0; i < 16; i++) bm = max(bm, wmax[i]);
        blk_max[s] = bm;
        offT[(int64_t)s * m + slot] = s * kb;
        if (s == nsl - 1) offT[(int64_t)nsl * m + slot] = (int32_t)k;
    }

    // ---- digit 2: bits 19..10 of the keys in bin1
    hist[tid] = 0u;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kPerThread; i++) {
        const uint32_t key = mag_key(a[i]);
        if ((key >> 20) == bin1) atomicAdd(&hist[(key >> 10) & 1023u], 1u);
    }
    __syncthreads();
    pick_bin<kBins2>(hist, kr, tmp, res);
    const uint32_t pre2 = (bin1 << 10) | res[0];
    kr -= res[1];
    __syncthreads();

    // ---- digit 3: bits 9..0
    hist[tid] = 0u;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kPerThread; i++) {
        const uint32_t key = mag_key(a[i]);
        if ((key >> 10) == pre2) atomicAdd(&hist[key & 1023u], 1u);
    }
    __syncthreads();
    pick_bin<kBins2>(hist, kr, tmp, res);
    const uint32_t tau = (pre2 << 10) | res[0];
    const uint32_t quota = kr - res[1];          // keys == tau to keep, lowest indices first

    // ---- ordered compaction.  Index order inside the block is (group u, thread, c).  Per group
    // the number of keys > tau (low half) and == tau (high half) before each thread: wave scan,
    // then one 64-entry scan over (u, wave).  Both counts stay below 2^15, so the halves never mix.
    uint32_t packed[4], incl[4];
#pragma unroll
    for (int u = 0; u < 4; u++) {
        uint32_t p = 0;
#pragma unroll
        for (int c = 0; c < 4; c++) {
            const uint32_t key = mag_key(a[u * 4 + c]);
            p += (key > tau ? 1u : 0u) + (key == tau ? 0x10000u : 0u);
        }
        packed[u] = p;
        incl[u] = wave_incl_scan_u32(p);
        if (lane == 63) wtot[u * 16 + wv] = incl[u];
    }
    __syncthreads();
    if (wv == 0) {
        const uint32_t v = wtot[lane];
        wbase[lane] = wave_incl_scan_u32(v) - v;
    }
    __syncthreads();

    uint8_t *row = ring + (int64_t)slot * row_stride * Fmt<FMT>::kEntryBytes;
    const uint32_t run_first = (uint32_t)s * (uint32_t)kb;           // this block's entries start here
#pragma unroll
    for (int u = 0; u < 4; u++) {
        uint32_t before = wbase[u * 16 + wv] + incl[u] - packed[u];
        float ev[4];
#pragma unroll
        for (int c = 0; c < 4; c++) {
            const float av = a[u * 4 + c];
            const uint32_t key = mag_key(av);
            const uint32_t gtb = before & 0xffffu, eqb = before >> 16;
            const bool gt = key > tau, eq = key == tau;
            const bool sel = gt || (eq && eqb < quota);
            const int32_t i = u * 4096 + tid * 4 + c;
            float rest = av;
            if (sel) {
                const uint32_t pos = run_first + gtb + min(eqb, quota);
                *entry_idx_ptr<FMT>(row, pos) = (uint16_t)i;       // position inside the slice
                if constexpr (FMT == kFmtF32) {
                    *entry_val_ptr<FMT>(row, pos) = av;
                    rest = av - av;                              // a - c: +0 for every finite a
                } else {
                    const uint32_t hb = bf16_bits(av);
                    *entry_val_ptr<FMT>(row, pos) = (uint16_t)hb;
                    rest = av - __uint_as_float(hb << 16);       // e keeps the rounding remainder
                }
            }
            ev[c] = rest;
            before += (gt ? 1u : 0u) + (eq ? 0x10000u : 0u);
        }
        if (full) {
            store_stream_f4(e + base64 + u * 4096 + tid * 4, make_float4(ev[0], ev[1], ev[2], ev[3]));
        } else {
#pragma unroll
            for (int c = 0; c < 4; c++) {
                const int32_t i = u * 4096 + tid * 4 + c;
                if (i < len) e[base64 + i] = ev[c];
            }
        }
    }
}

// rowmax[slot] = upper edge of the 2^20-key bin that holds the largest |a_j| of the step: an upper
// bound of every stored magnitude of the new row, bfloat16 rounding included.
__global__ __launch_bounds__(1024) void k_block_finish(const uint32_t *__restrict__ blk_max, int32_t nsl,
                                                       uint32_t *__restrict__ rowmax, int32_t m,
                                                       const StepState *__restrict__ step,
                                                       SelState *__restrict__ sel)
{
    __shared__ uint32_t wmax[16];
    uint32_t mx = 0;
    for (int32_t i = threadIdx.x; i < nsl; i += 1024) mx = max(mx, blk_max[i]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = max(mx, (uint32_t)__shfl_xor((int)mx, o, 64));
    if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t bm = 0;
#pragma unroll
        for (int i = 0; i < 16; i++) bm = max(bm, wmax[i]);
        const uint32_t edge = ((bm >> 20) + 1u) << 20;
        rowmax[step_view(step, m, kBefore).slot] = edge < 0x7f7fffffu ? edge : 0x7f7fffffu;
        sel->tau = 0u;                          // no single threshold exists in this mode
        sel->quota = 0u;
    }
}

hipError_t launch_block_topk(const Geometry &g, const DevicePtrs &p, const float *grad, hipStream_t stream)
{
    if (g.fmt == kFmtBf16)
        hipLaunchKernelGGL(k_block_topk<kFmtBf16>, dim3(g.n_slices), dim3(kBlkThreads), 0, stream, grad, p.e,
                           g.d, g.m, p.step, g.row_stride, g.k, g.kb, g.n_slices,
                           p.ring, p.offT,
                           p.blk_max, p.blk_tlo);
    else
        hipLaunchKernelGGL(k_block_topk<kFmtF32>, dim3(g.n_slices), dim3(kBlkThreads), 0, stream, grad, p.e,
                           g.d, g.m, p.step, g.row_stride, g.k, g.kb, g.n_slices,
                           p.ring, p.offT,
                           p.blk_max, p.blk_tlo);
    hipLaunchKernelGGL(k_block_finish, dim3(1), dim3(1024), 0, stream, p.blk_max, g.n_slices,
                       p.rowmax, g.m, p.step, p.sel);
    return hipGetLastError();
}

}  // namespace efcp
