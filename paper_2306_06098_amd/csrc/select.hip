// select.hip -- error feedback and exact Top-k of one step (Algorithm 1,
// lines 5-7, with Compress = Top-k by magnitude, ties to the lower index).
//
// The magnitude of a float is ordered by the integer key = bits & 0x7fffffff.
// A three-digit radix select (11 + 10 + 10 bits, most significant first)
// finds the key tau of the k-th largest magnitude; the selected set is
// {key > tau} plus the first `quota` elements with key == tau in index order.
//
// Only the first pass touches the whole vector.  While it forms a = e + g and
// the histogram of the first digit, it also copies every element whose key is
// at least t_lo -- the lower edge of the bin below the previous step's threshold bin --
// to a candidate list, in index order, one segment per block (a d-slice, at
// most 16,384 coordinates).  All later passes (two digit histograms, per-block counts and
// the ordered compaction into the ring) read the candidates only: a few
// percent of d.  e = a - c is not finished by this step: clearing k scattered
// entries costs a partial HBM write each, so the buffer keeps a, and the NEXT
// step's first pass, which rewrites e anyway, drops the entries of the row
// inserted last (a bitmap in LDS, one bit per coordinate of the block).  Host code
// that reads e in between applies the same rule.  The first-digit histogram
// is exact, so it tells whether the threshold bin lies at or above t_lo; if it
// does not (the threshold fell into a bin at least two below the previous one), the
// later passes of that step read the accumulator itself instead of the
// candidate lists.  The result is exact either way; the prediction only saves
// traffic.
//
// Histograms are merged with integer atomics (order independent), candidates
// and rows are written at positions computed by prefix sums, so every output
// is deterministic.
#include "efcp_internal.h"
#include "evict.h"

namespace efcp {

// Streaming layout of a d-sized pass: a block owns one d-slice (`blk`
// consecutive coordinates, a multiple of 64 and at most 16,384), walked in
// chunks of 8,192 by 512 threads (measured against 256 and 1024 threads per
// block: 0.252 / 0.250 / 0.291 ms at d = 110M); inside a chunk wave w
// owns 1,024 consecutive coordinates and lane l holds, for it = 0..3, the four
// coordinates wave_first + it*256 + l*4 + (0..3), loaded as one 16-byte load.
// All four loads of a lane are issued before any is used.

// Appends this wave's flagged elements of one chunk to the block's candidate
// segment, in index order.  `flags`: bit it*4+c.  `base`: entries of the
// segment already used by earlier chunks and by lower waves of this chunk.
__device__ __forceinline__ void emit_candidates(const float (&v)[4][4], uint32_t flags, int64_t wave_base,
                                                uint32_t base, int32_t *__restrict__ seg_idx,
                                                float *__restrict__ seg_val)
{
    uint32_t run = base;
#pragma unroll
    for (int it = 0; it < 4; it++) {
        const uint32_t m4 = (flags >> (it * 4)) & 15u;
        const uint32_t cnt = __popc(m4);
        const uint32_t incl = wave_incl_scan_u32(cnt);
        uint32_t pos = run + incl - cnt;
        if (m4) {
#pragma unroll
            for (int c = 0; c < 4; c++) {
                if ((m4 >> c) & 1u) {
                    seg_idx[pos] = (int32_t)(wave_base + it * 256 + c);
                    seg_val[pos] = v[it][c];
                    pos++;
                }
            }
        }
        run += __shfl(incl, 63, 64);
    }
}

// a = e + g (written over e), histogram of key bits 30..20, candidates.
// (Launch bounds: at least 6 waves per SIMD, i.e. at most 80 vector registers, so that three
// blocks share a CU: with two, a vector of 768 slices met 512 places and ran a round and a half.
// Requesting the first chunk before the pending row is looked up was tried: the registers it
// holds across that stretch spill at this bound, and the pass got a fifth slower.)
// PEND (first pass only; 1: fp32 window, 2: bfloat16 window): if the step state names a pending
// slot, `e` still holds the previous step's accumulator; the entries of the row inserted then (the
// run of this block given by two entries of its offset column) count as +0, or as the rounding
// remainder a - bf16(a) when the window keeps bfloat16 values.
constexpr int kEfThreads = 512;                  // threads of a first-pass block
constexpr int kEfWaves = kEfThreads / 64;
constexpr int kEfChunk = kEfWaves * 1024;        // coordinates the block streams at a time

template <int PEND>
__global__ __launch_bounds__(kEfThreads, 6) void k_ef_hist(const float *__restrict__ g,
                                                         float *__restrict__ e, int64_t d,
                                                         uint32_t *__restrict__ hist,
                                                         const SelState *__restrict__ sel,
                                                         int32_t *__restrict__ cand_idx,
                                                         float *__restrict__ cand_val,
                                                         uint32_t *__restrict__ cand_cnt,
                                                         const uint8_t *__restrict__ ring,
                                                         int64_t row_bytes,
                                                         const int32_t *__restrict__ offT, int32_t m,
                                                         int32_t blk, const StepState *__restrict__ step)
{
    __shared__ uint32_t lh[kBins1];
    __shared__ uint32_t s_cnt[2][kEfWaves];
    __shared__ uint32_t pend[PEND ? kCandBlock / 32 : 1];       // one bit per coordinate of the block
    const uint32_t t_lo = sel->t_lo;
    for (int i = threadIdx.x; i < kBins1; i += kEfThreads) lh[i] = 0;
    if (PEND) {
        for (int i = threadIdx.x; i < kCandBlock / 32; i += kEfThreads) pend[i] = 0;
        __syncthreads();
        const int32_t ps = step->pend_slot;               // uniform
        if (ps >= 0) {
            const uint8_t *pend_row = ring + (int64_t)ps * row_bytes;
            const int32_t *pend_off = offT + ps;
            const int32_t p0 = pend_off[(int64_t)blockIdx.x * m], p1 = pend_off[(int64_t)(blockIdx.x + 1) * m];
            for (int32_t p = p0 + (int32_t)threadIdx.x; p < p1; p += kEfThreads) {
                constexpr int PF = PEND == 2 ? kFmtBf16 : kFmtF32;
                const uint32_t pos = *entry_idx_ptr<PF>(const_cast<uint8_t *>(pend_row), (uint32_t)p);
                atomicOr(&pend[pos >> 5], 1u << (pos & 31u));
            }
        }
    }
    __syncthreads();
    // value of e at a coordinate whose pending bit is set
    // a - c as written (Algorithm 1, line 7): +0 for every finite a, NaN for an infinite one
    auto settled = [](float a) {
        if (PEND == 2) return a - __uint_as_float(bf16_bits(a) << 16);
        return a - a;
    };
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int64_t block_first = (int64_t)blockIdx.x * blk;
    const int64_t block_end = block_first + blk < d ? block_first + blk : d;
    int32_t *seg_idx = cand_idx + block_first;
    float *seg_val = cand_val + block_first;
    uint32_t used = 0;                                    // entries of the segment written so far

    for (int cch = 0; cch * kEfChunk < blk; cch++) {
        const int64_t wave_first = block_first + cch * kEfChunk + w * 1024;
        const int64_t wave_base = wave_first + lane * 4;
        // Lanes hold whole 16-byte pieces wherever the wave's part of the block ends on a multiple
        // of 4 coordinates (always, except in the last block of a vector of ragged length): of a
        // lane's four pieces, 256 coordinates apart, the first nit exist.
        const int64_t rem = block_end - wave_first;        // scalar
        float a[4][4];
        uint32_t inmask;                                   // bit it*4+c: the coordinate exists
        auto vector_pieces = [&](const int nit) {
            float4 ev[4], gv[4];
#pragma unroll
            for (int it = 0; it < 4; it++) {
                ev[it] = make_float4(0.f, 0.f, 0.f, 0.f);
                gv[it] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (it < nit) {
                    ev[it] = load_stream_f4(e + wave_base + it * 256);
                    gv[it] = load_stream_f4(g + wave_base + it * 256);
                }
            }
#pragma unroll
            for (int it = 0; it < 4; it++) {
                if (PEND && it < nit) {
                    // the four coordinates of this load share one word of the bitmap
                    const uint32_t q = (uint32_t)(cch * kEfChunk + w * 1024 + it * 256 + lane * 4);
                    const uint32_t bits4 = (pend[q >> 5] >> (q & 31u)) & 15u;
                    if (bits4 & 1u) ev[it].x = settled(ev[it].x);
                    if (bits4 & 2u) ev[it].y = settled(ev[it].y);
                    if (bits4 & 4u) ev[it].z = settled(ev[it].z);
                    if (bits4 & 8u) ev[it].w = settled(ev[it].w);
                }
                a[it][0] = ev[it].x + gv[it].x;
                a[it][1] = ev[it].y + gv[it].y;
                a[it][2] = ev[it].z + gv[it].z;
                a[it][3] = ev[it].w + gv[it].w;
                if (it < nit)
                    store_stream_f4(e + wave_base + it * 256,
                                    make_float4(a[it][0], a[it][1], a[it][2], a[it][3]));
            }
        };
        if (rem >= 1024) {
            vector_pieces(4);
            inmask = 0xffffu;
        } else if (rem <= 0 || (rem & 3) == 0) {
            const int left = (int)rem - lane * 4;              // coordinates from this lane's first piece on
            const int nit = left <= 0 ? 0 : (left + 255) >> 8;
            vector_pieces(nit);
            inmask = (1u << (4 * nit)) - 1u;
        } else {
            inmask = 0;
#pragma unroll
            for (int it = 0; it < 4; it++) {
#pragma unroll
                for (int c = 0; c < 4; c++) {
                    const int64_t j = wave_base + it * 256 + c;
                    float t = 0.0f;
                    if (j < block_end) {
                        float ej = e[j];
                        if (PEND) {
                            const uint32_t q = (uint32_t)(j - block_first);
                            if ((pend[q >> 5] >> (q & 31u)) & 1u) ej = settled(ej);
                        }
                        t = ej + g[j];
                        e[j] = t;
                        inmask |= 1u << (it * 4 + c);
                    }
                    a[it][c] = t;
                }
            }
        }
        uint32_t flags = 0;
#pragma unroll
        for (int it = 0; it < 4; it++) {
#pragma unroll
            for (int c = 0; c < 4; c++) {
                const uint32_t key = mag_key(a[it][c]);
                if ((inmask >> (it * 4 + c)) & 1u) {
                    atomicAdd(&lh[key >> 20], 1u);
                    if (key >= t_lo) flags |= 1u << (it * 4 + c);
                }
            }
        }
        const uint32_t wave_cnt = wave_sum_u32(__popc(flags));
        if (lane == 0) s_cnt[cch & 1][w] = wave_cnt;
        __syncthreads();
        uint32_t base = used, total = 0;
#pragma unroll
        for (int i = 0; i < kEfWaves; i++) {
            const uint32_t c = s_cnt[cch & 1][i];
            if (i < w) base += c;
            total += c;
        }
        if (wave_cnt) emit_candidates(a, flags, wave_base, base, seg_idx, seg_val);
        used += total;
    }
    if (threadIdx.x == 0) cand_cnt[blockIdx.x] = used;
    __syncthreads();
    // Most keys fall into a few dozen bins, which every block adds to at about the same time:
    // the adds to one address queue up, so the blocks are spread over kHist1Copies histograms.
    uint32_t *mine = hist + (blockIdx.x % kHist1Copies) * kBins1;
    for (int i = threadIdx.x; i < kBins1; i += kEfThreads) {
        const uint32_t c = lh[i];
        if (c) atomicAdd(&mine[i], c);
    }
}

// ------------------------------------------------------------------
// The passes after the first one.  Each is ONE kernel of 1024-thread workgroups that starts by
// settling the previous digit itself: every workgroup adds up the kHist1Copies histograms that
// the pass before left in memory and locates the bin of the kr-th largest remaining key (a few
// KB of loads and one block-wide scan, the same in every workgroup, so all agree), workgroup 0
// records the outcome in the select state, and the body goes on with it.  A histogram is
// cleared by the pass after the one that read it.  Compared with one-workgroup kernels between
// the passes this halves the number of dependent launches of a step (four instead of nine).
//
//   k_cand_hist<1>   settles digit 1 (bits 30..20); histogram of digit 2 (bits 19..10)
//   k_cand_hist<2>   settles digit 2; histogram of digit 3 (bits 9..0); clears histogram 1
//   k_cand_count     settles digit 3 = the threshold tau and the tie quota; counts keys > tau
//                    and == tau per segment and per workgroup; clears histogram 2
//   k_cand_compact   prefix sums of those counts (workgroup totals, then the 16 segments of
//                    the workgroup), ordered compaction into the ring; clears histogram 3
//
// If the threshold bin turns out to lie below t_lo (the threshold fell by two bins or more in
// one step: a bin is an eighth of an octave), the candidate lists do not hold every key that matters.  The passes then read the
// accumulator itself (it is in `e`), a whole slice in place of its candidate segment: the
// result is the same, the step moves 16 more bytes per coordinate.

constexpr int kSegsPerBlock = 16;        // one wave per segment

// One segment as the passes see it: values in index order, and where each one sits.
struct Segment {
    const float *val;
    const int32_t *idx;      // coordinates, or nullptr: value i is coordinate first + i
    uint32_t cnt;
    int32_t first;           // first coordinate of the slice
};

__device__ __forceinline__ Segment segment_of(int32_t b, int32_t blk, int64_t d, uint32_t redo,
                                              const float *__restrict__ e,
                                              const float *__restrict__ cand_val,
                                              const int32_t *__restrict__ cand_idx,
                                              const uint32_t *__restrict__ cand_cnt)
{
    Segment sg;
    const int64_t first = (int64_t)b * blk;
    sg.first = (int32_t)first;
    if (redo) {
        sg.val = e + first;
        sg.idx = nullptr;
        sg.cnt = (uint32_t)(d - first < (int64_t)blk ? d - first : (int64_t)blk);
    } else {
        sg.val = cand_val + first;
        sg.idx = cand_idx + first;
        sg.cnt = cand_cnt[b];
    }
    return sg;
}

// Which of the NB bins of a digit holds the kr-th largest remaining key: the bins are walked
// from the largest digit down.  `hist`: kHist1Copies histograms of NB bins each.  All 1024
// threads call it and all get the result.  res: 3 words of LDS; tmp: 33 words of LDS.
//   bin      the digit
//   kr_rem   rank of the wanted key among the keys of that bin
//   top      the highest occupied bin
template <int NB>
__device__ __forceinline__ void settle_digit(const uint32_t *__restrict__ hist, uint32_t kr, uint32_t *tmp,
                                             uint32_t *res, uint32_t &bin_out, uint32_t &kr_rem,
                                             uint32_t &top)
{
    constexpr int PER = NB / 1024;
    if (threadIdx.x < 3) res[threadIdx.x] = 0;
    uint32_t c[PER];
    uint32_t local = 0;
#pragma unroll
    for (int i = 0; i < PER; i++) {
        const int bin = NB - 1 - (threadIdx.x * PER + i);
        uint32_t t = 0;
#pragma unroll
        for (int u = 0; u < kHist1Copies; u++) t += hist[u * NB + bin];
        c[i] = t;
        local += t;
    }
    uint32_t total;
    uint32_t above = block_excl_scan_u32(local, tmp, &total);     // count in larger digits; syncs
#pragma unroll
    for (int i = 0; i < PER; i++) {
        const int bin = NB - 1 - (threadIdx.x * PER + i);
        if (c[i]) atomicMax(&res[2], (uint32_t)bin);
        if (above < kr && kr <= above + c[i]) {
            res[0] = (uint32_t)bin;
            res[1] = kr - above;
        }
        above += c[i];
    }
    __syncthreads();
    bin_out = res[0];
    kr_rem = res[1];
    top = res[2];
    __syncthreads();
}

__device__ __forceinline__ void clear_histogram(uint32_t *__restrict__ hist, int words)
{
    for (int i = blockIdx.x * 1024 + threadIdx.x; i < words; i += gridDim.x * 1024) hist[i] = 0;
}

// The passes are a handful of dependent memory round trips long, so each one asks for
// everything it can before it knows anything: a wave requests the size and the first 512 values
// of its (first) candidate segment together with the histogram of the previous digit, and only
// then settles that digit.  The candidate buffer of a segment is as long as the slice (at least
// 256 entries), so a read clamped to the slice is in bounds whatever the segment holds; entries
// past its size are masked afterwards.  (The accumulator fallback cannot use the early read
// and starts over from `e`.)
struct FirstBatch {
    float v[8];
    uint32_t cnt;
};

__device__ __forceinline__ void request_first_batch(int32_t b, int32_t nb, int32_t blk,
                                                    const float *__restrict__ cand_val,
                                                    const uint32_t *__restrict__ cand_cnt, int lane,
                                                    FirstBatch &fb)
{
    const int32_t bc = min(b, nb - 1);
    fb.cnt = cand_cnt[bc];
    const float *seg = cand_val + (int64_t)bc * blk;
#pragma unroll
    for (int u = 0; u < 8; u++) fb.v[u] = seg[min(u * 64 + lane, blk - 1)];
    if (b >= nb) fb.cnt = 0;
}

// f(key, exists) for the entries [i_begin, cnt) of a segment, 512 at a time: eight loads per lane
// are issued before any is used (unconditional, clamped addresses).
template <class F>
__device__ __forceinline__ void for_each_key(const Segment &sg, int lane, uint32_t i_begin, F f)
{
    for (uint32_t i0 = i_begin; i0 < sg.cnt; i0 += 512) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; u++) v[u] = sg.val[min(i0 + u * 64 + lane, sg.cnt - 1)];
#pragma unroll
        for (int u = 0; u < 8; u++) f(mag_key(v[u]), i0 + u * 64 + lane < sg.cnt);
    }
}

// Segment b through f: the early read first if it is usable.
template <class F>
__device__ __forceinline__ void first_segment(int32_t b, int32_t blk, int64_t d, uint32_t redo,
                                              const float *__restrict__ e,
                                              const float *__restrict__ cand_val,
                                              const int32_t *__restrict__ cand_idx,
                                              const uint32_t *__restrict__ cand_cnt,
                                              const FirstBatch &fb, int lane, F f)
{
    if (redo) {
        for_each_key(segment_of(b, blk, d, 1u, e, cand_val, cand_idx, cand_cnt), lane, 0u, f);
        return;
    }
#pragma unroll
    for (int u = 0; u < 8; u++) f(mag_key(fb.v[u]), (uint32_t)(u * 64 + lane) < fb.cnt);
    Segment sg;
    sg.first = (int32_t)((int64_t)b * blk);
    sg.val = cand_val + (int64_t)b * blk;
    sg.idx = cand_idx + (int64_t)b * blk;
    sg.cnt = fb.cnt;
    for_each_key(sg, lane, 512u, f);
}

// LEVEL 1: digit 1 is settled from hist_prev (2048 bins) and the histogram of digit 2 is built;
// LEVEL 2: digit 2 is settled from hist_prev (1024 bins), histogram of digit 3; `hist_clear`
// (the histogram the previous pass read) is zeroed.
// `groups` workgroups (at most kHistGroups); a wave takes one segment at a time.  Every workgroup
// counts in its own 1024-bin histogram in LDS (device-scope atomics on a few hot addresses from
// thousands of waves serialise) and adds it once, at the end, into one of kHist1Copies
// histograms in memory.
// LEVEL 1 carries `n_evict` more workgroups in front of the `groups` that count: each deletes the
// oldest row from 16 columns of the inverse factor W of the coefficient step (evict.h) when the
// step replaces a row.  That work depends on nothing in this step and nothing here depends on
// it; it sits in this kernel because the kernels of the selection leave most of the machine
// idle, and as workgroups of a kernel of the stream it costs no second stream and no events.
template <int LEVEL>
__global__ __launch_bounds__(1024) void k_cand_hist(const float *__restrict__ e, int64_t d,
                                                    const float *__restrict__ cand_val,
                                                    const int32_t *__restrict__ cand_idx,
                                                    const uint32_t *__restrict__ cand_cnt, int32_t nb,
                                                    SelState *__restrict__ sel,
                                                    const uint32_t *__restrict__ hist_prev,
                                                    uint32_t *__restrict__ hist_out,
                                                    uint32_t *__restrict__ hist_clear, uint32_t k,
                                                    int32_t blk, int32_t groups,
                                                    uint32_t *__restrict__ rowmax, int32_t m,
                                                    const StepState *__restrict__ step, int32_t n_evict,
                                                    int32_t ldm, double *__restrict__ W)
{
    if (LEVEL == 1 && (int32_t)blockIdx.x < n_evict) {            // uniform per workgroup
        const StepView sv = step_view(step, m, kBefore);
        if (sv.evict) evict_block((int32_t)blockIdx.x, m, ldm, sv.slot, W);
        return;
    }
    const int32_t bid = (int32_t)blockIdx.x - (LEVEL == 1 ? n_evict : 0);    // among the workgroups that count
    __shared__ uint32_t lh[kBins2];
    __shared__ uint32_t tmp[33], res[3];
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    int32_t b = bid * kSegsPerBlock + w;
    FirstBatch fb;
    request_first_batch(b, nb, blk, cand_val, cand_cnt, lane, fb);
    lh[threadIdx.x] = 0;
    uint32_t prefix, redo;
    if (LEVEL == 1) {
        const uint32_t t_lo = sel->t_lo;
        uint32_t bin, kr1, top;
        settle_digit<kBins1>(hist_prev, k, tmp, res, bin, kr1, top);
        prefix = bin;
        // candidates hold every key >= t_lo: enough iff the threshold bin starts at or above t_lo
        redo = (bin << 20) < t_lo ? 1u : 0u;
        if (bid == 0 && threadIdx.x == 0) {
            sel->p1 = bin;
            sel->kr1 = kr1;
            sel->redo = redo;
            // every |a_j| of this step is below the upper edge of the highest occupied bin:
            // an upper bound on the largest stored magnitude, enough to scale the LCG sum
            const uint32_t edge = (top + 1u) << 20;
            rowmax[step_view(step, m, kBefore).slot] = edge < 0x7f7fffffu ? edge : 0x7f7fffffu;
        }
    } else {
        const uint32_t kr1 = sel->kr1, p1 = sel->p1;
        redo = sel->redo;
        uint32_t bin, kr2, top;
        settle_digit<kBins2>(hist_prev, kr1, tmp, res, bin, kr2, top);
        prefix = (p1 << 10) | bin;
        if (bid == 0 && threadIdx.x == 0) {
            sel->p2 = prefix;
            sel->kr2 = kr2;
        }
        clear_histogram(hist_clear, kHist1Copies * kBins1);
    }
    constexpr int shift_hi = LEVEL == 1 ? 20 : 10, shift_lo = LEVEL == 1 ? 10 : 0;
    auto count_key = [&](uint32_t kk, bool exists) {
        if (exists && (kk >> shift_hi) == prefix) atomicAdd(&lh[(kk >> shift_lo) & (kBins2 - 1)], 1u);
    };
    if (b < nb) {
        first_segment(b, blk, d, redo, e, cand_val, cand_idx, cand_cnt, fb, lane, count_key);
        for (b += groups * kSegsPerBlock; b < nb; b += groups * kSegsPerBlock)
            for_each_key(segment_of(b, blk, d, redo, e, cand_val, cand_idx, cand_cnt), lane, 0u, count_key);
    }
    __syncthreads();
    const uint32_t c = lh[threadIdx.x];
    if (c) atomicAdd(&hist_out[(bid % kHist1Copies) * kBins2 + threadIdx.x], c);
}

// ------------------------------------------------------------------
// Settles the last digit: tau, the tie quota, where the next step starts collecting candidates.
// Then, per segment, how many keys are > tau and == tau, and the same per workgroup (its 16
// segments), which is what the compaction's prefix sums start from.
__global__ __launch_bounds__(1024) void k_cand_count(const float *__restrict__ e, int64_t d,
                                                     const float *__restrict__ cand_val,
                                                     const int32_t *__restrict__ cand_idx,
                                                     const uint32_t *__restrict__ cand_cnt, int32_t nb,
                                                     SelState *__restrict__ sel,
                                                     const uint32_t *__restrict__ hist_prev,
                                                     uint32_t *__restrict__ hist_clear, uint32_t k,
                                                     uint32_t *__restrict__ cnt_gt,
                                                     uint32_t *__restrict__ cnt_eq,
                                                     uint32_t *__restrict__ blk_gt,
                                                     uint32_t *__restrict__ blk_eq, int32_t blk)
{
    __shared__ uint32_t tmp[33], res[3];
    __shared__ uint32_t s_g[kSegsPerBlock], s_q[kSegsPerBlock];
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int32_t b = blockIdx.x * kSegsPerBlock + w;
    FirstBatch fb;
    request_first_batch(b, nb, blk, cand_val, cand_cnt, lane, fb);
    const uint32_t kr2 = sel->kr2, p2 = sel->p2, redo = sel->redo;
    uint32_t bin, quota, top;
    settle_digit<kBins2>(hist_prev, kr2, tmp, res, bin, quota, top);
    const uint32_t tau = (p2 << 10) | bin;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        sel->tau = tau;
        sel->quota = quota;
        sel->n_gt = k - quota;
        // The next step collects from one bin below this threshold's bin.  (Two bins: a third more
        // candidates to write and to read four times; d = 340M: 9.06 -> 8.96 ms per step.  The
        // accumulator fallback then needs a threshold that falls by 9-19 % in one step.)
        const uint32_t tb = tau >> 20;
        sel->t_lo = (tb >= 1 ? tb - 1 : 0u) << 20;
    }
    clear_histogram(hist_clear, kHist1Copies * kBins2);

    uint32_t g = 0, q = 0;
    if (b < nb) {
        first_segment(b, blk, d, redo, e, cand_val, cand_idx, cand_cnt, fb, lane,
                      [&](uint32_t key, bool exists) {
                          g += exists && key > tau;
                          q += exists && key == tau;
                      });
        g = wave_sum_u32(g);
        q = wave_sum_u32(q);
        if (lane == 0) { cnt_gt[b] = g; cnt_eq[b] = q; }
    }
    if (lane == 0) { s_g[w] = g; s_q[w] = q; }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t tg = 0, tq = 0;
#pragma unroll
        for (int i = 0; i < kSegsPerBlock; i++) { tg += s_g[i]; tq += s_q[i]; }
        blk_gt[blockIdx.x] = tg;
        blk_eq[blockIdx.x] = tq;
    }
}

// ------------------------------------------------------------------
// Ordered compaction of the selected candidates of segment b into the ring row (16-bit
// positions inside the segment = slice; fp32 or bfloat16 values), one wave per segment,
// candidates already in index order.  Where a segment's entries go follows from the counts of
// the pass before: the ties taken among the first E keys == tau (in index order) are
// min(quota, E), so
//   entries before segment b = (keys > tau before b) + min(quota, keys == tau before b),
// with "before b" = the totals of the workgroups before this one plus the segments of this
// workgroup before b.  The error buffer is left as it is: see the top of this file.
template <int FMT>
__global__ __launch_bounds__(1024) void k_cand_compact(const float *__restrict__ e, int64_t d,
                                                       const float *__restrict__ cand_val,
                                                       const int32_t *__restrict__ cand_idx,
                                                       const uint32_t *__restrict__ cand_cnt,
                                                       int32_t nb, SelState *__restrict__ sel,
                                                       const uint32_t *__restrict__ cnt_gt,
                                                       const uint32_t *__restrict__ cnt_eq,
                                                       const uint32_t *__restrict__ blk_gt,
                                                       const uint32_t *__restrict__ blk_eq,
                                                       uint32_t *__restrict__ hist_clear,
                                                       uint8_t *__restrict__ ring, int64_t row_bytes,
                                                       int32_t blk, int32_t *__restrict__ offT,
                                                       int32_t m, const StepState *__restrict__ step,
                                                       uint32_t k, uint32_t *__restrict__ status)
{
    __shared__ uint32_t s_part[2][16];
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int32_t b0 = blockIdx.x * kSegsPerBlock, b = b0 + w;
    // everything this wave will need is requested first: the segment's size and its first 256
    // entries, the counts of the workgroup's segments, the totals of the workgroups before it
    const int32_t bc = min(b, nb - 1);
    const uint32_t cnt_early = cand_cnt[bc];
    float v0[4];
    int32_t j0[4];
    {
        const float *sv = cand_val + (int64_t)bc * blk;
        const int32_t *si = cand_idx + (int64_t)bc * blk;
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const int32_t ic = min(u * 64 + lane, blk - 1);
            v0[u] = sv[ic];
            j0[u] = si[ic];
        }
    }
    const int32_t bl = min(b0 + (lane & 15), nb - 1);
    uint32_t cg = cnt_gt[bl], ce = cnt_eq[bl];
    const uint32_t tau = sel->tau, quota = sel->quota, redo = sel->redo;
    uint32_t pg = 0, pq = 0;
    for (int32_t j = threadIdx.x; j < (int32_t)blockIdx.x; j += 1024) {
        pg += blk_gt[j];
        pq += blk_eq[j];
    }
    clear_histogram(hist_clear, kHist1Copies * kBins2);
    // totals of the workgroups before this one (integer sums: exact in any order)
    pg = wave_sum_u32(pg);
    pq = wave_sum_u32(pq);
    if (lane == 0) { s_part[0][w] = pg; s_part[1][w] = pq; }
    __syncthreads();
    if (b >= nb) return;
    uint32_t gt_before = 0, eq_before = 0;
#pragma unroll
    for (int i = 0; i < 16; i++) { gt_before += s_part[0][i]; eq_before += s_part[1][i]; }
    // the segments of this workgroup before b, and b's own counts
    const bool earlier = lane < w && b0 + lane < nb;
    const uint32_t own_g = __shfl(cg, w, 64), own_q = __shfl(ce, w, 64);
    gt_before += wave_sum_u32(earlier ? cg : 0u);
    eq_before += wave_sum_u32(earlier ? ce : 0u);

    const int32_t slot = step_view(step, m, kBefore).slot;
    uint8_t *row = ring + (int64_t)slot * row_bytes;
    uint32_t eq_run = eq_before;
    uint32_t out_run = gt_before + min(quota, eq_before);
    if (lane == 0) offT[(int64_t)b * m + slot] = (int32_t)out_run;     // where this slice's run starts
    if (b == nb - 1 && lane == 0) {
        // the end of the row: everything before the last segment plus the last segment's own share
        const uint32_t total = gt_before + own_g + min(quota, eq_before + own_q);
        offT[(int64_t)nb * m + slot] = (int32_t)total;
        sel->total = total;
        if (total != k) atomicOr(status, kStatusCount);
    }
    // 256 entries: which are taken, and where they go
    auto place = [&](const float (&vv)[4], const int32_t (&pp)[4], uint32_t i0, uint32_t cnt) {
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const bool in = i0 + u * 64 + lane < cnt;
            const float v = vv[u];
            const uint32_t key = mag_key(v);
            const bool is_eq = in && key == tau;
            const uint64_t eq_mask = __ballot(is_eq);
            const uint32_t eq_rank = eq_run + __popcll(eq_mask & ((1ull << lane) - 1ull));
            const bool take = in && (key > tau || (is_eq && eq_rank < quota));
            const uint64_t take_mask = __ballot(take);
            if (take) {
                const uint32_t pos = out_run + __popcll(take_mask & ((1ull << lane) - 1ull));
                *entry_idx_ptr<FMT>(row, pos) = (uint16_t)pp[u];                   // position inside the slice
                if constexpr (FMT == kFmtF32) *entry_val_ptr<FMT>(row, pos) = v;
                else *entry_val_ptr<FMT>(row, pos) = (uint16_t)bf16_bits(v);
            }
            eq_run += __popcll(eq_mask);
            out_run += __popcll(take_mask);
        }
    };
    Segment sg;
    uint32_t i_begin = 0;
    if (redo) {
        sg = segment_of(b, blk, d, 1u, e, cand_val, cand_idx, cand_cnt);
    } else {
        sg.first = (int32_t)((int64_t)b * blk);
        sg.val = cand_val + (int64_t)b * blk;
        sg.idx = cand_idx + (int64_t)b * blk;
        sg.cnt = cnt_early;
        int32_t p0[4];
#pragma unroll
        for (int u = 0; u < 4; u++) p0[u] = j0[u] - sg.first;
        place(v0, p0, 0u, sg.cnt);
        i_begin = 256;
    }
    for (uint32_t i0 = i_begin; i0 < sg.cnt; i0 += 256) {
        float vv[4];
        int32_t pp[4];
#pragma unroll
        for (int u = 0; u < 4; u++) {          // unconditional loads, clamped addresses
            const uint32_t ic = min(i0 + u * 64 + lane, sg.cnt - 1);
            vv[u] = sg.val[ic];
            pp[u] = sg.idx ? sg.idx[ic] - sg.first : (int32_t)ic;
        }
        place(vv, pp, i0, sg.cnt);
    }
}

// ------------------------------------------------------------------

hipError_t launch_ef_hist(const Geometry &g, const DevicePtrs &p, const float *grad, hipStream_t stream)
{
    if (g.fmt == kFmtBf16)
        hipLaunchKernelGGL((k_ef_hist<2>), dim3(g.n_slices), dim3(kEfThreads), 0, stream, grad, p.e,
                           g.d, p.hist1, p.sel, p.cand_idx, p.cand_val, p.cand_cnt, p.ring, g.row_bytes, p.offT,
                           g.m, g.slice, p.step);
    else
        hipLaunchKernelGGL((k_ef_hist<1>), dim3(g.n_slices), dim3(kEfThreads), 0, stream, grad, p.e,
                           g.d, p.hist1, p.sel, p.cand_idx, p.cand_val, p.cand_cnt, p.ring, g.row_bytes, p.offT,
                           g.m, g.slice, p.step);
    return hipGetLastError();
}

hipError_t launch_select(const Geometry &g, const DevicePtrs &p, bool evict, hipStream_t stream)
{
    const int32_t nb = g.n_slices;
    const int32_t nblk = (nb + kSegsPerBlock - 1) / kSegsPerBlock;
    // one wave per candidate segment until every workgroup of a histogram pass is in use
    const int32_t groups = nblk < kHistGroups ? nblk : kHistGroups;
    const int32_t n_evict = evict ? evict_blocks(g.m) : 0;
    // With the eviction update in it the first pass needs so many registers that one workgroup
    // fills a CU: it gets no more workgroups than there are CUs (kMaxWgs), the counting ones
    // taking several groups of segments each, rather than a second round behind the first.
    int32_t groups1 = groups;
    if (n_evict && groups1 + n_evict > kMaxWgs) groups1 = kMaxWgs - n_evict;       // n_evict <= 64
    hipLaunchKernelGGL(k_cand_hist<1>, dim3(groups1 + n_evict), dim3(1024), 0, stream, p.e, g.d, p.cand_val,
                       p.cand_idx, p.cand_cnt, nb, p.sel, p.hist1, p.hist2, (uint32_t *)nullptr, (uint32_t)g.k,
                       g.slice, groups1, p.rowmax, g.m, p.step, n_evict, g.ldm, p.W);
    hipLaunchKernelGGL(k_cand_hist<2>, dim3(groups), dim3(1024), 0, stream, p.e, g.d, p.cand_val, p.cand_idx,
                       p.cand_cnt, nb, p.sel, p.hist2, p.hist3, p.hist1, (uint32_t)g.k, g.slice, groups,
                       p.rowmax, g.m, p.step, 0, g.ldm, (double *)nullptr);
    hipLaunchKernelGGL(k_cand_count, dim3(nblk), dim3(1024), 0, stream, p.e, g.d, p.cand_val, p.cand_idx,
                       p.cand_cnt, nb, p.sel, p.hist3, p.hist2, (uint32_t)g.k, p.cnt_gt, p.cnt_eq, p.blk_gt,
                       p.blk_eq, g.slice);
    return hipGetLastError();
}

hipError_t launch_compact(const Geometry &g, const DevicePtrs &p, hipStream_t stream)
{
    const int32_t nblk = (g.n_slices + kSegsPerBlock - 1) / kSegsPerBlock;
    if (g.fmt == kFmtBf16)
        hipLaunchKernelGGL(k_cand_compact<kFmtBf16>, dim3(nblk), dim3(1024), 0, stream, p.e, g.d, p.cand_val,
                           p.cand_idx, p.cand_cnt, g.n_slices, p.sel, p.cnt_gt, p.cnt_eq, p.blk_gt, p.blk_eq,
                           p.hist3, p.ring, g.row_bytes, g.slice, p.offT, g.m, p.step, (uint32_t)g.k, p.status);
    else
        hipLaunchKernelGGL(k_cand_compact<kFmtF32>, dim3(nblk), dim3(1024), 0, stream, p.e, g.d, p.cand_val,
                           p.cand_idx, p.cand_cnt, g.n_slices, p.sel, p.cnt_gt, p.cnt_eq, p.blk_gt, p.blk_eq,
                           p.hist3, p.ring, g.row_bytes, g.slice, p.offT, g.m, p.step, (uint32_t)g.k, p.status);
    return hipGetLastError();
}

}  // namespace efcp
