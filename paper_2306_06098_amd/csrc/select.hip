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
// at least t_lo -- a bin edge two bins below the previous step's threshold --
// to a candidate list, in index order, one segment per block (a d-slice, at
// most 16,384 coordinates).  All later passes (two digit histograms, per-block counts and
// the ordered compaction into the ring) read the candidates only: a few
// percent of d.  e = a - c is not finished by this step: clearing k scattered
// entries costs a partial HBM write each, so the buffer keeps a, and the NEXT
// step's first pass, which rewrites e anyway, drops the entries of the row
// inserted last (a bitmap in LDS, one bit per coordinate of the block).  Host code
// that reads e in between applies the same rule.  The first-digit histogram
// is exact, so it tells whether the threshold bin lies at or above t_lo; if it
// does not (the threshold dropped by more than two bins in one step), one
// extra pass over a rebuilds the candidates from the now known bin.  The
// result is exact either way; the prediction only saves traffic.
//
// Histograms are merged with integer atomics (order independent), candidates
// and rows are written at positions computed by prefix sums, so every output
// is deterministic.
#include "efcp_internal.h"

namespace efcp {

// Streaming layout of a d-sized pass: a block owns one d-slice (`blk`
// consecutive coordinates, a multiple of 256 and at most 16,384), walked in
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
// REDO = true: the pass that rebuilds the candidates from a (already in e)
// with the threshold bin found by the first digit; it exits at once unless
// the select state asks for it.
// PEND (first pass only; 1: fp32 window, 2: bfloat16 window): if the step state names a pending
// slot, `e` still holds the previous step's accumulator; the entries of the row inserted then (the
// run of this block given by two entries of its offset column) count as +0, or as the rounding
// remainder a - bf16(a) when the window keeps bfloat16 values.
constexpr int kEfThreads = 512;                  // threads of a first-pass block
constexpr int kEfWaves = kEfThreads / 64;
constexpr int kEfChunk = kEfWaves * 1024;        // coordinates the block streams at a time

template <bool REDO, int PEND>
__global__ __launch_bounds__(kEfThreads) void k_ef_hist(const float *__restrict__ g,
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
    __shared__ uint32_t lh[REDO ? 1 : kBins1];
    __shared__ uint32_t s_cnt[2][kEfWaves];
    __shared__ uint32_t pend[PEND ? kCandBlock / 32 : 1];       // one bit per coordinate of the block
    uint32_t t_lo;
    if (REDO) {
        if (!sel->redo) return;
        t_lo = sel->prefix << 20;
    } else {
        t_lo = sel->t_lo;
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
    }
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
        // of 256 coordinates (always, except in the last block of a vector of ragged length):
        // nit of the wave's four 256-coordinate pieces exist.
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
                    if (!REDO) gv[it] = load_stream_f4(g + wave_base + it * 256);
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
                if (REDO) {
                    a[it][0] = ev[it].x; a[it][1] = ev[it].y; a[it][2] = ev[it].z; a[it][3] = ev[it].w;
                } else {
                    a[it][0] = ev[it].x + gv[it].x;
                    a[it][1] = ev[it].y + gv[it].y;
                    a[it][2] = ev[it].z + gv[it].z;
                    a[it][3] = ev[it].w + gv[it].w;
                    if (it < nit)
                        store_stream_f4(e + wave_base + it * 256,
                                        make_float4(a[it][0], a[it][1], a[it][2], a[it][3]));
                }
            }
        };
        if (rem >= 1024) {
            vector_pieces(4);
            inmask = 0xffffu;
        } else if (rem <= 0 || (rem & 255) == 0) {
            const int nit = rem <= 0 ? 0 : (int)(rem >> 8);
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
                        t = REDO ? ej : ej + g[j];
                        if (!REDO) e[j] = t;
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
                    if (!REDO) atomicAdd(&lh[key >> 20], 1u);
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
    if (!REDO) {
        __syncthreads();
        // Most keys fall into a few dozen bins, which every block adds to at about the same time:
        // the adds to one address queue up, so the blocks are spread over kHist1Copies histograms.
        uint32_t *mine = hist + (blockIdx.x % kHist1Copies) * kBins1;
        for (int i = threadIdx.x; i < kBins1; i += kEfThreads) {
            const uint32_t c = lh[i];
            if (c) atomicAdd(&mine[i], c);
        }
    }
}

// ------------------------------------------------------------------
// Histogram of the next 10-bit digit over the candidates whose higher key
// bits equal the prefix found so far.  `groups` (at most kHistGroups) workgroups of 16 waves; a
// wave takes one candidate segment at a time.  Every workgroup counts in its own
// 1024-bin histogram in LDS (device-scope atomics on a few hot addresses from
// thousands of waves serialise) and adds it once, at the end, into one of
// kHist1Copies histograms in memory; k_pick_digit adds those up and clears them.

__global__ __launch_bounds__(1024) void k_cand_hist(const float *__restrict__ cand_val,
                                                    const uint32_t *__restrict__ cand_cnt, int32_t nb,
                                                    const SelState *__restrict__ sel,
                                                    uint32_t *__restrict__ hist_priv, int shift_hi,
                                                    int shift_lo, int32_t blk, int32_t groups)
{
    __shared__ uint32_t lh[kBins2];
    lh[threadIdx.x] = 0;
    __syncthreads();
    const uint32_t prefix = sel->prefix;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    // The count of the wave's next segment is fetched while the current one is processed, and
    // eight loads per lane are issued before any is used (unconditional, clamped addresses).
    int32_t b = blockIdx.x * 16 + w;
    uint32_t cnt = b < nb ? cand_cnt[b] : 0u;
    while (b < nb) {
        const int32_t bn = b + groups * 16;
        const uint32_t cnt_next = cand_cnt[min(bn, nb - 1)];
        const float *seg = cand_val + (int64_t)b * blk;
        for (uint32_t i0 = 0; i0 < cnt; i0 += 512) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; u++) v[u] = seg[min(i0 + u * 64 + lane, cnt - 1)];
#pragma unroll
            for (int u = 0; u < 8; u++) {
                const uint32_t kk = mag_key(v[u]);
                if (i0 + u * 64 + lane < cnt && (kk >> shift_hi) == prefix)
                    atomicAdd(&lh[(kk >> shift_lo) & (kBins2 - 1)], 1u);
            }
        }
        b = bn;
        cnt = cnt_next;
    }
    __syncthreads();
    const uint32_t c = lh[threadIdx.x];
    if (c) atomicAdd(&hist_priv[(blockIdx.x % kHist1Copies) * kBins2 + threadIdx.x], c);
}

// ------------------------------------------------------------------
// One workgroup: locate the digit in which the kr-th largest remaining key
// falls and update the select state.
// pass 0: 2048 bins (bits 30..20); pass 1, 2: 1024 bins.
template <int NB>
__global__ __launch_bounds__(1024) void k_pick_digit(uint32_t *__restrict__ hist,
                                                     SelState *__restrict__ sel, int pass,
                                                     uint32_t k, uint32_t *__restrict__ rowmax, int32_t m,
                                                     const StepState *__restrict__ step)
{
    __shared__ uint32_t tmp[33];
    __shared__ int top_bin;
    if (threadIdx.x == 0) top_bin = 0;
    __syncthreads();
    constexpr int PER = NB / 1024;
    const uint32_t kr = (pass == 0) ? k : sel->kr;
    const uint32_t prefix = (pass == 0) ? 0u : sel->prefix;
    const uint32_t t_lo = sel->t_lo;

    // Walk the bins from the largest digit down: rb = NB-1-bin.  `hist` holds kHist1Copies
    // histograms filled by atomics; they are added up here and cleared for the next step.
    uint32_t c[PER];
    uint32_t local = 0;
#pragma unroll
    for (int i = 0; i < PER; i++) {
        const int bin = NB - 1 - (threadIdx.x * PER + i);
        uint32_t v[kHist1Copies];
#pragma unroll
        for (int u = 0; u < kHist1Copies; u++) v[u] = hist[u * NB + bin];
        uint32_t t = 0;
#pragma unroll
        for (int u = 0; u < kHist1Copies; u++) {
            t += v[u];
            if (v[u]) hist[u * NB + bin] = 0;
        }
        c[i] = t;
        if (pass == 0 && t) atomicMax(&top_bin, bin);
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
            if (pass == 0) {
                // candidates hold every key >= t_lo: enough iff the threshold bin starts at or above t_lo
                sel->redo = ((uint32_t)bin << 20) < t_lo ? 1u : 0u;
            }
            if (pass == 2) {
                sel->tau = np;
                sel->quota = kr - above;
                sel->n_gt = k - (kr - above);
                const uint32_t tb = np >> 20;             // next step collects from two bins below
                sel->t_lo = (tb >= 2 ? tb - 2 : 0u) << 20;
            }
        }
        above += c[i];
    }
    if (pass == 0 && threadIdx.x == 0) {
        // every |a_j| of this step is below the upper edge of the highest occupied bin:
        // an upper bound on the largest stored magnitude, enough to scale the LCG sum
        const uint32_t edge = ((uint32_t)top_bin + 1u) << 20;
        rowmax[step_view(step, m, kBefore).slot] = edge < 0x7f7fffffu ? edge : 0x7f7fffffu;
    }
}

// ------------------------------------------------------------------
// Per candidate segment: how many keys are > tau and == tau.  One wave per segment.
__global__ __launch_bounds__(kSelThreads) void k_cand_count(const float *__restrict__ cand_val,
                                                            const uint32_t *__restrict__ cand_cnt,
                                                            int32_t nb, const SelState *__restrict__ sel,
                                                            uint32_t *__restrict__ cnt_gt,
                                                            uint32_t *__restrict__ cnt_eq, int32_t blk)
{
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int32_t b = blockIdx.x * 4 + w;
    if (b >= nb) return;
    const uint32_t tau = sel->tau;
    const uint32_t cnt = cand_cnt[b];
    const float *seg = cand_val + (int64_t)b * blk;
    uint32_t g = 0, q = 0;
    for (uint32_t i0 = 0; i0 < cnt; i0 += 512) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; u++) v[u] = seg[min(i0 + u * 64 + lane, cnt - 1)];
#pragma unroll
        for (int u = 0; u < 8; u++) {
            const uint32_t key = mag_key(v[u]);
            const bool in = i0 + u * 64 + lane < cnt;
            g += in && key > tau;
            q += in && key == tau;
        }
    }
    g = wave_sum_u32(g);
    q = wave_sum_u32(q);
    if (lane == 0) { cnt_gt[b] = g; cnt_eq[b] = q; }
}

// ------------------------------------------------------------------
// One workgroup: exclusive scans over the candidate segments.
//   eq_before[b] = number of keys == tau in segments before b
//   sel_off[b]   = number of selected entries in segments before b
// and the end of the new row's offset column, offT[n_slices][slot] = k; the other entries of
// the column (offT[s][slot] = sel_off[s]: a segment is a slice) are strided single stores, which
// the compaction kernel spreads over its waves.
__global__ __launch_bounds__(1024) void k_scan_blocks(const uint32_t *__restrict__ cnt_gt,
                                                      const uint32_t *__restrict__ cnt_eq,
                                                      uint32_t *__restrict__ sel_off,
                                                      uint32_t *__restrict__ eq_before,
                                                      SelState *__restrict__ sel, int32_t nb,
                                                      int32_t m, const StepState *__restrict__ step,
                                                      int32_t *__restrict__ offT, uint32_t k,
                                                      uint32_t *__restrict__ status)
{
    __shared__ uint32_t tmp[33];
    const uint32_t quota = sel->quota;
    uint32_t carry_eq = 0, carry_sel = 0;
    for (int32_t tile = 0; tile < nb; tile += 4096) {
        const int32_t b = tile + (int32_t)threadIdx.x * 4;
        uint32_t ce[4] = {0, 0, 0, 0}, cg[4] = {0, 0, 0, 0};
        if (b + 3 < nb) {
            const uint4 t0 = *reinterpret_cast<const uint4 *>(cnt_eq + b);
            const uint4 t1 = *reinterpret_cast<const uint4 *>(cnt_gt + b);
            ce[0] = t0.x; ce[1] = t0.y; ce[2] = t0.z; ce[3] = t0.w;
            cg[0] = t1.x; cg[1] = t1.y; cg[2] = t1.z; cg[3] = t1.w;
        } else {
            for (int i = 0; i < 4; i++)
                if (b + i < nb) { ce[i] = cnt_eq[b + i]; cg[i] = cnt_gt[b + i]; }
        }
        uint32_t total_eq, total_sel;
        uint32_t run = carry_eq + block_excl_scan_u32(ce[0] + ce[1] + ce[2] + ce[3], tmp, &total_eq);
        uint32_t sc[4], eb[4];
#pragma unroll
        for (int i = 0; i < 4; i++) {
            eb[i] = run;
            const uint32_t take = run >= quota ? 0u : min(quota - run, ce[i]);
            sc[i] = cg[i] + take;
            run += ce[i];
        }
        uint32_t run2 = carry_sel + block_excl_scan_u32(sc[0] + sc[1] + sc[2] + sc[3], tmp, &total_sel);
#pragma unroll
        for (int i = 0; i < 4; i++) {
            if (b + i < nb) {
                eq_before[b + i] = eb[i];
                sel_off[b + i] = run2;           // k_cand_compact copies it into the offset table
            }
            run2 += sc[i];
        }
        carry_eq += total_eq;
        carry_sel += total_sel;
    }
    if (threadIdx.x == 0) {
        offT[(int64_t)nb * m + step_view(step, m, kBefore).slot] = (int32_t)carry_sel;
        sel->total = carry_sel;
        if (carry_sel != k) atomicOr(status, kStatusCount);
    }
}

// ------------------------------------------------------------------
// Ordered compaction of the selected candidates of segment b into the ring
// row (16-bit positions inside the segment = slice; fp32 or bfloat16 values).
// The error buffer is left as it is: see the top of this file.
// One wave per segment; candidates are already in index order.
template <int FMT>
__global__ __launch_bounds__(kSelThreads) void k_cand_compact(const int32_t *__restrict__ cand_idx,
                                                              const float *__restrict__ cand_val,
                                                              const uint32_t *__restrict__ cand_cnt,
                                                              int32_t nb,
                                                              const SelState *__restrict__ sel,
                                                              const uint32_t *__restrict__ sel_off,
                                                              const uint32_t *__restrict__ eq_before,
                                                              uint8_t *__restrict__ ring,
                                                              int64_t row_bytes, int32_t blk,
                                                              int32_t *__restrict__ offT, int32_t m,
                                                              const StepState *__restrict__ step)
{
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int32_t b = blockIdx.x * 4 + w;
    if (b >= nb) return;
    const int32_t slot = step_view(step, m, kBefore).slot;
    uint8_t *row = ring + (int64_t)slot * row_bytes;
    const int32_t seg_first = b * blk;
    const uint32_t tau = sel->tau, quota = sel->quota;
    const uint32_t cnt = cand_cnt[b];
    const int32_t *sidx = cand_idx + (int64_t)b * blk;
    const float *sval = cand_val + (int64_t)b * blk;
    uint32_t eq_run = eq_before[b];
    uint32_t out_run = sel_off[b];
    if (lane == 0) offT[(int64_t)b * m + slot] = (int32_t)out_run;     // where this slice's run starts
    for (uint32_t i0 = 0; i0 < cnt; i0 += 256) {
        float vv[4];
        int32_t jj[4];
#pragma unroll
        for (int u = 0; u < 4; u++) {          // unconditional loads, clamped addresses
            const uint32_t ic = min(i0 + u * 64 + lane, cnt - 1);
            vv[u] = sval[ic];
            jj[u] = sidx[ic];
        }
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const bool in = i0 + u * 64 + lane < cnt;
            const float v = vv[u];
            const int32_t j = jj[u];
            const uint32_t key = mag_key(v);
            const bool is_eq = in && key == tau;
            const uint64_t eq_mask = __ballot(is_eq);
            const uint32_t eq_rank = eq_run + __popcll(eq_mask & ((1ull << lane) - 1ull));
            const bool take = in && (key > tau || (is_eq && eq_rank < quota));
            const uint64_t take_mask = __ballot(take);
            if (take) {
                const uint32_t pos = out_run + __popcll(take_mask & ((1ull << lane) - 1ull));
                *entry_idx_ptr<FMT>(row, pos) = (uint16_t)(j - seg_first);     // position inside the slice
                if constexpr (FMT == kFmtF32) *entry_val_ptr<FMT>(row, pos) = v;
                else *entry_val_ptr<FMT>(row, pos) = (uint16_t)bf16_bits(v);
            }
            eq_run += __popcll(eq_mask);
            out_run += __popcll(take_mask);
        }
    }
}

// ------------------------------------------------------------------

hipError_t launch_ef_hist(const Geometry &g, const DevicePtrs &p, const float *grad, hipStream_t stream)
{
    if (g.fmt == kFmtBf16)
        hipLaunchKernelGGL((k_ef_hist<false, 2>), dim3(g.n_slices), dim3(kEfThreads), 0, stream, grad, p.e,
                           g.d, p.hist1, p.sel, p.cand_idx, p.cand_val, p.cand_cnt, p.ring, g.row_bytes, p.offT,
                           g.m, g.slice, p.step);
    else
        hipLaunchKernelGGL((k_ef_hist<false, 1>), dim3(g.n_slices), dim3(kEfThreads), 0, stream, grad, p.e,
                           g.d, p.hist1, p.sel, p.cand_idx, p.cand_val, p.cand_cnt, p.ring, g.row_bytes, p.offT,
                           g.m, g.slice, p.step);
    return hipGetLastError();
}

hipError_t launch_select(const Geometry &g, const DevicePtrs &p, hipStream_t stream)
{
    const int32_t nb = g.n_slices;
    // one wave per candidate segment until every private histogram is in use
    const int32_t groups = (nb + 15) / 16 < kHistGroups ? (nb + 15) / 16 : kHistGroups;
    hipLaunchKernelGGL(k_pick_digit<kBins1>, dim3(1), dim3(1024), 0, stream, p.hist1, p.sel, 0,
                       (uint32_t)g.k, p.rowmax, g.m, p.step);
    hipLaunchKernelGGL((k_ef_hist<true, 0>), dim3(nb), dim3(kEfThreads), 0, stream, (const float *)nullptr,
                       p.e, g.d, p.hist1, p.sel, p.cand_idx, p.cand_val, p.cand_cnt, p.ring, g.row_bytes,
                       p.offT, g.m, g.slice, p.step);
    hipLaunchKernelGGL(k_cand_hist, dim3(groups), dim3(1024), 0, stream, p.cand_val, p.cand_cnt, nb,
                       p.sel, p.hist2, 20, 10, g.slice, groups);
    hipLaunchKernelGGL(k_pick_digit<kBins2>, dim3(1), dim3(1024), 0, stream, p.hist2, p.sel, 1,
                       (uint32_t)g.k, p.rowmax, g.m, p.step);
    hipLaunchKernelGGL(k_cand_hist, dim3(groups), dim3(1024), 0, stream, p.cand_val, p.cand_cnt, nb,
                       p.sel, p.hist3, 10, 0, g.slice, groups);
    hipLaunchKernelGGL(k_pick_digit<kBins2>, dim3(1), dim3(1024), 0, stream, p.hist3, p.sel, 2,
                       (uint32_t)g.k, p.rowmax, g.m, p.step);
    hipLaunchKernelGGL(k_cand_count, dim3((nb + 3) / 4), dim3(kSelThreads), 0, stream, p.cand_val,
                       p.cand_cnt, nb, p.sel, p.cnt_gt, p.cnt_eq, g.slice);
    hipLaunchKernelGGL(k_scan_blocks, dim3(1), dim3(1024), 0, stream, p.cnt_gt, p.cnt_eq, p.sel_off,
                       p.eq_before, p.sel, nb, g.m, p.step, p.offT,
                       (uint32_t)g.k, p.status);
    return hipGetLastError();
}

hipError_t launch_compact(const Geometry &g, const DevicePtrs &p, hipStream_t stream)
{
    if (g.fmt == kFmtBf16)
        hipLaunchKernelGGL(k_cand_compact<kFmtBf16>, dim3((g.n_slices + 3) / 4), dim3(kSelThreads), 0,
                           stream, p.cand_idx, p.cand_val, p.cand_cnt, g.n_slices, p.sel, p.sel_off,
                           p.eq_before, p.ring, g.row_bytes, g.slice, p.offT, g.m, p.step);
    else
        hipLaunchKernelGGL(k_cand_compact<kFmtF32>, dim3((g.n_slices + 3) / 4), dim3(kSelThreads), 0,
                           stream, p.cand_idx, p.cand_val, p.cand_cnt, g.n_slices, p.sel, p.sel_off,
                           p.eq_before, p.ring, g.row_bytes, g.slice, p.offT, g.m, p.step);
    return hipGetLastError();
}

}  // namespace efcp
