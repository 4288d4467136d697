// efcp_internal.h -- shared declarations of the libefcp HIP sources (gfx950 only).
//
// Data layout in device memory (one context):
//   e         float  [d]                 error feedback xi (Algorithm 1); with the global
//                                        Top-k it holds the accumulator a between steps and
//                                        the entries of the newest row are dropped by the
//                                        next step's first pass (or by the host on read-out)
//   ring      bytes  [m][row_stride*E]   window G = (I, V), one row per slot, entries in
//                                        ascending index order, stored in groups of EPL
//                                        entries: the EPL indices (each a 16-bit position
//                                        inside its d-slice), then the EPL values (fp32 or
//                                        bfloat16).  E = 6 or 4 bytes per entry; the run of a
//                                        row inside one slice is one contiguous piece of memory
//   offT      int32  [n_slices+1][m]     offT[s][r] = first entry of row r whose
//                                        index is >= s*slice (slice-major so one
//                                        workgroup reads its m offsets contiguously).
//                                        slice = Geometry::slice coordinates, a multiple of
//                                        64 and at most 16,384, fixed when the context is made
//   S         double [m][m]              Gram matrix by slot
//   W         double [m rows][ldm]       inverse of the Cholesky factor of
//                                        m*lambda*I + S (rows in age order), stored
//                                        row-major by slot; zero above the diagonal
//                                        in age order and for unfilled slots
//   cand_*    [n_slices][slice]          Top-k candidates of the current step, one
//                                        segment per slice
//                                        (global Top-k only; block-wise Top-k keeps
//                                        two uint32 per block instead)
//   partial   double2[sp_grid][m]        per-workgroup (q, Gram) partial sums
//   sq        double2[m]                 (q_r, S[slot][r]) of the current step
//   zw        double2[m]                 (W s, W q) of the current step
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace efcp {

constexpr int kCandBlock = 16384;    // widest d-slice (its accumulators fill the LDS); block of the block-wise Top-k
constexpr int kMinSlice = 1024;      // narrowest slice chosen automatically
constexpr int kMaxWgs = 256;         // persistent SP / LCG workgroups at most: 32 on each of 8 XCDs
constexpr int kMaxM = 1024;          // window slots == threads of the m x m kernel
constexpr int kBins1 = 2048;         // first radix digit: key bits 30..20
constexpr int kHist1Copies = 4;      // copies of a digit's histogram that the blocks add into
constexpr int kBins2 = 1024;         // second: bits 19..10, third: bits 9..0
constexpr int kHistGroups = 1024;    // workgroups of a candidate histogram pass at most
constexpr int kGgtMaxM = 128;        // largest window of the Sparse GGT path (its matrix lives in LDS)
constexpr int kGgtMaxSweeps = 30;    // Jacobi sweeps at most (a sweep without rotations ends earlier)

// Window entry formats.  Indices are always stored as 16-bit positions inside the d-slice the
// entry falls in (the slice follows from the row's offset table), values as fp32 or bfloat16:
// 6 or 4 bytes per entry where an absolute int32 index next to an fp32 value would need 8.
// EPL = entries one lane takes per chunk (one load per array: iraw_t of indices, vraw_t of
// values); a chunk is what the GW lanes that share a row (16, or 4 where runs are short: see
// Geometry::row_lanes) read with these, GW * EPL entries; kBatch = chunks a lane keeps in flight.
enum : int { kFmtF32 = 0, kFmtBf16 = 1 };

template <int FMT> struct Fmt;
template <> struct Fmt<kFmtF32> {
    using idx_t = uint16_t;
    using val_t = float;
    using iraw_t = int2;     // 4 x uint16
    static constexpr int EPL = 4, kBatch = 3, kEntryBytes = 6;
};
template <> struct Fmt<kFmtBf16> {
    using idx_t = uint16_t;
    using val_t = uint16_t;
    using iraw_t = int2;     // 4 x uint16
    // A group is 4 entries = 16 bytes: one load per lane and chunk.  (Groups of 8, two 16-byte
    // loads per lane, left 36 % of the lanes idle on the ~164-entry runs of a 1 % window: a run
    // then needs two 128-entry chunks, and these passes are bound by vector-ALU work.)
    static constexpr int EPL = 4, kBatch = 3, kEntryBytes = 4;
};

// Entry p of a row lives in group p / EPL: [EPL x uint16 index][EPL x value].
template <int FMT>
__host__ __device__ __forceinline__ uint64_t group_offset(uint64_t p)
{
    return (p / Fmt<FMT>::EPL) * (uint64_t)(Fmt<FMT>::EPL * Fmt<FMT>::kEntryBytes);
}
template <int FMT>
__device__ __forceinline__ uint16_t *entry_idx_ptr(uint8_t *row, uint32_t p)
{
    return reinterpret_cast<uint16_t *>(row + group_offset<FMT>(p)) + (p % Fmt<FMT>::EPL);
}
template <int FMT>
__device__ __forceinline__ typename Fmt<FMT>::val_t *entry_val_ptr(uint8_t *row, uint32_t p)
{
    return reinterpret_cast<typename Fmt<FMT>::val_t *>(row + group_offset<FMT>(p) + 2 * Fmt<FMT>::EPL) +
           (p % Fmt<FMT>::EPL);
}
// One lane's group of a chunk: p is a multiple of EPL.  The fp32 values of a group start 8 bytes
// into it.
template <int FMT>
__device__ __forceinline__ void load_group(const uint8_t *row, uint32_t p, typename Fmt<FMT>::iraw_t &iv, int4 &vv)
{
    const uint8_t *g = row + (uint64_t)p * Fmt<FMT>::kEntryBytes;
    if constexpr (FMT == kFmtF32) {
        iv = *reinterpret_cast<const int2 *>(g);
        // 16 bytes at an 8-byte boundary: the compiler picks the widest load the target allows
        __builtin_memcpy(&vv, __builtin_assume_aligned(g + 8, 8), 16);
    } else {
        const int4 t = *reinterpret_cast<const int4 *>(g);       // indices and values of the group at once
        iv = make_int2(t.x, t.y);
        vv = make_int4(t.z, t.w, 0, 0);
    }
}

// Entry c (0..EPL-1) of a lane's loads: position inside the slice and value.
template <int FMT>
__device__ __forceinline__ int32_t entry_pos(const typename Fmt<FMT>::iraw_t &raw, int c, int32_t mask)
{
    const int32_t w[2] = {raw.x, raw.y};
    return (int32_t)(((uint32_t)w[c >> 1] >> ((c & 1) * 16)) & 0xffffu) & mask;
}

template <int FMT>
__device__ __forceinline__ float entry_val(const int4 &raw, int c)
{
    const int32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
    if constexpr (FMT == kFmtF32) return __int_as_float(w[c]);
    else return __uint_as_float((((uint32_t)w[c >> 1] >> ((c & 1) * 16)) & 0xffffu) << 16);
}

// A single stored entry as (position in its slice, fp32 value).
__device__ __forceinline__ float stored_val(float v) { return v; }
__device__ __forceinline__ float stored_val(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }
__device__ __forceinline__ int32_t stored_pos(uint16_t i, int32_t mask) { return (int32_t)i & mask; }

// fp32 -> bfloat16 bits, round to nearest even (inputs are finite).
__device__ __forceinline__ uint32_t bf16_bits(float a)
{
    const uint32_t b = __float_as_uint(a);
    return (b + 0x7fffu + ((b >> 16) & 1u)) >> 16;
}

// Device-resident state of the radix select of the current step.  Each field has one writer
// (workgroup 0 of the pass that settles it) and is read only by later kernels.
struct SelState {
    uint32_t p1, kr1;    // digit 1 (key bits 30..20) and the rank still wanted inside that bin
    uint32_t p2, kr2;    // digits 1 and 2 (bits 30..10), rank inside that bin
    uint32_t tau;        // final threshold key (k-th largest magnitude key)
    uint32_t quota;      // how many keys == tau are selected (lowest indices first)
    uint32_t n_gt;       // number of keys > tau
    uint32_t total;      // entries written to the new row (must equal k)
    uint32_t t_lo;       // keys >= t_lo are copied to the candidate list by the first pass
    uint32_t redo;       // 1: the threshold bin lies below t_lo, the passes read the accumulator
};

enum : uint32_t { kStatusPivot = 1u, kStatusCount = 2u, kStatusRange = 4u };

// Where the context is in its sequence of steps.  It lives in device memory and is advanced by
// the step's own kernels, so that no kernel argument depends on the step number: a step captured
// in a HIP graph can be replayed as every later step.
//   t_done      steps completed.  A step's kernels up to and including the SP pass run with
//               t_done = t - 1 ("before": the slot written is t_done mod m, t_done + 1 rows are
//               filled afterwards at most m, the oldest row is evicted iff t_done >= m); the
//               reduction of the SP partial sums then adds one, and everything after it (the
//               coefficient kernels, the LCG pass, efcp_apply) sees t_done = t ("after").
//   pend_slot   global Top-k: the slot whose row still has to be taken out of e (the next step's
//               first pass does it; read-outs do it on the host); -1: e is final.
struct StepState {
    long long t_done;
    int32_t pend_slot;
    int32_t reserved;
};

struct StepView {
    int32_t slot;        // before: the slot this step writes; after: the slot written last
    int32_t n_filled;    // rows of the window that hold a vector (including this step's)
    int32_t evict;       // before: this step replaces a row (the window was full)
};

enum : int { kBefore = 0, kAfter = 1 };

__device__ __forceinline__ StepView step_view(const StepState *__restrict__ st, int32_t m, int phase)
{
    const long long td = st->t_done;
    StepView v;
    if (phase == kBefore) {
        v.slot = (int32_t)(td % m);
        v.n_filled = (int32_t)(td + 1 < (long long)m ? td + 1 : (long long)m);
        v.evict = td >= (long long)m ? 1 : 0;
    } else {
        v.slot = td > 0 ? (int32_t)((td - 1) % m) : 0;
        v.n_filled = (int32_t)(td < (long long)m ? td : (long long)m);
        v.evict = 0;
    }
    return v;
}

struct Geometry {
    int64_t d, k, row_stride;    // row_stride: entries per row of the ring (k rounded up to 64)
    int64_t row_bytes;           // row_stride * bytes per entry
    int32_t kb;              // 0: global Top-k; > 0: Top-k in blocks, entries kept per full block
    int32_t ggt;             // 0: Sparse M-FAC coefficients; 1: Sparse GGT
    int32_t m, ldm;
    int32_t fmt;             // kFmtF32 / kFmtBf16
    int32_t slice, n_slices; // coordinates per d-slice (multiple of 64, <= kCandBlock), number of slices
    int32_t sp_grid;         // persistent SP workgroups: 8 * (workgroups per XCD)
    int32_t row_lanes;       // lanes of the SP / LCG workgroups that share a row: 16, or 4 where a row has few
                             // entries per slice (a workgroup then works on 256 rows at once instead of 64)
    size_t lds_sp, lds_lcg;
};

struct DevicePtrs {
    float *e;
    uint8_t *ring;           // [m][row_stride * bytes per entry], see the top of this file
    int32_t *offT;
    double *S, *W;
    double2 *partial, *sq, *zw;
    double *q, *coef;
    uint32_t *rowmax;
    uint32_t *hist1, *hist2, *hist3;
    SelState *sel;
    uint32_t *cnt_gt, *cnt_eq;       // [n_slices] keys > tau / == tau per candidate segment
    uint32_t *blk_gt, *blk_eq;       // the same per workgroup of 16 segments
    int32_t *cand_idx;       // [n_slices][slice] candidate indices, ascending per segment
    float *cand_val;         // [n_slices][slice] candidate values
    uint32_t *cand_cnt;      // [n_slices] entries used per segment
    uint32_t *blk_max;       // [n_slices] largest key per block          (block-wise Top-k only)
    uint32_t *blk_tlo;       // [n_slices] where each block's first histogram starts counting
    double *lam;             // [m] eigenvalues of S                      (Sparse GGT only)
    double2 *rot;            // [kGgtMaxSweeps*(kGgtMaxM-1)][64] logged rotations (c, s)
    int32_t *n_stages;       // stages logged by the last decomposition
    int32_t *col;            // [n_slices+1] one column of offT, gathered for read-outs
    uint32_t *status;
    StepState *step;
};

// Launchers (each enqueues on `stream` and returns hipGetLastError()).
// No launcher takes the step number, the slot or the number of filled rows: the kernels read them
// from p.step.
hipError_t launch_ef_hist(const Geometry &g, const DevicePtrs &p, const float *grad, hipStream_t stream);
hipError_t launch_select(const Geometry &g, const DevicePtrs &p, bool evict, hipStream_t stream);
hipError_t launch_compact(const Geometry &g, const DevicePtrs &p, hipStream_t stream);
hipError_t launch_block_topk(const Geometry &g, const DevicePtrs &p, const float *grad, hipStream_t stream);
// x_source: 0 = dense x next to the newest row (a step), 1 = the newest row is x (a step),
// 2 = dense x only, on the window as it stands (efcp_apply)
hipError_t launch_sp(const Geometry &g, const DevicePtrs &p, const float *x, int32_t x_source,
                     hipStream_t stream);
// commit: this reduction ends the "before" part of a step: it advances p.step
hipError_t launch_sp_reduce(const Geometry &g, const DevicePtrs &p, bool commit, hipStream_t stream);
hipError_t launch_evict(const Geometry &g, const DevicePtrs &p, hipStream_t stream);
hipError_t launch_coef(const Geometry &g, const DevicePtrs &p, double lambda, hipStream_t stream);
// Coefficients for an arbitrary x on the window as it stands (nothing is inserted).
hipError_t launch_coef_apply(const Geometry &g, const DevicePtrs &p, double lambda, hipStream_t stream);
hipError_t launch_ggt_step(const Geometry &g, const DevicePtrs &p, double eps, hipStream_t stream);
hipError_t launch_ggt_apply(const Geometry &g, const DevicePtrs &p, double eps, hipStream_t stream);
hipError_t launch_ggt_refresh(const Geometry &g, const DevicePtrs &p, hipStream_t stream);
hipError_t configure_ggt();
struct LcgMode {
    bool x_is_newest_row = false;    // x is the row written last (the dense pointer is not read)
    bool update = false;             // out holds parameters: theta <- decay*theta - lr*(F^-1 x)
    double decay = 1.0, lr = 0.0;
};
hipError_t launch_lcg(const Geometry &g, const DevicePtrs &p, const float *x, float *out, double lambda,
                      const LcgMode &md, hipStream_t stream);
hipError_t configure_sp(const Geometry &g);
hipError_t configure_lcg(const Geometry &g);

// ---- small device helpers shared by the kernels ----

// Static list of the d-slices one persistent SP / LCG workgroup walks.  An XCD owns the
// contiguous range [first, end); its `cpx` workgroups take it in rounds of cpx neighbouring
// slices, and in round i workgroup `cu` takes position (cu + i) mod cpx of the round.  The
// rotation matters most when every row has the same run boundaries (Top-k applied in blocks):
// how a slice's runs sit relative to cache lines depends on s mod 8, and without it a
// workgroup keeps the same s mod 8, good or bad, for the whole pass (measured on one box:
// LCG pass 5 % slower without the rotation at 164 entries per block, 1 % with global Top-k).
struct SliceList {
    int32_t first, cu, cpx, count;
    __device__ __forceinline__ SliceList(int32_t first_, int32_t end, int32_t cu_, int32_t cpx_)
        : first(first_), cu(cu_), cpx(cpx_)
    {
        const int32_t n = end > first_ ? end - first_ : 0;
        const int32_t rounds = (n + cpx_ - 1) / cpx_;
        // all rounds but the last are complete; in the last one only the first n - (rounds-1)*cpx
        // positions exist
        count = rounds == 0 ? 0 : (rounds - 1) + ((first_ + pos(rounds - 1)) < end ? 1 : 0);
    }
    __device__ __forceinline__ int32_t pos(int32_t i) const { return i * cpx + (cu + i) % cpx; }
    __device__ __forceinline__ int32_t at(int32_t i) const { return first + pos(i); }
};

// Streaming accesses: data read or written exactly once per step (the gradient, the error
// buffer, the output) is moved with the non-temporal hint so that it does not displace the
// window lines that neighbouring workgroups share in L2.  (Measured: the hint on the output
// store shortens the LCG pass by 10 %; on the window loads themselves it costs 30 %.)
typedef float efcp_v4f __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float4 load_stream_f4(const float *p)
{
    const efcp_v4f t = __builtin_nontemporal_load(reinterpret_cast<const efcp_v4f *>(p));
    return make_float4(t.x, t.y, t.z, t.w);
}

__device__ __forceinline__ void store_stream_f4(float *p, float4 v)
{
    const efcp_v4f t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, reinterpret_cast<efcp_v4f *>(p));
}

__device__ __forceinline__ uint32_t mag_key(float a) { return __float_as_uint(a) & 0x7fffffffu; }

__device__ __forceinline__ uint32_t wave_incl_scan_u32(uint32_t v)
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        uint32_t n = __shfl_up(v, o, 64);
        if (lane >= o) v += n;
    }
    return v;
}

// A double moved between lanes by a DPP pattern that gives every lane a source lane (rotations,
// mirrors and quad permutations inside a row of 16): no LDS traffic.
template <int CTRL>
__device__ __forceinline__ double dpp_moved(double v)
{
    const int lo = __builtin_amdgcn_mov_dpp(__double2loint(v), CTRL, 0xf, 0xf, false);
    const int hi = __builtin_amdgcn_mov_dpp(__double2hiint(v), CTRL, 0xf, 0xf, false);
    return __hiloint2double(hi, lo);
}

// Sums of TWO doubles over each aligned group of GW lanes (16 or 4), fixed order: the lower half
// of the group ends with the sum of a, the upper half with the sum of b.  In the first step each
// lane hands the value it will not keep to the lane half a group away; the rest stays inside the
// halves (16 lanes: lane i with 7 - i, then lane ^ 1, then lane ^ 2; 4 lanes: lane ^ 1).
template <int GW>
__device__ __forceinline__ double row_sum2_f64(double a, double b)
{
    static_assert(GW == 16 || GW == 4, "group width");
    const bool upper = (threadIdx.x & (GW / 2)) != 0;
    double keep = upper ? b : a;
    const double give = upper ? a : b;
    if constexpr (GW == 16) {
        keep += dpp_moved<0x128>(give);      // row_ror:8
        keep += dpp_moved<0x141>(keep);      // row_half_mirror
        keep += dpp_moved<0xB1>(keep);       // quad_perm [1,0,3,2]
        keep += dpp_moved<0x4E>(keep);       // quad_perm [2,3,0,1]
    } else {
        keep += dpp_moved<0x4E>(give);       // quad_perm [2,3,0,1]
        keep += dpp_moved<0xB1>(keep);       // quad_perm [1,0,3,2]
    }
    return keep;
}

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// Exclusive prefix sum over the threads of a block (blockDim.x multiple of 64,
// at most 1024).  `tmp` needs 33 uint32 of LDS.  Every thread must call it.
__device__ __forceinline__ uint32_t block_excl_scan_u32(uint32_t v, uint32_t *tmp, uint32_t *total)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const uint32_t incl = wave_incl_scan_u32(v);
    if (lane == 63) tmp[w] = incl;
    __syncthreads();
    if (w == 0) {
        const uint32_t s = lane < nw ? tmp[lane] : 0u;
        const uint32_t si = wave_incl_scan_u32(s);
        if (lane < nw) tmp[lane] = si - s;
        if (lane == 63) tmp[32] = si;
    }
    __syncthreads();
    const uint32_t res = tmp[w] + incl - v;
    *total = tmp[32];
    __syncthreads();
    return res;
}

}  // namespace efcp
