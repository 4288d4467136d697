// efcp.hip -- host side of libefcp: the C ABI declared in include/efcp.h.
// Validates arguments, lays the state out in one device workspace, and
// enqueues the kernels of one step (Algorithm 1, lines 5-8) on the caller's
// stream.  No host synchronisation and no allocation happen inside efcp_step.
#include "../../include/efcp.h"
#include "efcp_internal.h"

#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

using namespace efcp;

namespace {

constexpr int kProfSteps = 256;
constexpr int kProfEvents = EFCP_K_COUNT + 1;

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Entries per row when every block of kCandBlock coordinates keeps kb and a ragged last block
// keeps the same share rounded up.
int64_t block_row_length(int64_t d, int64_t kb)
{
    const int64_t full = d / kCandBlock, tail = d % kCandBlock;
    return full * kb + (tail ? (kb * tail + kCandBlock - 1) / kCandBlock : 0);
}

// Width of the d-slices that the SP and LCG workgroups stage in LDS, which are also the blocks of
// the Top-k passes.  With Top-k in blocks it is the block.  Otherwise: the widest slice leaves
// the persistent workgroups with unequal numbers of slices (684 slices of 16,384 over 256
// workgroups: three rounds, the last one two thirds empty; 6,714 slices: 26 rounds and 58 slices),
// and a last round costs the SP and the LCG pass almost a whole round however little it holds
// (measured at d = 110M: 40 and 44 us of the 47 and 55 us of a full one).  When the rounds would
// hold at least 2 % more slices than there are, the vector is therefore cut into nearly equal
// slices, a multiple of 64 coordinates each, as narrow as the same number of rounds allows, so that
// every workgroup takes part in every round (d = 110M: 6,903 slices of 15,936 = 27 rounds, 9 places
// empty: SP 1.243 -> 1.216 ms, LCG 1.356 -> 1.344, the first Top-k pass, which pays a fixed cost
// per block, 0.258 -> 0.261).  Below 2 % the widest slice stays (d = 340M, 1.1 %: equal slices
// measured 0.4 % slower overall).  A vector short enough for a single round gets a multiple of
// 256 (more, narrower slices only add workgroups there), at least kMinSlice coordinates.
// No result depends on the width except the order of the fp64 sums of the SP pass.
// forced: the width asked for in efcp_options (0 = choose as described).
int32_t pick_slice_width(int64_t d, int32_t kb, int32_t forced)
{
    if (kb) return kCandBlock;
    if (forced) return forced;
    const int64_t widest = (d + kCandBlock - 1) / kCandBlock;
    const int64_t rounds = (widest + kMaxWgs - 1) / kMaxWgs;
    if ((rounds * kMaxWgs - widest) * 50 < rounds * kMaxWgs) return kCandBlock;
    const int64_t unit = rounds == 1 ? 256 : 64;
    int64_t w = (d + kMaxWgs * rounds - 1) / (kMaxWgs * rounds);
    w = (w + unit - 1) / unit * unit;
    if (w < kMinSlice) w = kMinSlice;
    if (w > kCandBlock) w = kCandBlock;
    return (int32_t)w;
}

// k_in: entries per row (topk_block == 0) or per block of kCandBlock coordinates.
bool make_geometry(int64_t d, int32_t m, int64_t k_in, int32_t fmt, int32_t topk_block, int32_t ggt,
                   int32_t slice_width, Geometry &g, const char **why)
{
    g.ggt = ggt ? 1 : 0;
    if (ggt != 0 && ggt != 1) { *why = "unknown preconditioner"; return false; }
    if (slice_width != 0 && (slice_width < 256 || slice_width > kCandBlock || slice_width % 64 != 0)) {
        *why = "slice_width must be 0 or a multiple of 64 in [256, 16384]";
        return false;
    }
    if (ggt && m > kGgtMaxM) { *why = "Sparse GGT: m out of range [1, 128]"; return false; }
    if (fmt != kFmtF32 && fmt != kFmtBf16) { *why = "unknown value format"; return false; }
    if (d < 1 || d >= ((int64_t)1 << 31)) { *why = "d out of range [1, 2^31)"; return false; }
    if (m < 1 || m > kMaxM) { *why = "m out of range [1, 1024]"; return false; }
    if (topk_block != 0 && topk_block != kCandBlock) { *why = "topk_block must be 0 or 16384"; return false; }
    int64_t k = k_in;
    g.kb = 0;
    if (topk_block) {
        if (k_in < 1 || k_in > kCandBlock) { *why = "k per block out of range [1, 16384]"; return false; }
        g.kb = (int32_t)k_in;
        k = block_row_length(d, k_in);
    }
    if (k < 1 || k > d) { *why = "k out of range [1, d]"; return false; }
    int dev = 0, lds = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess) {
        *why = "no HIP device";
        return false;
    }
    g.d = d; g.k = k; g.m = m; g.fmt = fmt;
    g.row_stride = (int64_t)align_up((size_t)k, 64);
    g.row_bytes = g.row_stride * (fmt == kFmtBf16 ? 4 : 6);
    g.ldm = (int32_t)align_up((size_t)m, 8);
    const size_t fixed_sp = 16 + 2 * kMaxM * sizeof(int32_t) + kMaxM * sizeof(double2) + 2 * 512 * sizeof(int32_t);
    const size_t fixed_lcg = 4 * kMaxM * sizeof(int32_t) + kMaxM * sizeof(double);
    const int lg = 14;                             // kCandBlock coordinates: 128 KiB of the 160 KiB LDS
    if (((size_t)8 << lg) + fixed_sp > (size_t)lds || ((size_t)8 << lg) + fixed_lcg > (size_t)lds) {
        *why = "device LDS too small (needs the 160 KiB of gfx950)";
        return false;
    }
    g.slice = pick_slice_width(d, g.kb, slice_width);
    g.n_slices = (int32_t)((d + g.slice - 1) / g.slice);
    {
        const int32_t per = (g.n_slices + 7) / 8;
        g.sp_grid = 8 * (per < kMaxWgs / 8 ? per : kMaxWgs / 8);
        // the SP kernel keeps two numbers per slice of a workgroup in a fixed piece of LDS
        if ((per + kMaxWgs / 8 - 1) / (kMaxWgs / 8) > 512) { *why = "slice width too small for this d"; return false; }
    }
    // A row has k / n_slices entries per slice on average.  The SP / LCG workgroups give a row 16
    // lanes (a batch of 192 entries) or, where that would leave nearly all of them idle, 4 lanes (48
    // entries): the workgroup then works on 256 rows at once instead of 64, and the dependent
    // batches per lane, which is what a small vector's passes consist of, fall by four.
    g.row_lanes = g.k / g.n_slices <= 40 ? 4 : 16;
    g.lds_sp = ((size_t)8 << lg) + fixed_sp;
    g.lds_lcg = ((size_t)8 << lg) + fixed_lcg;
    return true;
}

size_t value_bytes(const Geometry &g) { return g.fmt == kFmtBf16 ? 2 : 4; }
int group_entries(const Geometry &) { return 4; }
// Bytes of a row that hold its k entries (whole groups).
size_t row_payload_bytes(const Geometry &g)
{
    const size_t ge = (size_t)group_entries(g);
    return ((size_t)g.k + ge - 1) / ge * ge * (2 + value_bytes(g));
}

struct Layout {
    size_t e, ring, offT, S, W, partial, sq, zw, q, coef, rowmax, hist, sel, cnt_gt,
        cnt_eq, blk_gt, blk_eq, status, cand_idx, cand_val, cand_cnt, blk_max, blk_tlo, lam, rot,
        n_stages, col, step, total;
};

Layout make_layout(const Geometry &g)
{
    Layout l{};
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    l.ring = take((size_t)g.m * (size_t)g.row_bytes);
    l.partial = take((size_t)g.sp_grid * g.m * sizeof(double2));
    // candidate lists exist for the global Top-k only
    l.cand_idx = take(g.kb ? 0 : (size_t)g.n_slices * g.slice * sizeof(int32_t));
    l.cand_val = take(g.kb ? 0 : (size_t)g.n_slices * g.slice * sizeof(float));
    l.e = take((size_t)g.d * sizeof(float));
    l.offT = take((size_t)(g.n_slices + 1) * g.m * sizeof(int32_t));
    l.S = take((size_t)g.m * g.m * sizeof(double));
    l.W = take(g.ggt ? 0 : (size_t)g.m * g.ldm * sizeof(double));
    l.sq = take((size_t)g.m * sizeof(double2));
    l.zw = take((size_t)g.m * sizeof(double2));
    l.q = take((size_t)g.m * sizeof(double));
    l.coef = take((size_t)g.m * sizeof(double));
    l.rowmax = take((size_t)g.m * sizeof(uint32_t));
    l.hist = take((size_t)kHist1Copies * (kBins1 + 2 * kBins2) * sizeof(uint32_t));
    l.sel = take(sizeof(SelState));
    l.cnt_gt = take((size_t)g.n_slices * sizeof(uint32_t));
    l.cnt_eq = take((size_t)g.n_slices * sizeof(uint32_t));
    l.blk_gt = take((size_t)g.n_slices * sizeof(uint32_t));
    l.blk_eq = take((size_t)g.n_slices * sizeof(uint32_t));
    l.cand_cnt = take((size_t)g.n_slices * sizeof(uint32_t));
    l.blk_max = take(g.kb ? (size_t)g.n_slices * sizeof(uint32_t) : 0);
    l.blk_tlo = take(g.kb ? (size_t)g.n_slices * sizeof(uint32_t) : 0);
    l.lam = take(g.ggt ? (size_t)g.m * sizeof(double) : 0);
    l.rot = take(g.ggt ? (size_t)kGgtMaxSweeps * (kGgtMaxM - 1) * 64 * sizeof(double2) : 0);
    l.n_stages = take(g.ggt ? 256 : 0);
    l.col = take(((size_t)g.n_slices + 1) * sizeof(int32_t));
    l.status = take(256);
    l.step = take(sizeof(StepState));
    l.total = o;
    return l;
}

}  // namespace

// One column of the slice-major offset table, made contiguous for a copy to the host.
__global__ void k_offset_column(const int32_t *__restrict__ offT, int32_t m, int32_t slot, int32_t n,
                                int32_t *__restrict__ out)
{
    const int32_t s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s < n) out[s] = offT[(int64_t)s * m + slot];
}

// ---- scratch memory of efcp_apply_noalloc ----
// The buffers that efcp_apply takes from the context's workspace and only uses as scratch (the
// per-workgroup partial sums of the SP pass, their reduction sq, the product zw with the inverse
// factor, q and the coefficients) exist once more here, in the code object itself, for callers
// that want the context's own copies left alone.  Sized for the largest context the library
// creates: kMaxWgs workgroups x kMaxM rows of double2, and four m-sized arrays.  Every device
// that loads the library holds its own copy at its own address; host code must never use the
// name `scratch` as an address, only what hipGetSymbolAddress returned with that device current.
constexpr size_t kStaticPartialBytes = (size_t)kMaxWgs * kMaxM * sizeof(double2);
constexpr size_t kStaticSmallBytes = (size_t)kMaxM * sizeof(double2);
constexpr size_t kStaticScratchBytes = kStaticPartialBytes + 4 * kStaticSmallBytes;     // 4 MiB + 64 KiB
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];            // device address of `scratch` on each device, once resolved

// Address of `scratch` on `device`, which must be current.
hipError_t static_scratch_address(int device, void **ptr)
{
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (device >= 0 && device < kMaxDevices && g_scratch_ptr[device]) {
        *ptr = g_scratch_ptr[device];
        return hipSuccess;
    }
    void *at = nullptr;
    const hipError_t rc = hipGetSymbolAddress(&at, HIP_SYMBOL(scratch));
    if (rc != hipSuccess) return rc;
    if (!at) return hipErrorInvalidSymbol;
    if (device >= 0 && device < kMaxDevices) g_scratch_ptr[device] = at;
    *ptr = at;
    return hipSuccess;
}

}  // namespace

struct efcp_ctx {
    Geometry g;
    DevicePtrs p;
    void *static_scratch;            // this device's copy of `scratch` (resolved in efcp_create)
    double lambda;
    int device;
    void *ws;
    size_t ws_bytes;
    bool own_ws;
    // The step count and the slot whose row is still to be taken out of e live in device memory
    // (p.step) and are advanced by the step's kernels; host code reads them only in the
    // inspection calls, after synchronising.
    bool broken;                     // a launch failed part-way: the state is undefined
    bool single_stream;              // the eviction update runs on the caller's stream (no fork)
    hipStream_t last_stream;
    // The eviction update of the inverse factor depends on the previous step only; it runs on
    // this stream next to the d-sized passes of the step and is joined before k_fwd.
    hipStream_t side;
    hipEvent_t ev_fork, ev_join;
    const char *err;
    // profiling
    bool prof_on;
    std::vector<hipEvent_t> ev;      // kProfSteps * kProfEvents
    int prof_count;                  // steps recorded since the last read
};

static int fail(efcp_ctx *ctx, int code, const char *msg)
{
    if (ctx) ctx->err = msg;
    return code;
}

// Every call on a context needs the device it was created on to be current: its memory, side
// stream and events live there.
static int wrong_device(efcp_ctx *ctx)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return fail(ctx, EFCP_EHIP, "no current HIP device");
    if (dev != ctx->device) return fail(ctx, EFCP_EINVAL, "the device of efcp_create is not current");
    return EFCP_OK;
}

static efcp_options options_of(int32_t value_format, int32_t topk_block, int32_t preconditioner)
{
    efcp_options o;
    o.value_format = value_format;
    o.topk_block = topk_block;
    o.preconditioner = preconditioner;
    o.slice_width = 0;
    o.single_stream = 0;
    return o;
}

extern "C" size_t efcp_workspace_bytes_opts(int64_t d, int32_t m, int64_t k, const efcp_options *opts)
{
    const efcp_options o = opts ? *opts : options_of(EFCP_VALUES_FP32, 0, EFCP_SPARSE_MFAC);
    Geometry g;
    const char *why = "";
    if (!make_geometry(d, m, k, o.value_format, o.topk_block, o.preconditioner, o.slice_width, g, &why)) return 0;
    return make_layout(g).total;
}

extern "C" size_t efcp_workspace_bytes_ex(int64_t d, int32_t m, int64_t k, int32_t value_format,
                                          int32_t topk_block)
{
    const efcp_options o = options_of(value_format, topk_block, EFCP_SPARSE_MFAC);
    return efcp_workspace_bytes_opts(d, m, k, &o);
}

extern "C" size_t efcp_workspace_bytes_ggt(int64_t d, int32_t m, int64_t k, int32_t value_format,
                                           int32_t topk_block)
{
    const efcp_options o = options_of(value_format, topk_block, EFCP_SPARSE_GGT);
    return efcp_workspace_bytes_opts(d, m, k, &o);
}

extern "C" size_t efcp_workspace_bytes_fmt(int64_t d, int32_t m, int64_t k, int32_t value_format)
{
    return efcp_workspace_bytes_ex(d, m, k, value_format, 0);
}

extern "C" int32_t efcp_default_slice_width(int64_t d, int32_t topk_block)
{
    if (d < 1 || d >= ((int64_t)1 << 31) || (topk_block != 0 && topk_block != kCandBlock)) return 0;
    return pick_slice_width(d, topk_block ? 1 : 0, 0);
}

extern "C" int64_t efcp_row_length(int64_t d, int64_t k, int32_t topk_block)
{
    if (topk_block == 0) return (k >= 1 && k <= d) ? k : 0;
    if (topk_block != kCandBlock || d < 1 || k < 1 || k > kCandBlock) return 0;
    return block_row_length(d, k);
}

extern "C" size_t efcp_workspace_bytes(int64_t d, int32_t m, int64_t k)
{
    return efcp_workspace_bytes_fmt(d, m, k, EFCP_VALUES_FP32);
}

extern "C" int efcp_create(efcp_ctx **out, int64_t d, int32_t m, int64_t k, double lambda,
                           void *workspace, size_t workspace_bytes)
{
    return efcp_create_fmt(out, d, m, k, lambda, EFCP_VALUES_FP32, workspace, workspace_bytes);
}

extern "C" int efcp_create_fmt(efcp_ctx **out, int64_t d, int32_t m, int64_t k, double lambda,
                               int32_t value_format, void *workspace, size_t workspace_bytes)
{
    return efcp_create_ex(out, d, m, k, lambda, value_format, 0, workspace, workspace_bytes);
}

extern "C" int efcp_create_ex(efcp_ctx **out, int64_t d, int32_t m, int64_t k, double lambda,
                              int32_t value_format, int32_t topk_block, void *workspace,
                              size_t workspace_bytes)
{
    const efcp_options o = options_of(value_format, topk_block, EFCP_SPARSE_MFAC);
    return efcp_create_opts(out, d, m, k, lambda, &o, workspace, workspace_bytes);
}

extern "C" int efcp_create_ggt(efcp_ctx **out, int64_t d, int32_t m, int64_t k, double epsilon,
                               int32_t value_format, int32_t topk_block, void *workspace,
                               size_t workspace_bytes)
{
    const efcp_options o = options_of(value_format, topk_block, EFCP_SPARSE_GGT);
    return efcp_create_opts(out, d, m, k, epsilon, &o, workspace, workspace_bytes);
}

extern "C" int efcp_create_opts(efcp_ctx **out, int64_t d, int32_t m, int64_t k, double lambda,
                                const efcp_options *opts, void *workspace, size_t workspace_bytes)
{
    const efcp_options o = opts ? *opts : options_of(EFCP_VALUES_FP32, 0, EFCP_SPARSE_MFAC);
    const int32_t value_format = o.value_format, topk_block = o.topk_block, ggt = o.preconditioner;

    if (!out) return EFCP_EINVAL;
    *out = nullptr;
    if (!(lambda > 0.0) || !std::isfinite(lambda)) return EFCP_EINVAL;
    Geometry g;
    const char *why = "";
    if (!make_geometry(d, m, k, value_format, topk_block, ggt, o.slice_width, g, &why)) return EFCP_EINVAL;
    const Layout l = make_layout(g);

    efcp_ctx *ctx = new (std::nothrow) efcp_ctx();
    if (!ctx) return EFCP_ENOMEM;
    ctx->g = g;
    ctx->lambda = lambda;
    ctx->broken = false;
    ctx->single_stream = o.single_stream != 0;
    ctx->last_stream = nullptr;
    ctx->err = "no error";
    ctx->prof_on = false;
    ctx->prof_count = 0;
    if (hipGetDevice(&ctx->device) != hipSuccess) { delete ctx; return EFCP_EHIP; }

    if (workspace) {
        if (workspace_bytes < l.total || (reinterpret_cast<uintptr_t>(workspace) & 255)) {
            delete ctx;
            return workspace_bytes < l.total ? EFCP_ENOMEM : EFCP_EINVAL;
        }
        ctx->ws = workspace;
        ctx->own_ws = false;
    } else {
        if (hipMalloc(&ctx->ws, l.total) != hipSuccess) {
            (void)hipGetLastError();
            delete ctx;
            return EFCP_ENOMEM;
        }
        ctx->own_ws = true;
    }
    ctx->ws_bytes = l.total;

    unsigned char *b = static_cast<unsigned char *>(ctx->ws);
    DevicePtrs &p = ctx->p;
    p.e = reinterpret_cast<float *>(b + l.e);
    p.ring = b + l.ring;
    p.offT = reinterpret_cast<int32_t *>(b + l.offT);
    p.S = reinterpret_cast<double *>(b + l.S);
    p.W = reinterpret_cast<double *>(b + l.W);
    p.partial = reinterpret_cast<double2 *>(b + l.partial);
    p.sq = reinterpret_cast<double2 *>(b + l.sq);
    p.zw = reinterpret_cast<double2 *>(b + l.zw);
    p.q = reinterpret_cast<double *>(b + l.q);
    p.coef = reinterpret_cast<double *>(b + l.coef);
    p.rowmax = reinterpret_cast<uint32_t *>(b + l.rowmax);
    p.hist1 = reinterpret_cast<uint32_t *>(b + l.hist);
    p.hist2 = p.hist1 + kHist1Copies * kBins1;
    p.hist3 = p.hist2 + kHist1Copies * kBins2;
    p.sel = reinterpret_cast<SelState *>(b + l.sel);
    p.cnt_gt = reinterpret_cast<uint32_t *>(b + l.cnt_gt);
    p.cnt_eq = reinterpret_cast<uint32_t *>(b + l.cnt_eq);
    p.blk_gt = reinterpret_cast<uint32_t *>(b + l.blk_gt);
    p.blk_eq = reinterpret_cast<uint32_t *>(b + l.blk_eq);
    p.cand_idx = reinterpret_cast<int32_t *>(b + l.cand_idx);
    p.cand_val = reinterpret_cast<float *>(b + l.cand_val);
    p.cand_cnt = reinterpret_cast<uint32_t *>(b + l.cand_cnt);
    p.blk_max = reinterpret_cast<uint32_t *>(b + l.blk_max);
    p.blk_tlo = reinterpret_cast<uint32_t *>(b + l.blk_tlo);
    p.lam = reinterpret_cast<double *>(b + l.lam);
    p.rot = reinterpret_cast<double2 *>(b + l.rot);
    p.n_stages = reinterpret_cast<int32_t *>(b + l.n_stages);
    p.col = reinterpret_cast<int32_t *>(b + l.col);
    p.status = reinterpret_cast<uint32_t *>(b + l.status);
    p.step = reinterpret_cast<StepState *>(b + l.step);

    // Everything starts as zero bytes: e = 0, offsets, Gram matrix, factor, histograms, counters,
    // and the ring too: the SP pass multiplies entries that lie outside a run (other slices' entries,
    // or the unused tail of a row's last group) by zero, so they must be finite numbers, never
    // whatever the memory held before.
    hipError_t rc = hipMemset(b, 0, l.total);
    const StepState first_state = {0, -1, 0};              // no step done, e is final
    if (rc == hipSuccess) rc = hipMemcpy(p.step, &first_state, sizeof first_state, hipMemcpyHostToDevice);
    ctx->side = nullptr;
    ctx->ev_fork = ctx->ev_join = nullptr;
    if (rc == hipSuccess && !ctx->single_stream) rc = hipStreamCreateWithFlags(&ctx->side, hipStreamNonBlocking);
    if (rc == hipSuccess) rc = hipEventCreateWithFlags(&ctx->ev_fork, hipEventDisableTiming);
    if (rc == hipSuccess) rc = hipEventCreateWithFlags(&ctx->ev_join, hipEventDisableTiming);
    ctx->static_scratch = nullptr;
    if (rc == hipSuccess) rc = static_scratch_address(ctx->device, &ctx->static_scratch);
    if (rc == hipSuccess) rc = configure_sp(g);
    if (rc == hipSuccess) rc = configure_lcg(g);
    if (rc == hipSuccess && g.ggt) rc = configure_ggt();
    if (rc == hipSuccess) rc = hipDeviceSynchronize();
    if (rc != hipSuccess) {
        (void)hipGetLastError();
        if (ctx->ev_fork) (void)hipEventDestroy(ctx->ev_fork);
        if (ctx->ev_join) (void)hipEventDestroy(ctx->ev_join);
        if (ctx->side) (void)hipStreamDestroy(ctx->side);
        if (ctx->own_ws) (void)hipFree(ctx->ws);
        delete ctx;
        return EFCP_EHIP;
    }
    *out = ctx;
    return EFCP_OK;
}

extern "C" int efcp_step(efcp_ctx *ctx, const float *grad, float *outp, void *stream_v)
{
    return efcp_step_ex(ctx, grad, EFCP_X_GRAD, outp, nullptr, 0.0, 0.0, stream_v);
}

static bool overlap(const void *a, const void *b, size_t bytes)
{
    const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
    return a && b && x < y + bytes && y < x + bytes;
}

extern "C" int efcp_step_ex(efcp_ctx *ctx, const float *grad, int32_t x_source, float *outp, float *param,
                            double lr, double weight_decay, void *stream_v)
{
    if (!ctx) return EFCP_EINVAL;
    if (int rc = wrong_device(ctx)) return rc;
    if (!grad) return fail(ctx, EFCP_EINVAL, "grad is NULL");
    if (x_source != EFCP_X_GRAD && x_source != EFCP_X_COMPRESSED)
        return fail(ctx, EFCP_EINVAL, "unknown x_source");
    if (outp && param) return fail(ctx, EFCP_EINVAL, "give out or param, not both");
    if (param && !(std::isfinite(lr) && std::isfinite(weight_decay)))
        return fail(ctx, EFCP_EINVAL, "lr / weight_decay not finite");
    float *dst = param ? param : outp;
    if ((reinterpret_cast<uintptr_t>(grad) & 15) || (reinterpret_cast<uintptr_t>(dst) & 15))
        return fail(ctx, EFCP_EINVAL, "grad/out/param not 16-byte aligned");
    const size_t bytes = (size_t)ctx->g.d * sizeof(float);
    if (overlap(grad, dst, bytes)) return fail(ctx, EFCP_EINVAL, "grad and out/param overlap");

    if (ctx->broken) return fail(ctx, EFCP_EHIP, "an earlier launch failed: the context can only be destroyed or re-imported");

    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    const Geometry &g = ctx->g;
    const DevicePtrs &p = ctx->p;
    const bool x_is_row = x_source == EFCP_X_COMPRESSED;
    // Nothing below depends on the step number: slot, rows filled and "does this step evict" are
    // read by the kernels from p.step, which the reduction after the SP pass advances.  The same
    // sequence of launches is therefore every step of the context (and a HIP graph captured
    // from it can be replayed as the following steps).
    const bool factor = !g.ggt;                          // Sparse GGT keeps no factor to update

    hipEvent_t *ev = nullptr;
    if (ctx->prof_on) ev = &ctx->ev[(size_t)(ctx->prof_count % kProfSteps) * kProfEvents];
    hipError_t rc = hipSuccess;
    auto mark = [&](int i) { if (ev && rc == hipSuccess) rc = hipEventRecord(ev[i], stream); };

    // Deleting the oldest row from the inverse factor (nothing happens until the window is full)
    // depends on nothing in this step.  With the global Top-k it rides in the first kernel of the
    // selection.  With Top-k in blocks it is a kernel of its own, on the side stream while the
    // d-sized passes run, or in line when the context keeps to one stream.
    const bool fork = factor && g.kb && !ctx->single_stream;
    if (factor && g.kb && !fork) {
        if (rc == hipSuccess) rc = launch_evict(g, p, stream);
    }
    if (fork) {
        if (rc == hipSuccess) rc = hipEventRecord(ctx->ev_fork, stream);
        if (rc == hipSuccess) rc = hipStreamWaitEvent(ctx->side, ctx->ev_fork, 0);
        if (rc == hipSuccess) rc = launch_evict(g, p, ctx->side);
        if (rc == hipSuccess) rc = hipEventRecord(ctx->ev_join, ctx->side);
    }
    mark(0);
    if (g.kb) {         // Top-k in blocks: error feedback, selection and compaction in one kernel
        if (rc == hipSuccess) rc = launch_block_topk(g, p, grad, stream);
        mark(1);
        mark(2);
    } else {
        if (rc == hipSuccess) rc = launch_ef_hist(g, p, grad, stream);
        mark(1);
        if (rc == hipSuccess) rc = launch_select(g, p, factor, stream);
        mark(2);
        if (rc == hipSuccess) rc = launch_compact(g, p, stream);
    }
    mark(3);
    if (rc == hipSuccess) rc = launch_sp(g, p, grad, x_is_row ? 1 : 0, stream);
    mark(4);
    // join before the reduction: it counts the step, and the eviction kernel reads the old count
    if (fork && rc == hipSuccess) rc = hipStreamWaitEvent(stream, ctx->ev_join, 0);
    if (rc == hipSuccess) rc = launch_sp_reduce(g, p, true, stream);
    if (rc == hipSuccess)
        rc = g.ggt ? launch_ggt_step(g, p, ctx->lambda, stream) : launch_coef(g, p, ctx->lambda, stream);
    mark(5);
    if (rc == hipSuccess && dst) {
        LcgMode md;
        md.x_is_newest_row = x_is_row;
        md.update = param != nullptr;
        md.lr = lr;
        md.decay = 1.0 - lr * weight_decay;
        rc = launch_lcg(g, p, grad, dst, ctx->lambda, md, stream);
    }
    mark(6);

    ctx->last_stream = stream;
    if (rc != hipSuccess) {
        ctx->broken = true;
        return fail(ctx, EFCP_EHIP, hipGetErrorString(rc));
    }
    if (ctx->prof_on) ctx->prof_count++;
    return EFCP_OK;
}

// p: the context's pointers, or a copy of them whose scratch members point somewhere else.
static int apply_impl(efcp_ctx *ctx, const DevicePtrs &p, const float *x, float *outp, void *stream_v)
{
    if ((reinterpret_cast<uintptr_t>(x) & 15) || (reinterpret_cast<uintptr_t>(outp) & 15))
        return fail(ctx, EFCP_EINVAL, "x/out not 16-byte aligned");
    if (overlap(x, outp, (size_t)ctx->g.d * sizeof(float))) return fail(ctx, EFCP_EINVAL, "x and out overlap");
    if (ctx->broken) return fail(ctx, EFCP_EHIP, "an earlier launch failed: the context can only be destroyed or re-imported");
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    const Geometry &g = ctx->g;
    hipError_t rc = hipSuccess;
    if (ctx->last_stream != stream && ctx->last_stream != nullptr) {
        // the window was written on another stream: order this call after it
        rc = hipEventRecord(ctx->ev_fork, ctx->last_stream);
        if (rc == hipSuccess) rc = hipStreamWaitEvent(stream, ctx->ev_fork, 0);
    }
    // the kernels take the number of filled rows from p.step; with an empty window they move no
    // row and the result is x/lambda
    if (rc == hipSuccess) rc = launch_sp(g, p, x, 2, stream);
    if (rc == hipSuccess) rc = launch_sp_reduce(g, p, false, stream);
    if (rc == hipSuccess)
        rc = g.ggt ? launch_ggt_apply(g, p, ctx->lambda, stream) : launch_coef_apply(g, p, ctx->lambda, stream);
    if (rc == hipSuccess) rc = launch_lcg(g, p, x, outp, ctx->lambda, LcgMode{}, stream);
    ctx->last_stream = stream;
    if (rc != hipSuccess) return fail(ctx, EFCP_EHIP, hipGetErrorString(rc));
    return EFCP_OK;
}

extern "C" int efcp_apply(efcp_ctx *ctx, const float *x, float *outp, void *stream_v)
{
    if (!ctx) return EFCP_EINVAL;
    if (int rc = wrong_device(ctx)) return rc;
    if (!x || !outp) return fail(ctx, EFCP_EINVAL, "x or out is NULL");
    return apply_impl(ctx, ctx->p, x, outp, stream_v);
}

extern "C" int efcp_apply_noalloc(efcp_ctx *ctx, const float *x, float *outp, void *stream_v)
{
    if (!ctx) return EFCP_EINVAL;
    if (int rc = wrong_device(ctx)) return rc;
    if (!x || !outp) return fail(ctx, EFCP_EINVAL, "x or out is NULL");
    const Geometry &g = ctx->g;
    const size_t partial_bytes = (size_t)g.sp_grid * g.m * sizeof(double2);
    const size_t small_bytes = (size_t)g.m * sizeof(double2);
    if (partial_bytes > kStaticPartialBytes || small_bytes > kStaticSmallBytes)
        return fail(ctx, EFCP_EINVAL, "window too large for the static scratch (256 workgroups x 1024 rows)");
    if (!ctx->static_scratch) return fail(ctx, EFCP_EHIP, "static scratch address was not resolved");
    unsigned char *b = static_cast<unsigned char *>(ctx->static_scratch);
    DevicePtrs p = ctx->p;
    p.partial = reinterpret_cast<double2 *>(b);
    p.sq = reinterpret_cast<double2 *>(b + kStaticPartialBytes);
    p.zw = reinterpret_cast<double2 *>(b + kStaticPartialBytes + kStaticSmallBytes);
    p.q = reinterpret_cast<double *>(b + kStaticPartialBytes + 2 * kStaticSmallBytes);
    p.coef = reinterpret_cast<double *>(b + kStaticPartialBytes + 3 * kStaticSmallBytes);
    return apply_impl(ctx, p, x, outp, stream_v);
}

extern "C" int efcp_destroy(efcp_ctx *ctx)
{
    if (!ctx) return EFCP_OK;
    int rcode = EFCP_OK;
    // the context's device is made current for the clean-up and the caller's restored afterwards
    int cur = ctx->device;
    (void)hipGetDevice(&cur);
    if (cur != ctx->device && hipSetDevice(ctx->device) != hipSuccess) rcode = EFCP_EHIP;
    if (hipDeviceSynchronize() != hipSuccess) rcode = EFCP_EHIP;
    for (hipEvent_t e : ctx->ev) (void)hipEventDestroy(e);
    (void)hipEventDestroy(ctx->ev_fork);
    (void)hipEventDestroy(ctx->ev_join);
    if (ctx->side) (void)hipStreamDestroy(ctx->side);
    if (ctx->own_ws && hipFree(ctx->ws) != hipSuccess) rcode = EFCP_EHIP;
    if (cur != ctx->device) (void)hipSetDevice(cur);
    delete ctx;
    return rcode;
}

static int sync_last(efcp_ctx *ctx)
{
    if (hipStreamSynchronize(ctx->last_stream) != hipSuccess)
        return fail(ctx, EFCP_EHIP, "stream synchronisation failed");
    return EFCP_OK;
}

// The step state as the device holds it, after the stream of the last call has drained.
static int read_step_state(efcp_ctx *ctx, StepState &st)
{
    if (int rc = sync_last(ctx)) return rc;
    if (hipMemcpy(&st, ctx->p.step, sizeof st, hipMemcpyDeviceToHost) != hipSuccess)
        return fail(ctx, EFCP_EHIP, "copy to host failed");
    return EFCP_OK;
}

static int64_t rows_filled(const efcp_ctx *ctx, const StepState &st)
{
    return st.t_done < ctx->g.m ? st.t_done : ctx->g.m;
}

extern "C" int efcp_get_row(efcp_ctx *ctx, int32_t slot, int32_t *idx_host, float *val_host)
{
    if (!ctx || !idx_host || !val_host) return EFCP_EINVAL;
    if (int rc = wrong_device(ctx)) return rc;
    const Geometry &g = ctx->g;
    StepState now;
    if (int rc = read_step_state(ctx, now)) return rc;
    if (slot < 0 || slot >= rows_filled(ctx, now)) return fail(ctx, EFCP_EINVAL, "slot not filled");
    // the row's groups ([indices][values]) and its slice offsets; 16-bit in-slice indices become
    // absolute with the offsets
    const size_t ge = (size_t)group_entries(g), vb = value_bytes(g), gb = ge * (2 + vb);
    std::vector<unsigned char> raw(row_payload_bytes(g));
    std::vector<int32_t> offs((size_t)g.n_slices + 1);
    hipLaunchKernelGGL(k_offset_column, dim3((g.n_slices + 1 + 255) / 256), dim3(256), 0, ctx->last_stream,
                       ctx->p.offT, g.m, slot, g.n_slices + 1, ctx->p.col);
    if (hipGetLastError() != hipSuccess || hipStreamSynchronize(ctx->last_stream) != hipSuccess ||
        hipMemcpy(raw.data(), ctx->p.ring + (size_t)slot * (size_t)g.row_bytes, raw.size(),
                  hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemcpy(offs.data(), ctx->p.col, ((size_t)g.n_slices + 1) * sizeof(int32_t),
                  hipMemcpyDeviceToHost) != hipSuccess)
        return fail(ctx, EFCP_EHIP, "copy to host failed");
    auto stored_index = [&](int64_t p) {
        uint16_t v;
        std::memcpy(&v, raw.data() + (size_t)(p / (int64_t)ge) * gb + 2 * (size_t)(p % (int64_t)ge), 2);
        return (int32_t)v;
    };
    for (int32_t s = 0; s < g.n_slices; s++) {
        const int32_t base = s * g.slice;
        for (int32_t p = offs[s]; p < offs[s + 1]; p++) idx_host[p] = base + stored_index(p);
    }
    for (int64_t p = 0; p < g.k; p++) {
        const unsigned char *at = raw.data() + (size_t)(p / (int64_t)ge) * gb + 2 * ge + vb * (size_t)(p % (int64_t)ge);
        if (g.fmt == kFmtF32) {
            std::memcpy(&val_host[p], at, 4);
        } else {
            uint16_t hb;
            std::memcpy(&hb, at, 2);
            const uint32_t bits = (uint32_t)hb << 16;
            std::memcpy(&val_host[p], &bits, 4);
        }
    }
    return EFCP_OK;
}

// e = a - c for a copy of the device buffer that still holds a at the entries of the newest row.
static int settle_error(efcp_ctx *ctx, float *e_host)
{
    StepState now;
    if (int rc = read_step_state(ctx, now)) return rc;
    if (now.pend_slot < 0) return EFCP_OK;
    const Geometry &g = ctx->g;
    std::vector<int32_t> idx((size_t)g.k);
    std::vector<float> val((size_t)g.k);
    if (int rc = efcp_get_row(ctx, now.pend_slot, idx.data(), val.data())) return rc;
    for (int64_t p = 0; p < g.k; p++) {
        float &ej = e_host[idx[(size_t)p]];
        ej = ej - val[(size_t)p];                 // ej is a, val the stored a or bf16(a): +0 or the remainder
    }
    return EFCP_OK;
}

extern "C" int efcp_get_error(efcp_ctx *ctx, float *e_host)
{
    if (!ctx || !e_host) return EFCP_EINVAL;
    if (int rc = wrong_device(ctx)) return rc;
    if (int rc = sync_last(ctx)) return rc;
    if (hipMemcpy(e_host, ctx->p.e, (size_t)ctx->g.d * 4, hipMemcpyDeviceToHost) != hipSuccess)
        return fail(ctx, EFCP_EHIP, "copy to host failed");
    return settle_error(ctx, e_host);
}

extern "C" int efcp_get_small(efcp_ctx *ctx, double *S_host, double *q_host, double *coef_host,
                              uint32_t *tau, int64_t *step)
{
    if (!ctx) return EFCP_EINVAL;
    if (int rc = wrong_device(ctx)) return rc;
    StepState now;
    if (int rc = read_step_state(ctx, now)) return rc;
    const Geometry &g = ctx->g;
    hipError_t rc = hipSuccess;
    if (S_host) rc = hipMemcpy(S_host, ctx->p.S, (size_t)g.m * g.m * 8, hipMemcpyDeviceToHost);
    if (rc == hipSuccess && q_host) rc = hipMemcpy(q_host, ctx->p.q, (size_t)g.m * 8, hipMemcpyDeviceToHost);
    if (rc == hipSuccess && coef_host)
        rc = hipMemcpy(coef_host, ctx->p.coef, (size_t)g.m * 8, hipMemcpyDeviceToHost);
    SelState st;
    uint32_t status = 0;
    if (rc == hipSuccess) rc = hipMemcpy(&st, ctx->p.sel, sizeof st, hipMemcpyDeviceToHost);
    if (rc == hipSuccess) rc = hipMemcpy(&status, ctx->p.status, 4, hipMemcpyDeviceToHost);
    if (rc != hipSuccess) return fail(ctx, EFCP_EHIP, "copy to host failed");
    if (tau) *tau = st.tau;
    if (step) *step = now.t_done;
    if (status & kStatusCount) return fail(ctx, EFCP_EHIP, "selection wrote a row whose length is not k");
    if (status & kStatusRange) return fail(ctx, EFCP_ENUMERIC, "coefficients are not finite");
    if (status & kStatusPivot) return fail(ctx, EFCP_ENUMERIC, "non-positive pivot in the factor update");
    return EFCP_OK;
}

// ---------------------------------------------------------------- checkpoint

namespace {

struct StateHeader {
    uint64_t magic;          // "EFCPST05"
    int64_t d, k, row_stride, t;
    int32_t m, ldm, slice, n_slices;
    double lambda;
    uint32_t t_lo, status;
    int32_t filled, fmt;
    int32_t kb, ggt;
};
constexpr uint64_t kStateMagic = 0x3530545350434645ull;

size_t state_bytes(const efcp_ctx *ctx, int64_t t_done)
{
    const Geometry &g = ctx->g;
    const size_t filled = (size_t)(t_done < g.m ? t_done : g.m);
    return sizeof(StateHeader) + (size_t)g.d * 4 + filled * row_payload_bytes(g) +
           (size_t)(g.n_slices + 1) * g.m * 4 + (size_t)g.m * g.m * 8 +
           (g.ggt ? 0 : (size_t)g.m * g.ldm * 8) + (size_t)g.m * 4;
}

}  // namespace

extern "C" size_t efcp_state_bytes(efcp_ctx *ctx)
{
    if (!ctx || wrong_device(ctx) != EFCP_OK) return 0;
    StepState now;
    if (read_step_state(ctx, now) != EFCP_OK) return 0;
    return state_bytes(ctx, now.t_done);
}

extern "C" int efcp_export_state(efcp_ctx *ctx, void *host_buf, size_t bytes)
{
    if (!ctx || !host_buf) return EFCP_EINVAL;
    if (int rc = wrong_device(ctx)) return rc;
    StepState now;
    if (int rc = read_step_state(ctx, now)) return rc;
    if (bytes < state_bytes(ctx, now.t_done)) return fail(ctx, EFCP_ENOMEM, "state buffer too small");
    if (reinterpret_cast<uintptr_t>(host_buf) & 7) return fail(ctx, EFCP_EINVAL, "state buffer not 8-byte aligned");
    const Geometry &g = ctx->g;
    const DevicePtrs &p = ctx->p;
    SelState st;
    uint32_t status = 0;
    if (hipMemcpy(&st, p.sel, sizeof st, hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemcpy(&status, p.status, 4, hipMemcpyDeviceToHost) != hipSuccess)
        return fail(ctx, EFCP_EHIP, "copy to host failed");
    StateHeader h{};
    h.magic = kStateMagic;
    h.d = g.d; h.k = g.k; h.row_stride = g.row_stride; h.t = now.t_done;
    h.m = g.m; h.ldm = g.ldm; h.slice = g.slice; h.n_slices = g.n_slices;
    h.lambda = ctx->lambda;
    h.t_lo = st.t_lo; h.status = status;
    h.filled = (int32_t)rows_filled(ctx, now);
    h.fmt = g.fmt;
    h.kb = g.kb;
    h.ggt = g.ggt;
    unsigned char *o = static_cast<unsigned char *>(host_buf);
    std::memcpy(o, &h, sizeof h);
    o += sizeof h;
    hipError_t rc = hipSuccess;
    auto pull = [&](const void *dev, size_t n) {
        if (rc == hipSuccess) rc = hipMemcpy(o, dev, n, hipMemcpyDeviceToHost);
        o += n;
    };
    float *e_blob = reinterpret_cast<float *>(o);
    pull(p.e, (size_t)g.d * 4);
    if (rc == hipSuccess && settle_error(ctx, e_blob) != EFCP_OK) return EFCP_EHIP;
    for (int32_t r = 0; r < h.filled; r++) {
        pull(p.ring + (size_t)r * (size_t)g.row_bytes, row_payload_bytes(g));
    }
    pull(p.offT, (size_t)(g.n_slices + 1) * g.m * 4);
    pull(p.S, (size_t)g.m * g.m * 8);
    if (!g.ggt) pull(p.W, (size_t)g.m * g.ldm * 8);
    pull(p.rowmax, (size_t)g.m * 4);
    if (rc != hipSuccess) return fail(ctx, EFCP_EHIP, "copy to host failed");
    return EFCP_OK;
}

extern "C" int efcp_import_state(efcp_ctx *ctx, const void *host_buf, size_t bytes)
{
    if (!ctx || !host_buf) return EFCP_EINVAL;
    if (int rc = wrong_device(ctx)) return rc;
    if (bytes < sizeof(StateHeader)) return fail(ctx, EFCP_EINVAL, "state buffer truncated");
    StateHeader h;
    std::memcpy(&h, host_buf, sizeof h);
    const Geometry &g = ctx->g;
    if (h.magic != kStateMagic || h.d != g.d || h.k != g.k || h.m != g.m || h.row_stride != g.row_stride ||
        h.ldm != g.ldm || h.slice != g.slice || h.n_slices != g.n_slices || h.lambda != ctx->lambda ||
        h.fmt != g.fmt || h.kb != g.kb || h.ggt != g.ggt ||
        h.t < 0 || h.filled != (int32_t)(h.t < g.m ? h.t : g.m))
        return fail(ctx, EFCP_EINVAL, "state does not belong to a context of this shape");
    if (bytes < state_bytes(ctx, h.t)) return fail(ctx, EFCP_EINVAL, "state buffer truncated");
    if (hipDeviceSynchronize() != hipSuccess) return fail(ctx, EFCP_EHIP, "sync failed");
    const DevicePtrs &p = ctx->p;
    const unsigned char *o = static_cast<const unsigned char *>(host_buf) + sizeof h;
    hipError_t rc = hipSuccess;
    auto push = [&](void *dev, size_t n) {
        if (rc == hipSuccess) rc = hipMemcpy(dev, o, n, hipMemcpyHostToDevice);
        o += n;
    };
    push(p.e, (size_t)g.d * 4);
    for (int32_t r = 0; r < h.filled; r++) {
        push(p.ring + (size_t)r * (size_t)g.row_bytes, row_payload_bytes(g));
    }
    push(p.offT, (size_t)(g.n_slices + 1) * g.m * 4);
    push(p.S, (size_t)g.m * g.m * 8);
    if (!g.ggt) push(p.W, (size_t)g.m * g.ldm * 8);
    push(p.rowmax, (size_t)g.m * 4);
    SelState st{};
    st.t_lo = h.t_lo;
    if (rc == hipSuccess) rc = hipMemcpy(p.sel, &st, sizeof st, hipMemcpyHostToDevice);
    if (rc == hipSuccess) rc = hipMemcpy(p.status, &h.status, 4, hipMemcpyHostToDevice);
    const StepState imported = {h.t, -1, 0};         // an exported e is final: nothing is pending
    if (rc == hipSuccess) rc = hipMemcpy(p.step, &imported, sizeof imported, hipMemcpyHostToDevice);
    if (rc == hipSuccess) rc = hipMemset(p.hist1, 0, (size_t)kHist1Copies * (kBins1 + 2 * kBins2) * sizeof(uint32_t));
    // where each block starts counting is a hint only: start from "count everything"
    if (rc == hipSuccess && g.kb) rc = hipMemset(p.blk_tlo, 0, (size_t)g.n_slices * sizeof(uint32_t));
    // Sparse GGT: the decomposition that efcp_apply replays is rebuilt from the imported S
    if (rc == hipSuccess && g.ggt && h.filled > 0) rc = launch_ggt_refresh(g, p, nullptr);
    if (rc == hipSuccess) rc = hipDeviceSynchronize();
    if (rc != hipSuccess) {
        ctx->broken = true;
        return fail(ctx, EFCP_EHIP, "copy to device failed");
    }
    ctx->broken = false;                             // a complete state replaces whatever was there
    return EFCP_OK;
}

extern "C" int efcp_get_geometry(efcp_ctx *ctx, int32_t *slice, int32_t *n_slices, int64_t *row_stride)
{
    if (!ctx) return EFCP_EINVAL;
    if (slice) *slice = ctx->g.slice;
    if (n_slices) *n_slices = ctx->g.n_slices;
    if (row_stride) *row_stride = ctx->g.row_stride;
    return EFCP_OK;
}

extern "C" int efcp_profile_enable(efcp_ctx *ctx, int enable)
{
    if (!ctx) return EFCP_EINVAL;
    ctx->prof_count = 0;
    if (!enable) { ctx->prof_on = false; return EFCP_OK; }
    if (ctx->ev.empty()) {
        ctx->ev.reserve((size_t)kProfSteps * kProfEvents);
        for (int i = 0; i < kProfSteps * kProfEvents; i++) {
            hipEvent_t e;
            if (hipEventCreate(&e) != hipSuccess) return fail(ctx, EFCP_EHIP, "hipEventCreate failed");
            ctx->ev.push_back(e);
        }
    }
    ctx->prof_on = true;
    return EFCP_OK;
}

extern "C" int efcp_profile_read(efcp_ctx *ctx, double *ms_total, int64_t *steps)
{
    if (!ctx || !ms_total || !steps) return EFCP_EINVAL;
    for (int i = 0; i < EFCP_K_COUNT; i++) ms_total[i] = 0.0;
    *steps = 0;
    if (!ctx->prof_on) return fail(ctx, EFCP_EINVAL, "profiling is not enabled");
    if (int rc = sync_last(ctx)) return rc;
    const int n = ctx->prof_count < kProfSteps ? ctx->prof_count : kProfSteps;
    for (int s = 0; s < n; s++) {
        hipEvent_t *ev = &ctx->ev[(size_t)s * kProfEvents];
        for (int i = 0; i < EFCP_K_COUNT; i++) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, ev[i], ev[i + 1]) != hipSuccess)
                return fail(ctx, EFCP_EHIP, "hipEventElapsedTime failed");
            ms_total[i] += ms;
        }
    }
    *steps = n;
    ctx->prof_count = 0;
    return EFCP_OK;
}

extern "C" const char *efcp_last_error(efcp_ctx *ctx) { return ctx ? ctx->err : "null context"; }
