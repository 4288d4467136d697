/*
 * efcp.h -- C ABI of libefcp: one EFCP / Sparse M-FAC optimizer step on one
 * AMD MI355X (gfx950).
 *
 * One call to efcp_step performs, for the step t = 1, 2, ... it is called on
 * (paper: Algorithm 1, lines 5-8; Section "Efficient Full-Matrix
 * Preconditioners", WSM recursion and eq. (2); Section "Compressing
 * Preconditioners via Sparsity", sparse window G = (I, V), SP and LCG):
 *
 *   a    = e + grad                         fp32, round to nearest even
 *   c    = TopK(a)                          the k largest |a_j|; ties at the
 *                                           threshold go to the lower index
 *   e    = a - c                            +0 where selected, a_j elsewhere
 *   slot (t-1) mod m of the window <- c     (index, fp32 value) pairs, indices
 *                                           ascending, oldest row replaced.  In memory an
 *                                           index is its 16-bit position inside the d-slice
 *                                           (at most 16384 coordinates) it falls in (the slice
 *                                           follows from a per-row offset table): lossless,
 *                                           6 bytes per entry instead of 8; efcp_get_row
 *                                           returns plain int32 indices
 *   S[slot][r] = S[r][slot] = <c_r, c>      fp64, every filled row r
 *   q[r] = <c_r, grad>                      fp64 (x = grad is the vector preconditioned)
 *   coef = (1/lambda) (m*lambda*I + S)^-1 q fp64, the coefficients of eq. (2)
 *   out  = grad/lambda - sum_r coef[r] c_r  = F^-1 grad,
 *          F = lambda*I + (1/m) sum_r c_r c_r^T over the filled rows
 *          (unfilled slots are zero rows, the divisor stays m).
 *
 * All pointers named "device" are HIP device pointers on the device that was
 * current when efcp_create ran, and that device has to be current in every
 * later call on the context (EFCP_EINVAL otherwise; efcp_destroy switches to it
 * by itself and back); pointers named "host" are ordinary host memory.  Every
 * function returns EFCP_OK (0) or a negative efcp_status; no function throws,
 * aborts or prints.  A context may be used by one host thread at a time.
 */
#ifndef EFCP_H
#define EFCP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct efcp_ctx efcp_ctx;

typedef enum {
    EFCP_OK = 0,
    EFCP_EINVAL = -1,   /* bad argument (range, NULL, aliasing, alignment) */
    EFCP_ENOMEM = -2,   /* device or host allocation failed, or workspace too small */
    EFCP_EHIP = -3,     /* a HIP runtime call or kernel launch reported an error */
    EFCP_ENUMERIC = -4  /* the coefficient factorisation met a non-positive pivot */
} efcp_status;

/* Storage format of the values V of the window G = (I, V) (Section "Format for V"); indices are
 * 16-bit in-slice positions in both. */
typedef enum {
    EFCP_VALUES_FP32 = 0,  /* fp32 values, exactly a_j (6 bytes per entry), the default          */
    EFCP_VALUES_BF16 = 1   /* bfloat16 values (4 bytes per entry).
                              c holds bf16(a_j) (round to nearest even) at the
                              selected positions and, as xi = a - c says, e keeps the rounding
                              remainder a_j - bf16(a_j) there instead of 0.  Selection is still
                              done on the fp32 accumulator.                                     */
} efcp_value_format;

/* Bytes of device memory a context for (d, m, k) needs; 0 if the arguments
 * are invalid (or the device lacks the 160 KiB of LDS per workgroup of gfx950). */
size_t efcp_workspace_bytes(int64_t d, int32_t m, int64_t k);
size_t efcp_workspace_bytes_fmt(int64_t d, int32_t m, int64_t k, int32_t value_format);

/* Create a context: error feedback e = 0, empty window, S = 0, step count 0.
 *   d       dimension,            1 <= d < 2^31
 *   m       window slots,         1 <= m <= 1024
 *   k       entries kept per row, 1 <= k <= d
 *   lambda  damping, finite, > 0  (F_0 = lambda*I)
 *   workspace        device memory of at least efcp_workspace_bytes() bytes,
 *                    256-byte aligned, owned by the caller and kept alive
 *                    until efcp_destroy; or NULL, then the library allocates
 *                    (hipMalloc) and frees it in efcp_destroy.
 * Synchronises the device once (state initialisation). */
int efcp_create(efcp_ctx **ctx, int64_t d, int32_t m, int64_t k, double lambda,
                void *workspace, size_t workspace_bytes);

/* Same with an explicit window format (efcp_value_format); efcp_create is the fp32 format. */
int efcp_create_fmt(efcp_ctx **ctx, int64_t d, int32_t m, int64_t k, double lambda,
                    int32_t value_format, void *workspace, size_t workspace_bytes);

/* Top-k applied in blocks (Section "Sparsity Pattern"; the selection rule of the paper's own
 * implementation): every block of EFCP_TOPK_BLOCK consecutive coordinates keeps exactly k
 * entries, its k largest |a_j| (ties -> lower index); a ragged last block of len coordinates
 * keeps ceil(k*len/EFCP_TOPK_BLOCK).  The block is the d-slice the SP and LCG kernels stage in
 * LDS.  Error feedback, selection and compaction are then one kernel with minimal traffic.
 *   topk_block   0: global Top-k of k entries (efcp_create_fmt); EFCP_TOPK_BLOCK: in blocks,
 *                k = entries per block, 1 <= k <= EFCP_TOPK_BLOCK; anything else: EFCP_EINVAL
 * The row length (entries efcp_get_row returns) is efcp_row_length(d, k, topk_block). */
#define EFCP_TOPK_BLOCK 16384
int efcp_create_ex(efcp_ctx **ctx, int64_t d, int32_t m, int64_t k, double lambda,
                   int32_t value_format, int32_t topk_block, void *workspace, size_t workspace_bytes);
size_t efcp_workspace_bytes_ex(int64_t d, int32_t m, int64_t k, int32_t value_format,
                               int32_t topk_block);
/* Entries per window row for these arguments; 0 if they are invalid. */
int64_t efcp_row_length(int64_t d, int64_t k, int32_t topk_block);

/* Sparse GGT instead of Sparse M-FAC on the same error feedback, Top-k, window and SP / LCG
 * kernels (Appendix "Sparse GGT", Algorithm "Detailed Sparse GGT Implementation"): every step
 * and efcp_apply then produce u = ((G G^T)^{1/2} + epsilon I)^-1 x, G = the stored vectors as
 * columns, through the eigendecomposition of the m x m matrix G^T G (a Jacobi method in one
 * workgroup; directions with a zero singular value are left out).  The paper's algorithm
 * preconditions the compressed accumulator: efcp_step_ex with EFCP_X_COMPRESSED.
 *   m        1 <= m <= 128 (the matrix is diagonalised in LDS)
 *   epsilon  finite, > 0
 * Other arguments as efcp_create_ex.  efcp_get_small then reports S = G^T G, q = G^T x and
 * the multiples coef with u = x/epsilon - sum_r coef_r c_r. */
int efcp_create_ggt(efcp_ctx **ctx, int64_t d, int32_t m, int64_t k, double epsilon,
                    int32_t value_format, int32_t topk_block, void *workspace, size_t workspace_bytes);
size_t efcp_workspace_bytes_ggt(int64_t d, int32_t m, int64_t k, int32_t value_format,
                                int32_t topk_block);

/* The general constructor: everything the calls above choose, as one structure, plus the
 * d-slice width.  opts == NULL means all zeros (fp32 values, global Top-k, Sparse M-FAC,
 * automatic width, a second stream where the step has a use for one); the calls above are this one
 * with slice_width = 0 and single_stream = 0. */
typedef enum { EFCP_SPARSE_MFAC = 0, EFCP_SPARSE_GGT = 1 } efcp_preconditioner;
typedef struct efcp_options {
    int32_t value_format;    /* efcp_value_format */
    int32_t topk_block;      /* 0 or EFCP_TOPK_BLOCK, as in efcp_create_ex */
    int32_t preconditioner;  /* efcp_preconditioner; with EFCP_SPARSE_GGT `damping` is epsilon, m <= 128 */
    int32_t slice_width;     /* Coordinates per d-slice (the LDS tile of the SP and LCG kernels and the
                                block of the Top-k passes).  0: chosen from d so that the persistent
                                SP / LCG workgroups all get the same number of slices.  Otherwise a
                                multiple of 64 in [256, 16384]; a width too small for d (more than 512
                                slices per workgroup) is EFCP_EINVAL.  Ignored with Top-k in blocks,
                                where the slice is the block.  The Top-k, the stored rows and e do not
                                depend on the width; S, q, coef and with them F^-1 x do in the last bits
                                (order of the fp64 sums).  A state exported under one width is refused by
                                a context created under another. */
    int32_t single_stream;   /* Only matters with Top-k in blocks.  There the update of the coefficient
                                factor that a full window needs on every step (deleting the oldest row) is a
                                kernel of its own.  0: it runs on a stream of the library's own, beside the
                                step's first pass, forked from and joined to the caller's stream with events.
                                1: it runs on the caller's stream, in front of that pass: no second stream,
                                no events; a step then takes that kernel's time longer.  Results are bit for
                                bit the same.  For tools that want one queue (counter collection with
                                rocprofv3 --pmc, for one) and for callers who keep their own overlap.  With
                                the global Top-k that update is part of a kernel of the selection and every
                                step stays on the caller's stream whatever this says. */
} efcp_options;
int efcp_create_opts(efcp_ctx **ctx, int64_t d, int32_t m, int64_t k, double damping,
                     const efcp_options *opts, void *workspace, size_t workspace_bytes);
size_t efcp_workspace_bytes_opts(int64_t d, int32_t m, int64_t k, const efcp_options *opts);

/* One step (see the top of this file).
 *   grad    device, d floats, 16-byte aligned, read only.  Meant to be finite.  Infinities
 *           and NaN are not rejected: Top-k orders them by their bits (above every finite
 *           value), e = a - c turns them into NaN, and S, q, coef and out are then NaN too
 *   out     device, d floats, 16-byte aligned, receives F^-1 grad; must not
 *           overlap grad.  NULL: the state (e, window, S, the coefficient
 *           factor, q, coef) is updated exactly as usual but F^-1 grad is not
 *           formed (the LCG pass is skipped), e.g. to fill the window
 *   stream  hipStream_t (NULL = the default stream)
 * Asynchronous: enqueues kernels on `stream` and returns; no host
 * synchronisation and no allocation.  Steps of one context must be issued in
 * order on one stream, or on streams ordered by the caller, with the device of
 * efcp_create current.  EFCP_EINVAL leaves the context untouched; after
 * EFCP_EHIP (a launch failed part-way) its state is undefined: every later
 * efcp_step* / efcp_apply* returns EFCP_EHIP until efcp_import_state has
 * replaced the state, or the context is destroyed.
 *
 * HIP graphs: the step number, the slot written, the number of filled rows and whether a row is
 * evicted are kept in device memory and advanced by the step's own kernels; no kernel argument
 * depends on them.  A call captured into a HIP graph (stream capture; the call then only records)
 * is therefore not one particular step but "the next step": the graph can be replayed as every
 * later step of the context, from the empty window on, with new contents in the captured grad
 * buffer.  The inspection calls below synchronise the stream of the last efcp_* call only; after
 * graph replays on another stream, synchronise that stream before calling them. */
int efcp_step(efcp_ctx *ctx, const float *grad, float *out, void *stream);

/* Which vector the step preconditions (Algorithm 1, line 8). */
typedef enum efcp_x_source {
    EFCP_X_GRAD = 0,        /* x = grad: the dense gradient is preconditioned by the sparse window */
    EFCP_X_COMPRESSED = 1   /* x = c_t, the compressed accumulator just inserted, as line 8 is
                               printed (u_t = A(c_t)).  Nothing dense is read for x: x/lambda is
                               folded into the coefficient of the newest row, and q equals the
                               Gram row. */
} efcp_x_source;

/* efcp_step with options.  State update exactly as efcp_step; what is produced differs:
 *   x_source     efcp_x_source
 *   out          device, d floats, or NULL: receives u = F^-1 x
 *   param        device, d floats, 16-byte aligned, or NULL: the model parameters, updated in
 *                place by Algorithm 1 line 9 with decoupled weight decay,
 *                    theta_j <- fp32( (1 - lr*weight_decay) * theta_j - lr * u_j ),
 *                evaluated in fp64 from the fp64 value of u_j inside the LCG kernel, so u is
 *                never written to memory.  Must not overlap grad.
 *   lr, weight_decay   finite doubles, used only with param
 * At most one of out / param may be given (EFCP_EINVAL for both); with neither the LCG pass is
 * skipped.  efcp_step(ctx, grad, out, stream) is efcp_step_ex(ctx, grad, EFCP_X_GRAD, out, NULL,
 * 0, 0, stream).  Same asynchrony and ordering rules as efcp_step. */
int efcp_step_ex(efcp_ctx *ctx, const float *grad, int32_t x_source, float *out, float *param,
                 double lr, double weight_decay, void *stream);

/* out = F^-1 x for an arbitrary dense x and the window as it stands (eq. (2)): the SP pass,
 * the coefficient solve and the LCG pass without any insertion.  Error feedback, window, Gram
 * matrix, factor and step count are untouched; q and coef reported by efcp_get_small are
 * overwritten.  Before the first step F = lambda*I and out = x/lambda.
 *   x, out   device, d floats each, 16-byte aligned, not overlapping
 * Asynchronous on `stream`; ordered after the steps issued so far (also when those used
 * another stream).  Must not run concurrently with a step of the same context. */
int efcp_apply(efcp_ctx *ctx, const float *x, float *out, void *stream);

/* efcp_apply for callers that cannot allocate and want the context left exactly as it is: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels and bit for bit the same `out` as efcp_apply, but every scratch buffer
 * of the call (the per-workgroup partial sums of the SP pass, their reduction, the products
 * with the inverse factor, q and the coefficients) lives in a fixed array inside the library's
 * code object (4 MiB + 64 KiB on every device that loads the library, held until the process
 * ends) instead of the context's workspace.  So q and coef that efcp_get_small reports stay
 * those of the last step, and neither this call nor anything it calls allocates or frees
 * memory (no hipMalloc, no hipFree, no host allocation).  The array's address on the
 * context's device is resolved once, in efcp_create.
 *   EFCP_EINVAL  as efcp_apply, and if the context needs more scratch than the array holds
 *                (more than 256 SP workgroups x 1024 window rows: no context that efcp_create*
 *                accepts today does).
 * All calls on one device share the one array: two efcp_apply_noalloc calls (of the same or of
 * different contexts) that may overlap in time on a device race with each other; put them on
 * one stream or order them.  Nothing in the array needs to be cleared between calls: every
 * entry a call reads was written by that call. */
int efcp_apply_noalloc(efcp_ctx *ctx, const float *x, float *out, void *stream);

/* Frees the context (and its workspace if the library allocated it) after
 * synchronising the device.  efcp_destroy(NULL) is EFCP_OK. */
int efcp_destroy(efcp_ctx *ctx);

/* ---- inspection (parity tests, checkpointing); each synchronises `stream`
 * of the last step before copying to host memory ---- */

/* Row stored in `slot` (0 <= slot < m): k ascending (absolute) indices and k
 * values as fp32, whatever the storage format.  EFCP_EINVAL if the slot has
 * not been filled yet. */
int efcp_get_row(efcp_ctx *ctx, int32_t slot, int32_t *idx_host, float *val_host);

/* Error feedback vector e, d floats. */
int efcp_get_error(efcp_ctx *ctx, float *e_host);

/* Small state; any pointer may be NULL.
 *   S_host     m*m doubles, row-major by slot, zero for unfilled slots
 *   q_host     m doubles (by slot), of the last step
 *   coef_host  m doubles (by slot), of the last step
 *   tau        magnitude key (bits & 0x7fffffff) of the k-th largest |a_j| of the last step
 *   step       number of steps done
 * Returns EFCP_ENUMERIC if any step so far met a non-positive pivot. */
int efcp_get_small(efcp_ctx *ctx, double *S_host, double *q_host, double *coef_host,
                   uint32_t *tau, int64_t *step);

/* ---- checkpoint / resume ----
 * The complete state of a context (step count, e, the filled window rows with
 * their slice offsets, S, the coefficient factor, the Top-k prediction) as
 * one host buffer.  A context that imports it continues bit-identically to the
 * one that exported it.  The layout is private to the library version (a
 * header with a magic word, d, m, k, lambda and the geometry is checked on
 * import); both calls synchronise the stream of the last step. */

/* Bytes efcp_export_state writes now (grows with the rows filled); 0 if ctx is NULL. */
size_t efcp_state_bytes(efcp_ctx *ctx);

/* host_buf: at least efcp_state_bytes(ctx) bytes (EFCP_ENOMEM if `bytes` is smaller), 8-byte
 * aligned (EFCP_EINVAL otherwise). */
int efcp_export_state(efcp_ctx *ctx, void *host_buf, size_t bytes);

/* ctx must have been created with the same d, m, k and lambda as the exporter
 * (EFCP_EINVAL otherwise, and on a damaged or truncated buffer); its previous
 * state is replaced. */
int efcp_import_state(efcp_ctx *ctx, const void *host_buf, size_t bytes);

/* The d-slice width that slice_width = 0 stands for (host arithmetic only, no device needed):
 * the widest slice, 16384, unless rounds of 256 widest slices would be at least 2 % empty; then
 * nearly equal slices that fill every round, a multiple of 64 (of 256 and at least 1024 when one
 * round suffices).  0 if d or topk_block is invalid. */
int32_t efcp_default_slice_width(int64_t d, int32_t topk_block);

/* Geometry chosen at creation; any pointer may be NULL.
 *   slice      coordinates per d-slice staged in LDS by the SP and LCG kernels
 *              (a multiple of 64, at most 16384)
 *   n_slices   ceil(d / slice)
 *   row_stride entries between consecutive rows of I and V (k rounded up) */
int efcp_get_geometry(efcp_ctx *ctx, int32_t *slice, int32_t *n_slices, int64_t *row_stride);

/* ---- per-kernel timing with HIP events on the step's own stream ---- */

enum {
    EFCP_K_EF_HIST = 0,   /* a = e + grad, first radix histogram            */
    EFCP_K_SELECT = 1,    /* remaining radix passes, counts, scans           */
    EFCP_K_COMPACT = 2,   /* ordered compaction into the ring, e write-back  */
    EFCP_K_SP = 3,        /* q and Gram row: pass over the window            */
    EFCP_K_COEF = 4,      /* partial-sum reduction and m x m coefficient work */
    EFCP_K_LCG = 5,       /* out = grad/lambda - sum coef_r c_r: pass over the window */
    EFCP_K_COUNT = 6
};

/* enable != 0: later steps bracket each kernel group with hipEvents
 * (allocated once here, not in efcp_step).  enable == 0: stop and reset. */
int efcp_profile_enable(efcp_ctx *ctx, int enable);

/* Synchronises the stream, then accumulates the elapsed time of every step
 * recorded since the last call (at most the most recent 256 steps).
 *   ms_total  EFCP_K_COUNT doubles: summed milliseconds per kernel group
 *   steps     number of steps covered */
int efcp_profile_read(efcp_ctx *ctx, double *ms_total, int64_t *steps);

/* Static description of the last error of this context (never NULL). */
const char *efcp_last_error(efcp_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif
