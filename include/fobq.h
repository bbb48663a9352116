/*
 * libfobq -- sensitivity-guided, row-parallel, Hessian-compensated layer
 * quantization on one AMD MI355X (gfx950).  C ABI; every pointer named
 * "device" is HIP device memory on the context's GPU, everything else is host
 * memory.  No function throws; every function returns a fobq_status (or a
 * pointer, for fobq_last_error).
 *
 * The method (Zheng et al., "Sensitivity-Aware Post-Training Quantization for
 * Deep Neural Networks"), in the paper's notation: a layer has weights W
 * (d_row x d_col) and calibration inputs X (d_col x N); the layer objective is
 * |WX - W^X|^2 (Section 3, Eq. 2), whose Hessian with respect to one row of W
 * is 2 X X^T.  All rows share the one inverse Hessian Hinv (Section 4.2).
 *
 * Arithmetic: the whole path computes in fp64 (inputs W and X are fp32 and are
 * widened exactly).  The rounding decision code = rint(w / scale) + zero is
 * taken in fp64.
 *
 * Layouts: all matrices are dense row-major.  W is d_row x d_col, X is
 * d_col x n with row stride ld (elements), H is d_col x d_col.
 *
 * Ownership: inputs are never modified; outputs are caller-allocated and
 * caller-owned; scratch memory is owned by the context, grows on demand
 * (hipMalloc, which synchronises the device) and is released by fobq_destroy.
 * A context is bound to one device and one HIP stream and must not be used
 * from two threads at once.
 */
#ifndef FOBQ_H
#define FOBQ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fobq_ctx fobq_ctx;

typedef enum {
    FOBQ_OK = 0,
    FOBQ_EINVAL = -1, /* bad argument (shape, bits, group, NULL pointer, bad permutation)  */
    FOBQ_ENOMEM = -2, /* device or host allocation failed                                   */
    FOBQ_EHIP = -3,   /* a HIP call failed; fobq_last_error has the HIP error string        */
    FOBQ_ENOTPD = -4, /* a Cholesky / elimination pivot was <= 0 or not finite              */
    FOBQ_ESTATE = -5  /* call sequence error (e.g. accumulate before begin)                 */
} fobq_status;

/* Column processing order (Section 4.2, step 3).  The other keys and directions are the
 * ones of the ordering ablation (Section 4.1, Table 3: "err", "w", "sensi" x "des", "asc",
 * "No Sorting"), aggregated per column.  Equal keys keep index order. */
typedef enum {
    FOBQ_ORDER_NATURAL = 0,    /* columns 0, 1, 2, ... ("No Sorting")                         */
    FOBQ_ORDER_SENSI_DESC = 1, /* by S_j = sum_i L_q(w_ij), descending (the paper's method)   */
    FOBQ_ORDER_CUSTOM = 2,     /* caller-supplied permutation perm_in                         */
    FOBQ_ORDER_ERR_DESC = 3,   /* by sum_i (quant(w_ij) - w_ij)^2, descending                 */
    FOBQ_ORDER_W_DESC = 4,     /* by sum_i w_ij^2, descending                                 */
    FOBQ_ORDER_SENSI_ASC = 5,  /* ascending variants                                          */
    FOBQ_ORDER_ERR_ASC = 6,
    FOBQ_ORDER_W_ASC = 7,
    FOBQ_ORDER_SENSI_DYNAMIC = 8 /* Section 5 read literally (sorting repeated for every column): before   */
                                 /* each step S_j is recomputed from the current weights and the current */
                                 /* shared inverse and the largest is taken (smaller index among equals); */
                                 /* always runs one column per launch, `block` is ignored                 */
} fobq_order;

typedef struct {
    int32_t bits;       /* 2..8: grid has 2^bits levels, codes 0..2^bits-1                   */
    int32_t group;      /* 0: one grid per row; g > 0: one grid per row and per g consecutive */
                        /* original columns (g must divide d_col)                            */
    double  damp;       /* relative damping: lambda = damp * mean(diag H) + damp_abs          */
    double  damp_abs;   /* absolute addend to diag H (Section 6.1 "damping value")           */
    int32_t order;      /* fobq_order                                                        */
    int32_t block;      /* 1: unblocked rank-1 updates, one launch per column (Eq. 11, 12    */
                        /* literally); 0: default blocked form (64); 2..64: block width B of */
                        /* the deferred rank-B updates                                       */
    int32_t stop_after; /* -1: all columns; t >= 0: stop after t columns (test hook)         */
    int32_t reserved;   /* must be 0                                                         */
    const int32_t* perm_in; /* device, d_col entries; used iff order == FOBQ_ORDER_CUSTOM    */
} fobq_opts;

/* All device pointers, caller-allocated; NULL = output not wanted. */
typedef struct {
    uint8_t* codes;     /* d_row x d_col, original column order                               */
    float*   scales;    /* d_row x G, G = d_col / group (1 if group == 0)                     */
    float*   zeros;     /* d_row x G, integer-valued zero points                              */
    float*   Q;         /* d_row x d_col dequantized weights scale * (code - zero)            */
    int32_t* perm;      /* d_col: perm[t] = original index of the column processed at step t  */
    double*  W_work;    /* d_row x d_col running weights, PROCESSING order (column t = step t):*/
                        /* processed columns hold their value when quantized                  */
    double*  Hinv_work; /* d_col x d_col running shared inverse, PROCESSING order; rows and   */
                        /* columns of processed steps are 0                                   */
    double*  loss;      /* 1 value: sum over steps and rows of (w - q)^2 / (2 [Hinv]_tt)      */
} fobq_out;

/* Create a context on `device` whose work is enqueued on `hip_stream`
 * (a hipStream_t; NULL = the default stream).  Host call. */
int fobq_create(fobq_ctx** ctx, int device, void* hip_stream);
/* Synchronises the stream, frees all scratch memory.  NULL is accepted. */
int fobq_destroy(fobq_ctx* ctx);
/* Text of the last error on this context ("" if none).  Valid until the next call. */
const char* fobq_last_error(const fobq_ctx* ctx);

/* Device scratch the context holds right now, in bytes.  Scratch grows on demand and is only
 * released by fobq_destroy, so after a run this is the run's peak (the "Mem." column of the
 * paper's Tables 1-3 reports the same kind of figure for whole models).  Host call, no GPU work. */
int fobq_workspace_bytes(fobq_ctx* ctx, int64_t* bytes);

/*
 * Hessian of the layer objective (Section 3, Eq. 2): H = (2 / N) X X^T, N the
 * total number of calibration columns, accumulated over chunks of columns.
 *   begin       resets the accumulator for a d_col x d_col Hessian.
 *   accumulate  adds X_c X_c^T for a chunk X_c (device, fp32, d_col x n, row
 *               stride ld >= n).  Enqueues work and returns; X must stay valid
 *               until the stream reaches that work.
 *   finalize    applies 2 / N, mirrors to a full symmetric matrix kept in the
 *               context, and, if H_out != NULL (device, d_col x d_col fp64),
 *               copies it there.  Enqueues and returns.
 * Errors: EINVAL on bad sizes/NULL, ESTATE on wrong call order, ENOMEM, EHIP.
 */
int fobq_hessian_begin(fobq_ctx* ctx, int64_t d_col);

/*
 * How fobq_hessian_accumulate forms X_c X_c^T (Section 3, Eq. 2):
 *   FOBQ_HESSIAN_FP64         fp64 matrix instructions on the exactly widened fp32 inputs (default):
 *                             the sum differs from the exact one by fp64 rounding only.
 *   FOBQ_HESSIAN_INT8_SLICES  every row of X_c as a 40-bit fixed-point number under a per-row power of
 *                             two, cut into five signed 8-bit digits; the 19 digit-by-digit products
 *                             whose weights are 256^0 .. 256^-5 relative to the leading one are formed
 *                             exactly on the int8 matrix cores (int32 sums, folded into fp64), the rest
 *                             dropped.  H differs from the fp64 result by about 3e-13 of its largest
 *                             entry; several times faster on large layers.  Applies to calls with
 *                             d_col >= 384 and n >= 512 (for
 *                             fobq_hessian_accumulate_conv: output pixels of the call); other calls use the
 *                             fp64 form.  An Inf or NaN in X makes
 *                             H NaN throughout (the layer then fails with ENOTPD).  Scratch: 1.25 bytes
 *                             per element of X_c (of the unfolded input for a convolution), at most 2 GiB:
 *                             longer calls run as several launches.
 * Stays in force until changed; not while an accumulation has begun (ESTATE).
 */
typedef enum { FOBQ_HESSIAN_FP64 = 0, FOBQ_HESSIAN_INT8_SLICES = 1 } fobq_hessian_mode;
int fobq_hessian_set_mode(fobq_ctx* ctx, int mode);
int fobq_hessian_accumulate(fobq_ctx* ctx, const float* X, int64_t n, int64_t ld);
int fobq_hessian_finalize(fobq_ctx* ctx, double* H_out);

/*
 * The same accumulation for a k x k convolution, straight from its input feature maps
 * (Section 6.1: the quantized layers are convolutions; their X is the unfolded input).
 * Equivalent to fobq_hessian_accumulate on X = unfold(maps) without materialising X, where
 *   row    c * k * k + ky * k + kx   (the column order of a weight matrix W[out][c][ky][kx])
 *   column image * ho * wo + y * wo + x,  ho = (h + 2 pad - k) / stride + 1, wo likewise
 *   X[row][column] = maps[image][y * stride + ky - pad][x * stride + kx - pad][c], 0 outside the map.
 * maps: device fp32, n_img x h x w x c, channels innermost (NHWC).  d_col of fobq_hessian_begin
 * must equal c * k * k; 1 <= k <= 64, 1 <= stride <= 64, 0 <= pad <= 64.  The context keeps a
 * zero-padded copy of the maps of one call ((n_img + 1) (h + 2 pad) (w + 2 pad) c floats of scratch):
 * pass fewer images per call to bound it.  N grows by n_img * ho * wo (< 2^31 per call).  One accumulation uses
 * either this call (always with the same c and k) or fobq_hessian_accumulate, not both (ESTATE).
 * In the mode FOBQ_HESSIAN_INT8_SLICES a convolution with stride 1, k = 2 or 3 and a multiple of 64
 * channels (d_col >= 384) is accumulated by tap offsets: a block of H depends on its two taps through their
 * offset and the window of the padded map the first one sweeps, so the block rows of the taps
 * (0, 0) and (0, k - 1) are formed by exact digit products and every other block from one of
 * theirs by adding and removing single rows and columns of the map (fp64).  Same H to the
 * mode's accuracy, about half the matrix work.  The first call of an accumulation decides; if it
 * took this form, a later call with another stride fails with ESTATE.
 * Enqueues work and returns; maps must stay valid until the stream reaches that work.
 */
int fobq_hessian_accumulate_conv(fobq_ctx* ctx, const float* maps, int64_t n_img, int64_t h, int64_t w,
                                 int64_t c, int32_t k, int32_t stride, int32_t pad);

/* Which arithmetic the accumulation that is running (or was finalized last) on this context took,
 * decided by its accumulate calls: FOBQ_FORM_FP64 (no call yet, or fp64 products only),
 * FOBQ_FORM_INT8_SLICES (digit products over the lower triangle in at least one call),
 * FOBQ_FORM_INT8_TAP_OFFSETS (convolution by tap offsets).  For reports. */
typedef enum { FOBQ_FORM_FP64 = 0, FOBQ_FORM_INT8_SLICES = 1, FOBQ_FORM_INT8_TAP_OFFSETS = 2 } fobq_hessian_form_t;
int fobq_hessian_form(fobq_ctx* ctx, int32_t* form);

/*
 * Quantize one layer (Section 4.2, steps 1-5):
 *   damp H and invert it through its Cholesky factor (Section 5 item 1,
 *   Section 6.1); freeze the min-max grid of every row / group from W;
 *   column scores S_j (Eq. 10 summed over rows) and the processing order;
 *   then for each column in that order quantize all rows at once, push
 *   e = (w - q) / [Hinv]_tt into the columns not yet quantized (Eq. 9 / 11) and
 *   eliminate the column from the one shared Hinv (Eq. 12).
 * W: device fp32 d_row x d_col.  H: device fp64 d_col x d_col full symmetric
 * undamped Hessian, or NULL to use the one accumulated in the context
 * (fobq_hessian_finalize must have been called with the same d_col).
 * The call enqueues all work on the context's stream, then SYNCHRONISES the
 * stream and reports device-detected failures (ENOTPD, bad custom permutation).
 * On error the contents of the outputs are unspecified; a call that fails after work was enqueued
 * waits for that work (both of the context's streams) before it returns, so W, H and the outputs
 * may be released and the context used again.
 */
int fobq_quantize_layer(fobq_ctx* ctx, const float* W, int64_t d_row, int64_t d_col,
                        const double* H, const fobq_opts* opts, const fobq_out* out);

/*
 * The same in two halves, for callers that keep several contexts busy at once (layers are
 * independent of each other, Section 3; most of a layer's work is a chain of short dependent
 * launches that leaves the GPU nearly idle, so layers on different contexts / streams overlap well):
 *   fobq_quantize_layer_enqueue  checks the arguments, enqueues all work and returns without
 *                                waiting; W, H, perm_in and the outputs must stay valid until
 *                                fobq_finish returns.  Only Hessian accumulation for the next
 *                                layer may be called on the context before fobq_finish (ESTATE
 *                                otherwise).
 *   fobq_finish                  synchronises the context's stream and reports the enqueued
 *                                layer's device-detected failures (ENOTPD, bad permutation);
 *                                with nothing enqueued it only synchronises.
 */
int fobq_quantize_layer_enqueue(fobq_ctx* ctx, const float* W, int64_t d_row, int64_t d_col,
                                const double* H, const fobq_opts* opts, const fobq_out* out);
int fobq_finish(fobq_ctx* ctx);

/*
 * Several small layers in one call (Section 3: "each layer is quantized independently").  A layer of up
 * to 256 columns is a chain of short dependent steps that leaves the GPU idle; here every stage of the
 * path is ONE launch for all layers of the batch (grid and column sums, damped inverse, scores and order,
 * shared-Hinv elimination, column loop with emit, loss), one workgroup per layer walking the factor path
 * of its layer, so the cost of a batch is about that of one small layer.  Results per layer are those of
 * fobq_quantize_layer (same arithmetic in fp64; sums inside the deferred updates are taken in a
 * different order).
 *   layers   host array of n_layers entries: W (device fp32 d_row x d_col), H (device fp64 d_col x d_col,
 *            full symmetric, undamped: e.g. from fobq_hessian_finalize(ctx, H)), out (device pointers as in
 *            fobq_out; W_work and Hinv_work must be NULL)
 *   opts     one set of options for all layers: bits, group (must divide every d_col), damp, damp_abs, order
 *            (not CUSTOM, not SENSI_DYNAMIC); block 0 or 64; stop_after -1
 * Limits: n_layers <= 256, d_col <= 256 (EINVAL beyond).  Scratch comes from one pool of the context.
 * Enqueues everything on the context's stream, then SYNCHRONISES and reports the first layer whose damped
 * Hessian or running inverse is not positive definite (ENOTPD, layer index in fobq_last_error); the other
 * layers' outputs are complete all the same.
 */
typedef struct {
    const float*  W;
    int64_t       d_row, d_col;
    const double* H;
    fobq_out      out;
} fobq_layer;
int fobq_quantize_layers_batched(fobq_ctx* ctx, int32_t n_layers, const fobq_layer* layers, const fobq_opts* opts);

/* ---- stage-level entry points (test and benchmark hooks) ------------------ */

/* Hinv = H^-1 for symmetric positive definite H via H = L L^T, L^-1, L^-T L^-1
 * (Section 5 item 1).  H, Hinv: device fp64 d x d (Hinv full symmetric).
 * Synchronises; ENOTPD if a pivot is <= 0. */
int fobq_spd_inverse(fobq_ctx* ctx, const double* H, int64_t d, double* Hinv);

/* Column scores and order (Section 4.2 steps 1-3) from W and the diagonal of
 * Hinv (device fp64 d x d): S (device fp64 d_col, may be NULL; the sort key of
 * opts->order, S_j for NATURAL and CUSTOM) and perm (device int32 d_col, may be
 * NULL) for opts->order.  Uses opts->bits, group, order,
 * perm_in.  Synchronises. */
int fobq_sensitivity(fobq_ctx* ctx, const float* W, int64_t d_row, int64_t d_col,
                     const double* Hinv, const fobq_opts* opts, double* S, int32_t* perm);

/*
 * fobq_sensitivity for callers that cannot allocate device memory (code under HIP graph capture
 * elsewhere in the process, tight serving loops, harnesses that forbid hipMalloc): the same
 * kernels and results, but the scratch (grids, partial column sums, S, perm, status words) lives
 * in one file-scope device array of the library, about 4.1 MiB per GPU, held until the process
 * ends.  Its address on the context's GPU and the pinned status buffer are set up by fobq_create;
 * this call itself calls no hipMalloc / hipFree / hipHostMalloc, creates no stream and no event
 * (stage timing must be off: ESTATE otherwise).
 * Limits (EINVAL beyond them, with the numbers in fobq_last_error): d_col <= 8192,
 * d_row * G <= 131072 (G = d_col / group, 1 if group == 0), ceil(d_row / 64) * d_col <= 262144.
 * All calls on one GPU share the array, whatever their context: calls that overlap in time on one
 * GPU race; what must start at zero is cleared by the call itself.  Inputs, outputs, errors and
 * the synchronisation are those of fobq_sensitivity.
 */
int fobq_sensitivity_static(fobq_ctx* ctx, const float* W, int64_t d_row, int64_t d_col,
                            const double* Hinv, const fobq_opts* opts, double* S, int32_t* perm);

/* The baseline the method replaces (Section 4.2, first paragraphs; Eq. 9 - 12 per row): OBQ
 * quantizes every row on its own, with its own copy of the inverse Hessian and its own greedy
 * order -- at every step the not-yet-quantized weight of the row with the smallest loss term
 * (quant(w_p) - w_p)^2 / (2 [Hinv]_pp) (Eq. 10; the first in index order among equal ones) is
 * quantized, the rest of the row compensated (Eq. 9 / 11) and index p eliminated from the row's
 * inverse (Eq. 12).  Same frozen min-max grid as fobq_quantize_layer (opts: bits and group are
 * used, the order fields are ignored).  Cost O(d_col^3) per row: a measurement baseline for small
 * layers, d_col <= 4096 (FOBQ_EINVAL beyond).
 * W: device fp32 d_row x d_col.  Hinv: device fp64 d_col x d_col, full symmetric (what
 * fobq_spd_inverse returns for the damped Hessian); not modified.  Rows row_begin .. row_end - 1
 * are processed (rows do not interact); of the outputs only those rows are written:
 * codes (uint8, d_row x d_col), Q (fp32, d_row x d_col), order (int32, d_row x d_col: per row the
 * index processed at each step; may be NULL), lossrow (fp64, d_row: the row's summed loss terms).
 * All device pointers.  Scratch (the rows' running inverses beyond d_col = 128, at most 4 GiB at a
 * time) belongs to the context.  Synchronises; FOBQ_ENOTPD if a row meets a pivot <= 0. */
int fobq_obq_rows(fobq_ctx* ctx, const float* W, int64_t d_row, int64_t d_col, const double* Hinv,
                  const fobq_opts* opts, int64_t row_begin, int64_t row_end, uint8_t* codes, float* Q,
                  int32_t* order, double* lossrow);

/* Test hook for the error paths: the n-th internal status check from now on this context (n >= 1;
 * checks follow every HIP call and launch) reports FOBQ_EHIP although nothing failed; 0 disarms.
 * A call that fails this way with work already enqueued waits for that work before it returns and
 * leaves the context usable. */
int fobq_debug_fail_after(fobq_ctx* ctx, int n);

/* Test hook for the host side of the tap-offset form of fobq_hessian_accumulate_conv (stride 1; needs no GPU
 * and no context): the list of single-row / single-column correlations ("strips") and, for every pair of
 * taps that is not taken from a base block row, the signed sum of strips that turns the base block with the
 * same tap offset into the pair's block, for a k x k kernel on h x w maps padded by `pad`.  Written to out
 * (host, int32) as
 *   njobs, npairs, nterms,
 *   njobs  x (kind, coord, start, len, dy, dx)   kind 0: row `coord` of the padded map, columns start .. start+len-1;
 *                                                kind 1: column `coord`, rows start .. start+len-1; (dy, dx) = offset
 *                                                of the second factor,
 *   npairs x (tap_a, tap_b, first_term, end_term) taps as ky * k + kx,
 *   nterms x (job, sign).
 * *used = the number of words that takes; nothing is written when it exceeds cap (EINVAL), when an argument is
 * out of range (EINVAL) or when the geometry does not fit the library's tables (ESTATE: such a call of
 * fobq_hessian_accumulate_conv takes the general path). */
int fobq_debug_offset_tables(int32_t k, int32_t pad, int64_t h, int64_t w, int32_t* out, int64_t cap, int64_t* used);

/* Measurement aid for the X X^T kernel of the int8-slice mode (no part of the method): the rate, in
 * 1e12 int8 operations per second (multiply and add counted separately), at which this GPU's matrix
 * cores run that kernel's inner loop -- the 19 digit products of a k-step on 32 x 32 x 32 int8
 * matrix instructions, 8 wavefronts per compute unit -- when the operands sit in LDS and nothing is
 * fetched or synchronised.  The rate depends on the operand bytes (the chip holds its power limit by
 * slowing the matrix pipes), hence operand_kind: all bytes equal; uniformly random bytes; the digits
 * of ReLU(N(0,1)) values as the workloads' activations have them (half of the values zero).
 * Allocates a few KiB of device memory for the duration of the call, runs on the context's stream
 * and waits for it.  FOBQ_EINVAL for an unknown kind or a NULL pointer, FOBQ_EHIP / FOBQ_ENOMEM
 * from the runtime. */
typedef enum {
    FOBQ_PROBE_EQUAL_BYTES = 0,
    FOBQ_PROBE_RANDOM_BYTES = 1,
    FOBQ_PROBE_RELU_DIGITS = 2
} fobq_probe_operands;
int fobq_probe_int8_matrix_rate(fobq_ctx* ctx, int operand_kind, double* tera_ops_per_second);

/* ---- stage timing ---------------------------------------------------------- */
typedef enum {
    FOBQ_STAGE_XXT = 0,      /* the X X^T kernel launches only                              */
    FOBQ_STAGE_FINALIZE = 1, /* split reduction, 2/N, mirror                                */
    FOBQ_STAGE_CHOLESKY = 2, /* damping + H = L L^T (d_col <= 4096: also L^-1, L^-T L^-1)   */
    FOBQ_STAGE_INVERSE = 3,  /* L^-1 and L^-T L^-1 where they are separate launches         */
    FOBQ_STAGE_ORDER = 4,    /* column scores and sort (the grid runs beside the Cholesky)  */
    FOBQ_STAGE_PERMUTE = 5,  /* gather W and Hinv into processing order                     */
    FOBQ_STAGE_ELIMINATE = 6,/* shared-Hinv elimination (blocked form only)                 */
    FOBQ_STAGE_COLUMNS = 7,  /* column loop: quantize + compensate (+ Eq. 12 when unblocked)*/
    FOBQ_STAGE_EMIT = 8,     /* scatter to original order, loss                             */
    FOBQ_STAGE_SLICE = 9,    /* integer-slice mode: row exponents and digits of X           */
    FOBQ_STAGE_COUNT = 10
} fobq_stage;

/* Turn hipEvent timing of the stages on or off (off by default): on = 0 none, 1 every stage,
 * or a sum of FOBQ_PROFILE_STAGE(s) for the stages s to time (each timed interval costs two
 * event records on the stream, a few microseconds of launch gap each). */
#define FOBQ_PROFILE_STAGE(s) (2 << (s))
int fobq_profile_enable(fobq_ctx* ctx, int on);
/* Synchronises, folds pending events, returns accumulated milliseconds and the
 * number of timed intervals of `stage` since the last reset. */
int fobq_profile_get(fobq_ctx* ctx, int stage, double* ms, int64_t* intervals);
int fobq_profile_reset(fobq_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* FOBQ_H */
