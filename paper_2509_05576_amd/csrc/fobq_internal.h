// Internal declarations shared by the translation units of libfobq (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>
#include <vector>

#include "fobq.h"

namespace fobq {

// code = clamp(rint(w / scale) + zero, 0, maxq), rint = round half to even, all fp64 (Section 3: the fixed grid)
__device__ __forceinline__ double grid_code(double w, double scale, double zero, double maxq)
{
    double c = rint(w / scale) + zero;
    c = c < 0.0 ? 0.0 : c;
    c = c > maxq ? maxq : c;
    return c;
}

// ---------------------------------------------------------------------------
// Device buffer owned by the context; grows, never shrinks.
struct DevBuf {
    void*  p = nullptr;
    size_t cap = 0;
    hipError_t ensure(size_t bytes) {
        if (bytes <= cap) return hipSuccess;
        if (p) { (void)hipFree(p); p = nullptr; cap = 0; }
        size_t want = (bytes + 255) & ~size_t(255);
        hipError_t e = hipMalloc(&p, want);
        if (e == hipSuccess) cap = want; else p = nullptr;
        return e;
    }
    void release() { if (p) (void)hipFree(p); p = nullptr; cap = 0; }
    template <class T> T* as() const { return reinterpret_cast<T*>(p); }
};

// ---------------------------------------------------------------------------
// Generic fp64 MFMA GEMM:  C = beta*C + alpha * op(A) * op(B), row-major.
//   op(A) is M x K:  TA=false -> A[m*lda + k],  TA=true -> A[k*lda + m]
//   op(B) is K x N:  TB=false -> B[k*ldb + n],  TB=true -> B[n*ldb + k]
// Tiles of 64 x 64 per workgroup; tiles can be restricted to one triangle and
// the K range of a tile can be restricted when an operand is triangular.
enum { CMODE_ALL = 0, CMODE_LOWER = 1, CMODE_UPPER = 2 };
enum { KMODE_FULL = 0,      // k in [0, K)
       KMODE_GE_MAX_MN = 1, // k >= max(m0, n0)   (both operands zero above)
       KMODE_GE_N = 2,      // k >= n0            (op(B) lower triangular)
       KMODE_LT_M = 3 };    // k <  m0 + 64       (op(A) lower triangular)

struct GemmP {
    int M = 0, N = 0, K = 0;
    const double* A = nullptr; int64_t lda = 0;
    const double* B = nullptr; int64_t ldb = 0;
    double* C = nullptr;       int64_t ldc = 0;
    double* C2 = nullptr;              // optional second output: rowscale[m] * result
    const double* rowscale = nullptr;
    double alpha = 1.0, beta = 0.0;
    int cmode = CMODE_ALL, kmode = KMODE_FULL;
    int kmin = 0;                      // k starts no lower than this (a multiple of 64)
    int beta_ncols = -1;               // >= 0: beta applies only to the tiles left of this column (0 elsewhere)
    // batching (blockIdx.z): element strides and per-batch clamps
    int batches = 1;
    int64_t sA = 0, sB = 0, sC = 0;
    int Mtot = -1, mstep = 0;          // M_eff = min(M, Mtot - b*mstep) when Mtot >= 0
    int Ktot = -1, kstep = 0;          // K_eff likewise
};
// `done` (here and in the launchers below that take one; may be null): an event that is recorded when the launch
// completes.  It rides on the launch as its stop event (hipExtLaunchKernelGGL): a separate hipEventRecord
// between two dependent launches is a bubble of about 4 us on the stream.
hipError_t gemm64(hipStream_t s, const GemmP& p, bool TA, bool TB, hipEvent_t done = nullptr);

// ---------------------------------------------------------------------------
// Stage timing (hipEvents on the context's stream), off by default.
struct StageTimer {
    std::vector<std::pair<hipEvent_t, hipEvent_t>> pending[FOBQ_STAGE_COUNT];
    std::vector<hipEvent_t> pool;
    double  ms[FOBQ_STAGE_COUNT] = {0};
    int64_t launches[FOBQ_STAGE_COUNT] = {0};
};

}  // namespace fobq

constexpr int FLAG_WORDS = 16, FLAG_WORD_MATE = 8, FLAG_WORD_NONFINITE = 9;

struct fobq_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    std::string err;

    // Hessian accumulation state
    int64_t h_d = 0;        // d_col of the running accumulation (0 = none)
    int64_t h_n = 0;        // calibration columns seen so far
    int     h_splits = 0;   // split-K partial slabs in Hpart
    int     h_zeroed = 0;   // slabs of Hpart cleared (and possibly written) since hessian_begin
    bool    h_final = false;
    int     h_conv_c = 0;   // > 0: accumulation in convolution mode with this many channels ...
    int     h_conv_k = 0;   // ... and this kernel size; -1 in h_conv_c: plain mode
    int     h_mode = 0;     // fobq_hessian_mode
    bool    h_i8_used = false;  // the integer-slice kernels ran in this accumulation
    bool    h_offsets = false;  // convolution mode by tap offsets (hessian_offsets.hip) in this accumulation
    fobq::DevBuf hcorr;     // d x d fp64: the corrections of that mode, tap-major
    fobq::DevBuf strips;    // jobs x c x c fp64: the strips of one call
    fobq::DevBuf i8planes;  // digits of one accumulate call (see hessian_i8.hip)
    fobq::DevBuf i8sh;      // per-row shifts of that call
    fobq::DevBuf i8amax;    // per-channel maxima (convolution input)
    fobq::DevBuf batch_pool;    // scratch of all layers of a batched call
    fobq::DevBuf batch_desc;    // BatchLayer[n] + status words
    void* h_batch = nullptr;    // pinned host staging for the descriptors and the status read-back

    fobq::DevBuf Hpart;     // h_splits x d x d fp64 partial sums of X X^T (lower tiles)
    fobq::DevBuf maps_pad;  // zero-padded copy of the feature maps of one accumulate_conv call (+ 1 zero image)
    fobq::DevBuf H;         // d x d fp64, (2/N) X X^T, full symmetric

    // factorization / elimination workspace (all d x d fp64 unless noted)
    fobq::DevBuf Hd, Linv, T, Hinv, A, U, Un;
    fobq::DevBuf Dblk;      // diagonal-block scratch: 2 x (64 x 64) L11^-1, 2 x (64 x 64) G, 2 x 64 reciprocal pivots
    fobq::DevBuf scal;      // a few fp64 scalars (lambda, loss)
    fobq::DevBuf obq;       // running inverses of the per-row baseline (fobq_obq_rows), rows x d x d fp64
    fobq::DevBuf flags;     // FLAG_WORDS int32: status flags written by kernels (cleared per call), then words
                            // that live as long as the context (FLAG_WORD_MATE: see chol_iter_kernel)
    int mate_epoch = 0;     // number of the last launch that used FLAG_WORD_MATE
    int cus = 256;          // compute units of the device (fobq_create)
    int* h_flags = nullptr; // pinned host memory that the status flags are read back into (made by fobq_create)
    unsigned char* static_scratch = nullptr;   // this GPU's copy of the library's static scratch array
    int fail_countdown = 0; // test hook: > 0 = the n-th status check from now reports an injected failure
    // quantization workspace
    fobq::DevBuf Wp;        // d_row x d fp64, columns in processing order
    fobq::DevBuf DT;        // d x Rp fp64: (w - q) per processed column
    fobq::DevBuf corr;      // 2 x d_row x 64 fp64: compensation handed from one column block to the next
    fobq::DevBuf codesT;    // d x Rp u8
    fobq::DevBuf scale, zero;   // d_row x G fp64
    fobq::DevBuf S, Spart;  // d fp64, chunks x d fp64
    fobq::DevBuf perm, invperm; // d int32
    fobq::DevBuf lossrow;   // d_row fp64

    // second stream: the column loop of block k only needs the pivot rows of blocks <= k, so it
    // runs behind the shared-Hinv elimination on its own stream, ordered by one event per block
    hipStream_t side = nullptr;
    std::vector<hipEvent_t> sync_ev;

    bool pending = false;   // a layer was enqueued without the final status read (fobq_finish outstanding)
    unsigned profiling = 0;     // bit s: stage s is timed
    fobq::StageTimer timer;
};

namespace fobq {

// One layer of fobq_quantize_layers_batched as the kernels see it (an array of these lives in device memory).
// All pointers are device memory; the scratch pointers are carved out of one pool of the context.
struct BatchLayer {
    const float* W; const double* H;          // inputs
    int R, d, G, gs, Rp, chunks;              // G grids per row of gs columns; Rp = R rounded up to 64; chunks = sens_chunks(R)
    double maxq, damp, damp_abs;
    int order, kind, ascending;               // fobq_order; sort key (0 sensi, 1 err, 2 w); direction
    double *Hd, *Linv, *T, *Hinv, *A, *U, *Un;    // d x d each
    double *Gs, *rinv;                        // 64 x 64 and 64: diagonal-block scratch of the elimination
    double *Wp, *DT;                          // R x d; d x Rp
    uint8_t* codesT;                          // d x Rp
    double *scale, *zero;                     // R x G
    double *S, *Spart, *lossrow;              // d; chunks x d; R
    int *perm, *invperm, *flags;              // d; d; 4 status words (not positive definite: H, running Hinv)
    uint8_t* codes; float *scales, *zeros, *Q; int* perm_out; double* loss;   // outputs (may be null)
};
constexpr int BATCH_MAX_D = 256;      // columns of a layer in a batched call (4 panels of 64)
constexpr int BATCH_MAX_LAYERS = 256;

int set_err(fobq_ctx* c, int code, const char* fmt, ...);
int hip_err(fobq_ctx* c, hipError_t e, const char* what);

// Timing of a stage that is exactly one launch: the two events ride on the launch as its start and stop
// events (no bubble on the stream; StageScope's records cost about 4 us each).  Both null when the stage is
// not being timed.
struct LaunchEvents { hipEvent_t start = nullptr, stop = nullptr; };
LaunchEvents stage_launch_events(fobq_ctx* c, int stage);

struct StageScope {
    fobq_ctx* c; int stage; hipStream_t st; hipEvent_t e0 = nullptr, e1 = nullptr;
    StageScope(fobq_ctx* c_, int stage_, hipStream_t on = nullptr);   // on == nullptr: the context's stream
    ~StageScope();
};

// hessian.hip
hipError_t launch_xxt(hipStream_t s, const float* X, int64_t ld, int d, int64_t n, double* Hpart, int splits,
                      LaunchEvents ev = LaunchEvents());
int xxt_pick_splits(int d);
int xxt_slabs_touched(int d, int64_t n, int splits, bool conv);
hipError_t launch_clear_slabs(hipStream_t s, double* Hpart, int d, int first, int count);
hipError_t launch_pad_maps(hipStream_t s, const float* maps, int n_img, int h, int w, int c, int pad, float* out);
hipError_t launch_xxt_conv(hipStream_t s, const float* padded, int n_img, int hp, int wp, int c, int k, int stride,
                           int ho, int wo, int64_t npix, double* Hpart, int splits,
                           LaunchEvents ev = LaunchEvents());
hipError_t launch_hessian_finalize(hipStream_t s, double* Hpart, int splits, int d, double factor, double* H,
                                   int conv_c, int conv_kk, const int* poison);   // *poison != 0: H = NaN

// hessian_i8.hip: X X^T by exact integer slices on the int8 matrix cores
int i8_dpad(int d);
size_t i8_planes_bytes(int d, int64_t n);
// rect.cb > 0: instead of the lower triangle, all tile columns of two groups of rect.cb tile rows (the second group
// starts at tile row rect.gap), every entry stored.  rect.half (with cb = gap = 1): the two groups are the first 64 rows
// of tile rows 0 and 1 only, and one tile row made of those 128 rows is formed instead of two.
struct I8Rect { int cb = 0, gap = 0, half = 0; };
// full > 0: the workgroups go through the tiles in step (see xxt_i8_kernel): `full` rounds of whole tiles, then the
// `rem` tiles left over, each cut into `pieces` parts of piece_len k-steps
struct I8Lockstep { int full = 0, rem = 0, pieces = 0; int64_t piece_len = 0; };
int xxt_i8_slabs_touched(int d, int64_t n, int splits, I8Rect rect = I8Rect());
// slabs of partial sums that a launch over n columns would like to have (0: no wish beyond xxt_pick_splits)
int xxt_i8_wanted_splits(int d, int64_t n, I8Rect rect = I8Rect());
int64_t i8_block_columns(int d);      // most columns one launch of the matrix kernel takes (bounds the digit scratch)
hipError_t launch_i8_row_shifts(hipStream_t s, const float* X, int64_t ld, int d, int64_t n, int* sh, int* nonfinite);
hipError_t launch_i8_slice(hipStream_t s, const float* X, int64_t ld, int d, int64_t n, const int* sh, signed char* planes);
hipError_t launch_i8_chan_shifts(hipStream_t s, const float* padded, int64_t pixels, int c, int d, unsigned* amax, int* sh,
                                 int* nonfinite);
hipError_t launch_i8_slice_conv(hipStream_t s, const float* padded, int n_img, int hp, int wp, int c, int k, int stride,
                                int ho, int wo, int64_t npix, int64_t pix0, int64_t n, const int* sh, signed char* planes);
hipError_t launch_xxt_i8(hipStream_t s, const signed char* planes, const int* sh, int d, int64_t n, double* Hpart,
                         int splits, LaunchEvents ev = LaunchEvents(), I8Rect rect = I8Rect());
hipError_t launch_damp(hipStream_t s, const double* H, int d, double damp, double damp_abs, double* Hd, double* lam_out);
// hessian_offsets.hip: Hessian of a stride-1 convolution by tap offsets (two block rows from the digit-product kernel,
// the other blocks by corrections over single rows and columns of the padded maps)
constexpr int OFFSET_MAX_TAPS = 9, OFFSET_MAX_JOBS = 128, OFFSET_MAX_PAIRS = 81, OFFSET_MAX_TERMS = 384;
// one strip: kind 0 = row `coord` of the padded map, columns start .. start + len - 1; kind 1 = column `coord`, rows
// start .. start + len - 1; (dy, dx) = the offset of the second factor
struct OffsetJob { int coord, start, len; signed char kind, dy, dx, unused; };
// passed to the kernels by value (about 3 KiB)
struct OffsetTables {
    int njobs, npairs, nterms;
    OffsetJob jobs[OFFSET_MAX_JOBS];
    unsigned char pair_ta[OFFSET_MAX_PAIRS], pair_tb[OFFSET_MAX_PAIRS];   // tap indices ky * k + kx of a pair with corrections
    short pair_begin[OFFSET_MAX_PAIRS + 1];                               // its terms: [pair_begin[p], pair_begin[p + 1])
    unsigned char term_job[OFFSET_MAX_TERMS];
    signed char term_sign[OFFSET_MAX_TERMS];
};
bool offset_tables_build(int k, int pad, int h, int w, OffsetTables* tab);
size_t offset_strips_bytes(int njobs, int c);
hipError_t launch_clear_slab_rows(hipStream_t s, double* Hpart, int d, int first, int count, int row0, int n0, int row1, int n1);
hipError_t launch_offset_corrections(hipStream_t s, const float* padded, int n_img, int hp, int wp, int c, int d,
                                     const OffsetTables& tab, double* strips, double* corr);
hipError_t launch_hessian_finalize_offsets(hipStream_t s, const double* Hpart, int splits, int d, double factor, double* H, int c,
                                           int k, const double* corr, const int* poison);

// factor.hip
// Sacc != null (d x d scratch): L^-1 and the upper tiles of Hinv = L^-T L^-1 are completed alongside the
// factorization; Sacc == null: only the diagonal blocks of L^-1 are written and Hinv is not touched
// (trtri_lower and lauum_upper finish the job)
hipError_t cholesky_lower(fobq_ctx* c, double* Hd, double* L, int d, double* Linv, int* flag, double* Sacc,
                          double* Hinv);  // Hd = L L^T; Linv gets the diagonal-block inverses
hipError_t trtri_lower(fobq_ctx* c, const double* L, int d, double* Linv, double* T);      // completes Linv
hipError_t lauum_upper(fobq_ctx* c, const double* Linv, int d, double* Hinv);              // upper tiles of Linv^T Linv
// `rows_ready` (may be null): rows_ready[k] is recorded on the context's stream once the pivot rows of
// block k (rows k*block .. of U and Un) are complete.  In the fused form the event rides on the panel launch
// as its stop event: a separate hipEventRecord between two dependent launches would be a bubble of about 4 us.
hipError_t eliminate_blocked(fobq_ctx* c, double* A, int d, int steps, int block, double* U, double* Un, int* flag,
                             const std::vector<hipEvent_t>* rows_ready);

// batched small layers: factor.hip (batch_factor), quant.hip (the rest); grids have one dimension over the layers
hipError_t launch_batch_inverse(hipStream_t s, const BatchLayer* layers, int n);
hipError_t launch_batch_order(hipStream_t s, const BatchLayer* layers, int n);
hipError_t launch_batch_eliminate(hipStream_t s, const BatchLayer* layers, int n);
hipError_t launch_batch_grid(hipStream_t s, const BatchLayer* layers, int n, int max_pairs);
hipError_t launch_batch_sens_partial(hipStream_t s, const BatchLayer* layers, int n, int max_chunks);
hipError_t launch_batch_columns(hipStream_t s, const BatchLayer* layers, int n, int max_rows);
hipError_t launch_batch_loss(hipStream_t s, const BatchLayer* layers, int n);

// per-row baseline (obq.hip)
constexpr int OBQ_MAX_D = 4096;        // columns: a row's weights, pivot row and flags live in LDS
size_t obq_scratch_per_row(int d);
hipError_t launch_obq_rows(hipStream_t s, const float* W, int d, int bits, int group, const double* Hinv0, const double* scale,
                           const double* zero, int row_begin, int rows, double* Hscratch, uint8_t* codes, float* Q, int* order,
                           double* lossrow, int* flag);

// quant.hip
hipError_t launch_grid(hipStream_t s, const float* W, int R, int d, int bits, int group,
                       double* scale, double* zero, float* scales_out, float* zeros_out);
hipError_t launch_sens_partial(hipStream_t s, const float* W, int R, int d, int bits, int group,
                               const double* scale, const double* zero, double* Spart, int chunks, int kind, hipEvent_t done = nullptr);
hipError_t launch_sens_reduce(hipStream_t s, const double* Spart, int chunks, int d, const double* Hinv, double* S,
                              int kind);
int sens_chunks(int R);
hipError_t launch_rank_sort(hipStream_t s, const double* S, int d, int* perm, int* invperm, int ascending);
hipError_t launch_iota(hipStream_t s, int d, int* perm, int* invperm);
hipError_t launch_check_perm(hipStream_t s, const int* perm_in, int d, int* perm, int* invperm, int* flag);
hipError_t launch_gather(hipStream_t s, const float* W, int R, int d, const int* perm,
                         const double* Hinv_upper, double* Wp, double* A, hipEvent_t done = nullptr);
hipError_t launch_col_block(hipStream_t s, double* Wp, int R, int d, int o, int nb,
                            const double* Un, const double* U, const double* scale, const double* zero,
                            int G, int group, const int* perm, int bits,
                            uint8_t* codesT, double* DT, int Rp, double* lossrow,
                            const double* corr_in, double* corr_out, int nb_next,
                            int uo, int unb, int c0, hipEvent_t done = nullptr);
hipError_t launch_invert_perm(hipStream_t s, const int* perm, int d, int* invperm);
hipError_t launch_dyn_select(hipStream_t s, double* Wp, int R, int d, int t, double* A, const double* scale,
                             const double* zero, int G, int group, int* perm, int bits, double* Spart, int chunks);
hipError_t launch_step(hipStream_t s, double* Wp, int R, int d, int t, double* A,
                       const double* scale, const double* zero, int G, int group, const int* perm, int bits,
                       uint8_t* codesT, int Rp, double* lossrow, int* flag);   // *flag = 1 when the pivot is not > 0
hipError_t launch_emit(hipStream_t s, const uint8_t* codesT, int Rp, int R, int d, int steps,
                       const int* invperm, const double* scale, const double* zero, int G, int group,
                       uint8_t* codes, float* Q, const double* lossrow, double* loss);   // loss may be null
hipError_t launch_loss(hipStream_t s, const double* lossrow, int R, double* loss);
hipError_t launch_hinv_work(hipStream_t s, const double* A, int d, int steps, double* out);
hipError_t launch_fill_i32(hipStream_t s, int* p, int64_t n, int v);
hipError_t launch_clear_words(hipStream_t s, void* p1, int64_t n1, void* p2, int64_t n2,
                              hipEvent_t done = nullptr);   // 4-byte words

}  // namespace fobq
