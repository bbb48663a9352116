// C ABI of libfobq: argument checks, workspace, and the order in which the
// kernels of the path are enqueued.  No arithmetic of the method lives here.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>

#include "fobq_internal.h"

namespace fobq {

int set_err(fobq_ctx* c, int code, const char* fmt, ...)
{
    if (c) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        c->err = buf;
    }
    return code;
}

int hip_err(fobq_ctx* c, hipError_t e, const char* what)
{
    if (e == hipSuccess) return FOBQ_OK;
    if (e == hipErrorOutOfMemory) return set_err(c, FOBQ_ENOMEM, "%s: out of device memory", what);
    return set_err(c, FOBQ_EHIP, "%s: %s", what, hipGetErrorString(e));
}

static hipEvent_t take_event(fobq_ctx* c)
{
    if (!c->timer.pool.empty()) {
        hipEvent_t e = c->timer.pool.back();
        c->timer.pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

StageScope::StageScope(fobq_ctx* c_, int stage_, hipStream_t on) : c(c_), stage(stage_), st(on ? on : c_->stream)
{
    if (!(c->profiling >> stage & 1u)) return;
    e0 = take_event(c);
    e1 = take_event(c);
    if (e0) (void)hipEventRecord(e0, st);
}

StageScope::~StageScope()
{
    if (!e0 || !e1) return;
    (void)hipEventRecord(e1, st);
    c->timer.pending[stage].push_back({e0, e1});
}

LaunchEvents stage_launch_events(fobq_ctx* c, int stage)
{
    LaunchEvents ev;
    if (!(c->profiling >> stage & 1u)) return ev;
    ev.start = take_event(c);
    ev.stop = take_event(c);
    if (ev.start && ev.stop) c->timer.pending[stage].push_back({ev.start, ev.stop});
    else ev = LaunchEvents();
    return ev;
}

// events (no timing) that order the side stream behind the context's stream and back
static int ensure_sync_events(fobq_ctx* c, size_t n)
{
    if (!c->side && hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking) != hipSuccess) {
        c->side = nullptr;
        return set_err(c, FOBQ_EHIP, "cannot create the side stream");
    }
    while (c->sync_ev.size() < n) {
        hipEvent_t e = nullptr;
        if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess)
            return set_err(c, FOBQ_EHIP, "cannot create an event");
        c->sync_ev.push_back(e);
    }
    return FOBQ_OK;
}

static void fold_events(fobq_ctx* c)
{
    for (int st = 0; st < FOBQ_STAGE_COUNT; ++st) {
        for (auto& pr : c->timer.pending[st]) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, pr.first, pr.second) == hipSuccess) {
                c->timer.ms[st] += ms;
                c->timer.launches[st] += 1;
            }
            c->timer.pool.push_back(pr.first);
            c->timer.pool.push_back(pr.second);
        }
        c->timer.pending[st].clear();
    }
}

// `ctx->fail_countdown` (test hook, fobq_debug_fail_after): the n-th check from now reports a failure
// without the HIP call having failed, so that the error paths can be exercised from the host.
#define FOBQ_TRY(expr, what)                                                              \
    do {                                                                                  \
        hipError_t e__ = (expr);                                                          \
        if (e__ != hipSuccess) return hip_err(ctx, e__, what);                            \
        if (ctx->fail_countdown > 0 && --ctx->fail_countdown == 0)                        \
            return set_err(ctx, FOBQ_EHIP, "%s: injected failure (test hook)", what);     \
    } while (0)

struct DeviceGuard {
    int prev = -1;
    bool ok = true;
    explicit DeviceGuard(int dev)
    {
        if (hipGetDevice(&prev) != hipSuccess) prev = -1;
        if (prev != dev) ok = (hipSetDevice(dev) == hipSuccess);
    }
    ~DeviceGuard() { if (prev >= 0) (void)hipSetDevice(prev); }
};

constexpr int64_t MAX_DCOL = 32768;
// L^-1 and L^-T L^-1 fused into the factorization launches against the separate recursive-doubling
// inverse and product, damped inverse of a d x d matrix: 1.1 vs 1.5 ms at d = 2304, even from 4096 to
// 5120 (3.77 vs 3.80, 6.30 vs 6.29 ms), slower beyond (10.5 vs 9.8 ms at 6144, 25.9 vs 21.2 ms at 8192:
// three products per inverse tile against one, and the launches are full without them)
constexpr int FUSED_INVERSE_MAX_D = 4096;
constexpr int64_t MAX_DROW = 65535;
constexpr int I8_MIN_D = 384;     // below: too few 128-wide tiles for the digit traffic to pay (measured on 256- and 288-column layers)
constexpr int64_t I8_MIN_N = 512;

enum { FLAG_NOTPD_H = 0, FLAG_NOTPD_HINV = 1, FLAG_BADPERM = 2, FLAG_COUNT = 4 };

// The flag words; all of them start at zero when the buffer is made.
static int ensure_flags(fobq_ctx* ctx)
{
    static_assert(FLAG_COUNT <= FLAG_WORD_MATE && FLAG_WORD_MATE < FLAG_WORDS, "flag words overlap");
    if (ctx->flags.cap >= FLAG_WORDS * sizeof(int)) return FOBQ_OK;
    FOBQ_TRY(ctx->flags.ensure(FLAG_WORDS * sizeof(int)), "workspace flags");
    FOBQ_TRY(launch_clear_words(ctx->stream, ctx->flags.p, FLAG_WORDS, nullptr, 0), "clear flags");
    ctx->mate_epoch = 0;
    return FOBQ_OK;
}

static int ensure_factor_ws(fobq_ctx* ctx, int64_t d)
{
    const size_t dd = (size_t)d * d * sizeof(double);
    FOBQ_TRY(ctx->Hd.ensure(dd), "workspace Hd");
    FOBQ_TRY(ctx->Linv.ensure(dd), "workspace Linv");
    FOBQ_TRY(ctx->T.ensure(dd), "workspace T");
    FOBQ_TRY(ctx->Hinv.ensure(dd), "workspace Hinv");
    FOBQ_TRY(ctx->U.ensure(dd), "workspace U");
    FOBQ_TRY(ctx->Dblk.ensure((4 * 64 * 64 + 128) * sizeof(double)), "workspace Dblk");
    FOBQ_TRY(ctx->scal.ensure(16 * sizeof(double)), "workspace scal");
    return ensure_flags(ctx);
}

// damped H -> Hinv (upper tiles valid).  Enqueue only.
static int enqueue_inverse(fobq_ctx* ctx, const double* H, int d, double damp, double damp_abs)
{
    hipStream_t s = ctx->stream;
    int* flags = ctx->flags.as<int>();
    double* Hd = ctx->Hd.as<double>();
    double* L = ctx->U.as<double>();       // U is free until the elimination
    double* Linv = ctx->Linv.as<double>();
    bool fused = false;
    {
        StageScope sc(ctx, FOBQ_STAGE_CHOLESKY);
        FOBQ_TRY(launch_damp(s, H, d, damp, damp_abs, Hd, ctx->scal.as<double>()), "damp");
        // the triangular inverse and L^-T L^-1 ride along with the factorization (tiles in the shadow of
        // its critical path) while the launches are small; for large d the extra tiles would slow the launches down by
        // more than the separate recursive-doubling inverse costs
        const bool fused_inverse = d <= FUSED_INVERSE_MAX_D;
        // nothing reads L itself when the inverse rides along: it is not stored then
        FOBQ_TRY(cholesky_lower(ctx, Hd, fused_inverse ? nullptr : L, d, Linv, flags + FLAG_NOTPD_H, fused_inverse ? ctx->T.as<double>() : nullptr,
                                ctx->Hinv.as<double>()), "cholesky");
        fused = fused_inverse;
    }
    {
        StageScope sc(ctx, FOBQ_STAGE_INVERSE);
        if (!fused) {
            FOBQ_TRY(trtri_lower(ctx, L, d, Linv, ctx->T.as<double>()), "trtri");
            FOBQ_TRY(lauum_upper(ctx, Linv, d, ctx->Hinv.as<double>()), "lauum");
        }
    }
    return FOBQ_OK;
}

static int check_opts(fobq_ctx* ctx, const fobq_opts* o, int64_t d_col)
{
    if (!o) return set_err(ctx, FOBQ_EINVAL, "opts is NULL");
    if (o->bits < 2 || o->bits > 8) return set_err(ctx, FOBQ_EINVAL, "bits must be in 2..8 (got %d)", o->bits);
    if (o->group < 0 || (o->group > 0 && d_col % o->group != 0))
        return set_err(ctx, FOBQ_EINVAL, "group (%d) must be 0 or divide d_col (%lld)", o->group, (long long)d_col);
    if (!(o->damp >= 0.0) || !(o->damp_abs >= 0.0)) return set_err(ctx, FOBQ_EINVAL, "damp and damp_abs must be >= 0");
    if (o->order < FOBQ_ORDER_NATURAL || o->order > FOBQ_ORDER_SENSI_DYNAMIC)
        return set_err(ctx, FOBQ_EINVAL, "unknown order %d", o->order);
    if (o->order == FOBQ_ORDER_CUSTOM && !o->perm_in) return set_err(ctx, FOBQ_EINVAL, "order CUSTOM needs perm_in");
    if (o->block < 0 || o->block > 64) return set_err(ctx, FOBQ_EINVAL, "block must be in 0..64 (got %d)", o->block);
    if (o->stop_after < -1 || o->stop_after > d_col)
        return set_err(ctx, FOBQ_EINVAL, "stop_after must be in -1..d_col (got %d)", o->stop_after);
    if (o->reserved != 0) return set_err(ctx, FOBQ_EINVAL, "reserved must be 0");
    return FOBQ_OK;
}

static int check_shape(fobq_ctx* ctx, int64_t d_row, int64_t d_col)
{
    if (d_row < 1 || d_row > MAX_DROW) return set_err(ctx, FOBQ_EINVAL, "d_row must be in 1..%lld", (long long)MAX_DROW);
    if (d_col < 1 || d_col > MAX_DCOL) return set_err(ctx, FOBQ_EINVAL, "d_col must be in 1..%lld", (long long)MAX_DCOL);
    return FOBQ_OK;
}

// sort key: 0 "sensi", 1 "err", 2 "w" (Section 4.1, Table 3)
static int order_kind(const fobq_opts* o)
{
    return (o->order == FOBQ_ORDER_ERR_DESC || o->order == FOBQ_ORDER_ERR_ASC) ? 1
         : (o->order == FOBQ_ORDER_W_DESC || o->order == FOBQ_ORDER_W_ASC)   ? 2 : 0;
}

// Scratch of the ordering stage (grid, column scores, order), either the context's own buffers or the
// library's static scratch array (fobq_sensitivity_static).
struct OrderBufs {
    double* scale; double* zero;   // d_row x G
    double* Spart;                 // sens_chunks(d_row) x d_col
    double* S;                     // d_col
    int* perm; int* invperm;       // d_col
    int* flags;                    // FLAG_COUNT status words
};

static int ensure_order_bufs(fobq_ctx* ctx, int R, int d, int G, OrderBufs* b)
{
    FOBQ_TRY(ctx->scale.ensure((size_t)R * G * sizeof(double)), "workspace scale");
    FOBQ_TRY(ctx->zero.ensure((size_t)R * G * sizeof(double)), "workspace zero");
    FOBQ_TRY(ctx->Spart.ensure((size_t)sens_chunks(R) * d * sizeof(double)), "workspace Spart");
    FOBQ_TRY(ctx->S.ensure((size_t)d * sizeof(double)), "workspace S");
    FOBQ_TRY(ctx->perm.ensure((size_t)d * sizeof(int)), "workspace perm");
    FOBQ_TRY(ctx->invperm.ensure((size_t)d * sizeof(int)), "workspace invperm");
    int rc = ensure_flags(ctx);
    if (rc) return rc;
    *b = OrderBufs{ctx->scale.as<double>(), ctx->zero.as<double>(), ctx->Spart.as<double>(), ctx->S.as<double>(),
                   ctx->perm.as<int>(), ctx->invperm.as<int>(), ctx->flags.as<int>()};
    return FOBQ_OK;
}

// The part of the ordering that needs W only (grid, per-chunk column sums), on stream `st`: in the
// whole-layer path it runs beside the factorization.  Launches only.
static int enqueue_grid_scores(fobq_ctx* ctx, hipStream_t st, const float* W, int R, int d, const fobq_opts* o,
                               const OrderBufs& b, float* scales_out, float* zeros_out, hipEvent_t done = nullptr)
{
    FOBQ_TRY(launch_grid(st, W, R, d, o->bits, o->group, b.scale, b.zero, scales_out, zeros_out), "grid");
    FOBQ_TRY(launch_sens_partial(st, W, R, d, o->bits, o->group, b.scale, b.zero, b.Spart, sens_chunks(R),
                                 order_kind(o), done), "sensitivity");
    return FOBQ_OK;
}

// The rest, on the context's stream: scores (with the diagonal of Hinv, d x d) and the order.  Launches only.
static int enqueue_order(fobq_ctx* ctx, int R, int d, const fobq_opts* o, const double* Hinv, const OrderBufs& b)
{
    hipStream_t s = ctx->stream;
    StageScope sc(ctx, FOBQ_STAGE_ORDER);
    const int ascending = o->order >= FOBQ_ORDER_SENSI_ASC && o->order <= FOBQ_ORDER_W_ASC;
    FOBQ_TRY(launch_sens_reduce(s, b.Spart, sens_chunks(R), d, Hinv, b.S, order_kind(o)), "sensitivity");
    // the dynamic order starts from the identity and exchanges columns step by step
    if (o->order == FOBQ_ORDER_NATURAL || o->order == FOBQ_ORDER_SENSI_DYNAMIC)
        FOBQ_TRY(launch_iota(s, d, b.perm, b.invperm), "order");
    else if (o->order != FOBQ_ORDER_CUSTOM)
        FOBQ_TRY(launch_rank_sort(s, b.S, d, b.perm, b.invperm, ascending), "order");
    else
        FOBQ_TRY(launch_check_perm(s, o->perm_in, d, b.perm, b.invperm, b.flags + FLAG_BADPERM), "order");
    return FOBQ_OK;
}

// pinned host memory that the status flags are read back into (a copy to pageable memory goes through
// a staging buffer); made when the context is created
static int ensure_host_flags(fobq_ctx* ctx)
{
    if (ctx->h_flags) return FOBQ_OK;
    if (hipHostMalloc(reinterpret_cast<void**>(&ctx->h_flags), 64, hipHostMallocDefault) != hipSuccess) {
        ctx->h_flags = nullptr;
        return set_err(ctx, FOBQ_ENOMEM, "cannot allocate pinned host memory for the status flags");
    }
    return FOBQ_OK;
}

// Synchronises the context's stream and turns the status words at `dev_flags` into a status.  Allocates nothing.
static int read_flags(fobq_ctx* ctx, const int* dev_flags)
{
    int* h = ctx->h_flags;
    if (!h) return set_err(ctx, FOBQ_ESTATE, "the context has no host buffer for the status flags");
    FOBQ_TRY(hipMemcpyAsync(h, dev_flags, FLAG_COUNT * sizeof(int), hipMemcpyDeviceToHost, ctx->stream), "read status flags");
    FOBQ_TRY(hipStreamSynchronize(ctx->stream), "synchronize");
    if (h[FLAG_BADPERM]) return set_err(ctx, FOBQ_EINVAL, "perm_in is not a permutation of 0..d_col-1");
    if (h[FLAG_NOTPD_H]) return set_err(ctx, FOBQ_ENOTPD, "damped Hessian is not positive definite (Cholesky pivot <= 0)");
    if (h[FLAG_NOTPD_HINV]) return set_err(ctx, FOBQ_ENOTPD, "shared inverse Hessian lost positive definiteness (elimination pivot <= 0)");
    return FOBQ_OK;
}
static int read_flags(fobq_ctx* ctx) { return read_flags(ctx, ctx->flags.as<int>()); }

// After a failure with work already enqueued: wait for both streams, so that the caller may release its
// buffers and the context's scratch is not in use when the next call starts.  Keeps the first error.
static int drain_after_failure(fobq_ctx* ctx, int rc)
{
    if (ctx->side) (void)hipStreamSynchronize(ctx->side);
    (void)hipStreamSynchronize(ctx->stream);
    ctx->fail_countdown = 0;
    return rc;
}

// ---- static scratch of fobq_sensitivity_static -------------------------------------------------
// One array per GPU, held until the process ends.  The name `scratch` is only a host-side stand-in
// for the symbol: host code uses the address hipGetSymbolAddress returns for the current device.
constexpr int64_t STATIC_MAX_DCOL = 8192;        // columns
constexpr int64_t STATIC_MAX_GRIDS = 131072;     // d_row * G grids
constexpr int64_t STATIC_MAX_SPART = 262144;     // ceil(d_row / 64) * d_col partial column sums
constexpr size_t STATIC_OFF_FLAGS = 0;
constexpr size_t STATIC_OFF_S = 256;
constexpr size_t STATIC_OFF_PERM = STATIC_OFF_S + STATIC_MAX_DCOL * sizeof(double);
constexpr size_t STATIC_OFF_INVPERM = STATIC_OFF_PERM + STATIC_MAX_DCOL * sizeof(int);
constexpr size_t STATIC_OFF_SCALE = STATIC_OFF_INVPERM + STATIC_MAX_DCOL * sizeof(int);
constexpr size_t STATIC_OFF_ZERO = STATIC_OFF_SCALE + STATIC_MAX_GRIDS * sizeof(double);
constexpr size_t STATIC_OFF_SPART = STATIC_OFF_ZERO + STATIC_MAX_GRIDS * sizeof(double);
constexpr size_t STATIC_SCRATCH_BYTES = STATIC_OFF_SPART + STATIC_MAX_SPART * sizeof(double);   // about 4.1 MiB
static_assert(STATIC_OFF_S % 256 == 0 && STATIC_OFF_PERM % 256 == 0 && STATIC_OFF_INVPERM % 256 == 0 &&
              STATIC_OFF_SCALE % 256 == 0 && STATIC_OFF_ZERO % 256 == 0 && STATIC_OFF_SPART % 256 == 0, "alignment");
static_assert(FLAG_COUNT * sizeof(int) <= STATIC_OFF_S, "flag words");

static __device__ __align__(256) __attribute__((used)) unsigned char scratch[STATIC_SCRATCH_BYTES];

constexpr int STATIC_MAX_DEVICES = 64;
static std::mutex g_scratch_mutex;
static unsigned char* g_scratch_ptr[STATIC_MAX_DEVICES] = {nullptr};   // per device: where its copy of `scratch` lives

// With `device` current: the device address of this GPU's copy of `scratch` (looked up once per device).
static int static_scratch_lookup(fobq_ctx* ctx, int device)
{
    if (device < 0 || device >= STATIC_MAX_DEVICES) { ctx->static_scratch = nullptr; return FOBQ_OK; }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return hip_err(ctx, e == hipSuccess ? hipErrorInvalidSymbol : e, "address of the static scratch array");
        g_scratch_ptr[device] = static_cast<unsigned char*>(p);
    }
    ctx->static_scratch = g_scratch_ptr[device];
    return FOBQ_OK;
}

}  // namespace fobq

using namespace fobq;

static std::vector<DevBuf*> all_buffers(fobq_ctx* ctx)
{
    return {&ctx->Hpart, &ctx->H, &ctx->Hd, &ctx->Linv, &ctx->T, &ctx->Hinv, &ctx->A, &ctx->U, &ctx->Un,
            &ctx->Dblk, &ctx->scal, &ctx->flags, &ctx->Wp, &ctx->DT, &ctx->corr, &ctx->codesT, &ctx->scale, &ctx->zero,
            &ctx->S, &ctx->Spart, &ctx->perm, &ctx->invperm, &ctx->lossrow, &ctx->maps_pad, &ctx->i8planes, &ctx->i8sh, &ctx->i8amax, &ctx->batch_pool, &ctx->batch_desc, &ctx->obq, &ctx->hcorr, &ctx->strips};
}

extern "C" {

int fobq_create(fobq_ctx** out, int device, void* hip_stream)
{
    if (!out) return FOBQ_EINVAL;
    *out = nullptr;
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) return FOBQ_EINVAL;
    fobq_ctx* c = new (std::nothrow) fobq_ctx();
    if (!c) return FOBQ_ENOMEM;
    c->device = device;
    c->stream = reinterpret_cast<hipStream_t>(hip_stream);
    // set-up that the entry points which must not allocate rely on: the pinned status buffer and the
    // address of this GPU's copy of the static scratch array
    int rc = FOBQ_OK;
    {
        DeviceGuard g(device);
        rc = g.ok ? FOBQ_OK : FOBQ_EHIP;
        if (!rc) rc = ensure_host_flags(c);
        if (!rc) rc = static_scratch_lookup(c, device);
        int cus = 0;
        if (!rc && hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) == hipSuccess && cus > 0) c->cus = cus;
    }
    if (rc) {
        if (c->h_flags) (void)hipHostFree(c->h_flags);
        delete c;
        return rc;
    }
    *out = c;
    return FOBQ_OK;
}

int fobq_destroy(fobq_ctx* ctx)
{
    if (!ctx) return FOBQ_OK;
    DeviceGuard g(ctx->device);
    (void)hipStreamSynchronize(ctx->stream);
    fold_events(ctx);
    for (hipEvent_t e : ctx->timer.pool) (void)hipEventDestroy(e);
    if (ctx->side) {
        (void)hipStreamSynchronize(ctx->side);
        (void)hipStreamDestroy(ctx->side);
    }
    for (hipEvent_t e : ctx->sync_ev) (void)hipEventDestroy(e);
    for (DevBuf* b : all_buffers(ctx)) b->release();
    if (ctx->h_flags) (void)hipHostFree(ctx->h_flags);
    if (ctx->h_batch) (void)hipHostFree(ctx->h_batch);
    delete ctx;
    return FOBQ_OK;
}

const char* fobq_last_error(const fobq_ctx* ctx) { return ctx ? ctx->err.c_str() : "context is NULL"; }

int fobq_workspace_bytes(fobq_ctx* ctx, int64_t* bytes)
{
    if (!ctx || !bytes) return FOBQ_EINVAL;
    size_t total = 0;
    for (DevBuf* b : all_buffers(ctx)) total += b->cap;
    *bytes = (int64_t)total;
    return FOBQ_OK;
}

int fobq_hessian_set_mode(fobq_ctx* ctx, int mode)
{
    if (!ctx) return FOBQ_EINVAL;
    if (mode != FOBQ_HESSIAN_FP64 && mode != FOBQ_HESSIAN_INT8_SLICES) return set_err(ctx, FOBQ_EINVAL, "unknown Hessian mode %d", mode);
    if (ctx->h_d != 0 && !ctx->h_final && ctx->h_n > 0)
        return set_err(ctx, FOBQ_ESTATE, "the mode cannot change in the middle of an accumulation");
    ctx->h_mode = mode;
    return FOBQ_OK;
}

int fobq_hessian_begin(fobq_ctx* ctx, int64_t d_col)
{
    if (!ctx) return FOBQ_EINVAL;
    if (d_col < 1 || d_col > MAX_DCOL) return set_err(ctx, FOBQ_EINVAL, "d_col must be in 1..%lld", (long long)MAX_DCOL);
    DeviceGuard g(ctx->device);
    if (!g.ok) return set_err(ctx, FOBQ_EHIP, "cannot select device %d", ctx->device);
    const int splits = xxt_pick_splits((int)d_col);
    const size_t dd = (size_t)d_col * d_col * sizeof(double);
    FOBQ_TRY(ctx->Hpart.ensure(dd * splits), "workspace Hpart");
    FOBQ_TRY(ctx->H.ensure(dd), "workspace H");
    {
        int rc = ensure_flags(ctx);
        if (rc) return rc;
    }
    ctx->h_i8_used = false;
    ctx->h_offsets = false;
    ctx->h_zeroed = 0;      // slabs are cleared when a launch first needs them
    ctx->h_conv_c = 0;      // plain or convolution mode is fixed by the first accumulate call
    ctx->h_conv_k = 0;
    ctx->h_d = d_col;
    ctx->h_n = 0;
    ctx->h_splits = splits;
    ctx->h_final = false;
    ctx->err.clear();
    return FOBQ_OK;
}

// clears the slabs of Hpart that a launch over n calibration columns can touch for the first time
static int clear_slabs(fobq_ctx* ctx, int64_t n, bool conv, bool i8 = false)
{
    const int need = i8 ? xxt_i8_slabs_touched((int)ctx->h_d, n, ctx->h_splits)
                        : xxt_slabs_touched((int)ctx->h_d, n, ctx->h_splits, conv);
    if (need > ctx->h_zeroed) {
        FOBQ_TRY(launch_clear_slabs(ctx->stream, ctx->Hpart.as<double>(), (int)ctx->h_d, ctx->h_zeroed, need - ctx->h_zeroed),
                 "clear Hessian accumulator");
        ctx->h_zeroed = need;
    }
    return FOBQ_OK;
}

// Before its first launch an accumulation may still take more slabs than fobq_hessian_begin reserved (the digit-product
// kernel wants some for a wide layer with a long calibration dimension, and for a convolution taken by tap offsets, whose
// few tiles are cut into more pieces each); a failure leaves no accumulation open.
static int grow_i8_slabs(fobq_ctx* ctx, int64_t n_launch, I8Rect rect = I8Rect())
{
    if (ctx->h_n > 0 || ctx->h_zeroed > 0) return FOBQ_OK;
    const int want = xxt_i8_wanted_splits((int)ctx->h_d, n_launch, rect);
    if (want <= ctx->h_splits) return FOBQ_OK;
    const hipError_t e = ctx->Hpart.ensure((size_t)ctx->h_d * ctx->h_d * sizeof(double) * want);
    if (e != hipSuccess) {
        ctx->h_d = 0;
        return hip_err(ctx, e, "workspace Hpart");
    }
    ctx->h_splits = want;
    return FOBQ_OK;
}

int fobq_hessian_accumulate(fobq_ctx* ctx, const float* X, int64_t n, int64_t ld)
{
    if (!ctx) return FOBQ_EINVAL;
    if (ctx->h_d == 0 || ctx->h_final) return set_err(ctx, FOBQ_ESTATE, "hessian_accumulate needs hessian_begin first");
    if (!X) return set_err(ctx, FOBQ_EINVAL, "X is NULL");
    if (n < 0 || ld < n) return set_err(ctx, FOBQ_EINVAL, "need 0 <= n <= ld (n=%lld ld=%lld)", (long long)n, (long long)ld);
    if (ctx->h_conv_c > 0)
        return set_err(ctx, FOBQ_ESTATE, "this accumulation was started with fobq_hessian_accumulate_conv");
    if (n == 0) return FOBQ_OK;
    DeviceGuard g(ctx->device);
    if (!g.ok) return set_err(ctx, FOBQ_EHIP, "cannot select device %d", ctx->device);
    const int d = (int)ctx->h_d;
    // integer slices pay where the fp64 kernel is bound by the matrix pipes: 128-wide tiles and a call long
    // enough to amortise the slicing pass
    const bool i8 = ctx->h_mode == FOBQ_HESSIAN_INT8_SLICES && d >= I8_MIN_D && n >= I8_MIN_N;
    const int64_t blk = i8 ? i8_block_columns(d) : n;        // columns per launch of the int8 kernel
    if (i8) {
        FOBQ_TRY(ctx->i8planes.ensure(i8_planes_bytes(d, n < blk ? n : blk)), "workspace digit planes");
        FOBQ_TRY(ctx->i8sh.ensure((size_t)i8_dpad(d) * sizeof(int)), "workspace row shifts");
        const int grc = grow_i8_slabs(ctx, n < blk ? n : blk);
        if (grc) return grc;
    }
    int rc = clear_slabs(ctx, n < blk ? n : blk, false, i8);
    if (!rc && n > blk && n % blk) rc = clear_slabs(ctx, n % blk, false, i8);    // the shorter last launch
    if (rc) return rc;
    ctx->h_conv_c = -1;
    if (i8) {
        int* nonfinite = ctx->flags.as<int>() + FLAG_WORD_NONFINITE;
        if (!ctx->h_i8_used) FOBQ_TRY(launch_clear_words(ctx->stream, nonfinite, 1, nullptr, 0), "clear flag");
        ctx->h_i8_used = true;
        {
            StageScope sc(ctx, FOBQ_STAGE_SLICE);
            FOBQ_TRY(launch_i8_row_shifts(ctx->stream, X, ld, d, n, ctx->i8sh.as<int>(), nonfinite), "row exponents");
        }
        for (int64_t c0 = 0; c0 < n; c0 += blk) {
            const int64_t nb = n - c0 < blk ? n - c0 : blk;
            {
                StageScope sc(ctx, FOBQ_STAGE_SLICE);
                FOBQ_TRY(launch_i8_slice(ctx->stream, X + c0, ld, d, nb, ctx->i8sh.as<int>(), ctx->i8planes.as<signed char>()),
                         "integer slices");
            }
            FOBQ_TRY(launch_xxt_i8(ctx->stream, ctx->i8planes.as<signed char>(), ctx->i8sh.as<int>(), d, nb,
                                   ctx->Hpart.as<double>(), ctx->h_splits, stage_launch_events(ctx, FOBQ_STAGE_XXT)), "xxt (int8)");
        }
    } else {
        FOBQ_TRY(launch_xxt(ctx->stream, X, ld, d, n, ctx->Hpart.as<double>(), ctx->h_splits,
                            stage_launch_events(ctx, FOBQ_STAGE_XXT)), "xxt");
    }
    ctx->h_n += n;
    return FOBQ_OK;
}

int fobq_hessian_accumulate_conv(fobq_ctx* ctx, const float* maps, int64_t n_img, int64_t h, int64_t w, int64_t c,
                                 int32_t k, int32_t stride, int32_t pad)
{
    if (!ctx) return FOBQ_EINVAL;
    if (ctx->h_d == 0 || ctx->h_final) return set_err(ctx, FOBQ_ESTATE, "hessian_accumulate_conv needs hessian_begin first");
    if (!maps) return set_err(ctx, FOBQ_EINVAL, "maps is NULL");
    if (n_img < 0 || h < 1 || w < 1 || c < 1 || k < 1 || stride < 1 || pad < 0 || h > (1 << 20) || w > (1 << 20) ||
        k > 64 || pad > 64 || stride > 64)
        return set_err(ctx, FOBQ_EINVAL, "bad convolution geometry");
    if (c * (int64_t)k * k != ctx->h_d)
        return set_err(ctx, FOBQ_EINVAL, "channels * k * k = %lld does not match d_col = %lld", (long long)(c * (int64_t)k * k),
                       (long long)ctx->h_d);
    const int64_t ho = (h + 2 * pad - k) / stride + 1, wo = (w + 2 * pad - k) / stride + 1;
    if (h + 2 * pad < k || w + 2 * pad < k || ho < 1 || wo < 1)
        return set_err(ctx, FOBQ_EINVAL, "the kernel does not fit the padded map");
    const int64_t hp = h + 2 * pad, wp = w + 2 * pad;
    if ((k * wp + k) * c >= (1ll << 31))
        return set_err(ctx, FOBQ_EINVAL, "k rows of the padded map (k * (w + 2 pad) * c elements) must stay below 2^31 elements");
    if (ho * wo >= (1ll << 31) - 64 || n_img * ho * wo >= (1ll << 31) - 64)
        return set_err(ctx, FOBQ_EINVAL, "more than 2^31 - 1 output pixels in one call: accumulate in several calls");
    if (ctx->h_conv_c < 0)
        return set_err(ctx, FOBQ_ESTATE, "this accumulation was started with fobq_hessian_accumulate");
    if (ctx->h_conv_c > 0 && (ctx->h_conv_c != c || ctx->h_conv_k != k))
        return set_err(ctx, FOBQ_ESTATE, "channels and kernel size must stay the same within one accumulation");
    const int64_t npix = n_img * ho * wo;
    if (npix == 0) return FOBQ_OK;
    DeviceGuard g(ctx->device);
    if (!g.ok) return set_err(ctx, FOBQ_EHIP, "cannot select device %d", ctx->device);
    const int d = (int)ctx->h_d;
    bool i8 = ctx->h_mode == FOBQ_HESSIAN_INT8_SLICES && d >= I8_MIN_D && npix >= I8_MIN_N;
    // Stride 1 with whole 128-row tiles per tap: the Hessian by tap offsets (hessian_offsets.hip) -- two block rows
    // from the digit-product kernel, the rest by corrections over single rows and columns of the padded maps.
    // Decided by the first call of an accumulation; the later calls have to fit it.
    OffsetTables tab;
    const bool first_call = ctx->h_conv_c == 0;
    bool offsets = false;
    // the tile rows (128 rows each) that hold the rows of the two base taps: two groups of the same size, apart
    const int rect_cb = (int)((c + 127) / 128), rect_gap = (int)((k - 1) * c / 128);
    const bool rect_fits = c % 64 == 0 && rect_gap >= rect_cb && (int)((k * c + 127) / 128) - rect_gap == rect_cb;
    if (first_call ? (i8 && stride == 1 && k >= 2 && rect_fits) : ctx->h_offsets) {
        offsets = stride == 1 && offset_tables_build(k, pad, (int)h, (int)w, &tab);
        if (!offsets && !first_call)
            return set_err(ctx, FOBQ_ESTATE, "this accumulation takes the convolution by tap offsets (stride 1): a later call "
                                             "must have stride 1 and a map of at least k x k");
    }
    if (offsets) i8 = true;
    // 64 channels, 3 x 3: the base taps are the first halves of tile rows 0 and 1, formed as one tile row
    const I8Rect rect = offsets ? I8Rect{rect_cb, rect_gap, (c == 64 && k == 3) ? 1 : 0} : I8Rect();
    const int64_t blk = i8 ? i8_block_columns(d) : npix;
    FOBQ_TRY(ctx->maps_pad.ensure((size_t)(n_img + 1) * hp * wp * c * sizeof(float)), "workspace padded maps");
    if (i8) {
        FOBQ_TRY(ctx->i8planes.ensure(i8_planes_bytes(d, npix < blk ? npix : blk)), "workspace digit planes");
        FOBQ_TRY(ctx->i8sh.ensure((size_t)i8_dpad(d) * sizeof(int)), "workspace row shifts");
        FOBQ_TRY(ctx->i8amax.ensure((size_t)c * sizeof(unsigned)), "workspace channel maxima");
        const int grc = grow_i8_slabs(ctx, npix < blk ? npix : blk, rect);
        if (grc) return grc;
    }
    if (offsets) {
        FOBQ_TRY(ctx->hcorr.ensure((size_t)d * d * sizeof(double)), "workspace corrections");
        FOBQ_TRY(ctx->strips.ensure(offset_strips_bytes(tab.njobs, (int)c)), "workspace strips");
        if (first_call) FOBQ_TRY(launch_clear_words(ctx->stream, ctx->hcorr.p, (int64_t)d * d * 2, nullptr, 0), "clear corrections");
        // the slabs a launch can touch for the first time: the rows of the two base taps, all columns
        auto clear_rect = [&](int64_t n) -> int {
            const int need = xxt_i8_slabs_touched(d, n, ctx->h_splits, rect);
            if (need > ctx->h_zeroed) {
                const int last = d - rect_gap * 128 < rect_cb * 128 ? d - rect_gap * 128 : rect_cb * 128;     // rows past d do not exist
                FOBQ_TRY(launch_clear_slab_rows(ctx->stream, ctx->Hpart.as<double>(), d, ctx->h_zeroed, need - ctx->h_zeroed, 0,
                                                rect_cb * 128, rect_gap * 128, last), "clear Hessian accumulator");
                ctx->h_zeroed = need;
            }
            return FOBQ_OK;
        };
        int rc = clear_rect(npix < blk ? npix : blk);
        if (!rc && npix > blk && npix % blk) rc = clear_rect(npix % blk);
        if (rc) return rc;
    } else {
        int rc = clear_slabs(ctx, npix < blk ? npix : blk, true, i8);
        if (!rc && npix > blk && npix % blk) rc = clear_slabs(ctx, npix % blk, true, i8);    // the shorter last launch
        if (rc) return rc;
    }
    ctx->h_conv_c = (int)c;
    ctx->h_conv_k = k;
    if (first_call) ctx->h_offsets = offsets;
    // the padded copy is stream-ordered: a later call reuses the buffer only after this call's launches
    FOBQ_TRY(launch_pad_maps(ctx->stream, maps, (int)n_img, (int)h, (int)w, (int)c, pad, ctx->maps_pad.as<float>()),
             "pad maps");
    if (i8) {
        // the digits of the unfolded input are written out (1.25 bytes per element of the unfolded X, a block of
        // columns at a time) and the matrix kernel runs on them as it does on a plain X
        int* nonfinite = ctx->flags.as<int>() + FLAG_WORD_NONFINITE;
        if (!ctx->h_i8_used) FOBQ_TRY(launch_clear_words(ctx->stream, nonfinite, 1, nullptr, 0), "clear flag");
        ctx->h_i8_used = true;
        {
            StageScope sc(ctx, FOBQ_STAGE_SLICE);
            FOBQ_TRY(launch_i8_chan_shifts(ctx->stream, ctx->maps_pad.as<float>(), (n_img + 1) * hp * wp, (int)c, d,
                                           ctx->i8amax.as<unsigned>(), ctx->i8sh.as<int>(), nonfinite), "channel exponents");
        }
        for (int64_t p0 = 0; p0 < npix; p0 += blk) {
            const int64_t nb = npix - p0 < blk ? npix - p0 : blk;
            {
                StageScope sc(ctx, FOBQ_STAGE_SLICE);
                FOBQ_TRY(launch_i8_slice_conv(ctx->stream, ctx->maps_pad.as<float>(), (int)n_img, (int)hp, (int)wp, (int)c, k,
                                              stride, (int)ho, (int)wo, npix, p0, nb, ctx->i8sh.as<int>(),
                                              ctx->i8planes.as<signed char>()), "integer slices (convolution)");
            }
            FOBQ_TRY(launch_xxt_i8(ctx->stream, ctx->i8planes.as<signed char>(), ctx->i8sh.as<int>(), d, nb,
                                   ctx->Hpart.as<double>(), ctx->h_splits, stage_launch_events(ctx, FOBQ_STAGE_XXT), rect), "xxt (int8)");
        }
        if (offsets) {
            StageScope sc(ctx, FOBQ_STAGE_FINALIZE);
            FOBQ_TRY(launch_offset_corrections(ctx->stream, ctx->maps_pad.as<float>(), (int)n_img, (int)hp, (int)wp, (int)c, d, tab,
                                               ctx->strips.as<double>(), ctx->hcorr.as<double>()), "offset corrections");
        }
    } else {
        FOBQ_TRY(launch_xxt_conv(ctx->stream, ctx->maps_pad.as<float>(), (int)n_img, (int)hp, (int)wp, (int)c, k, stride,
                                 (int)ho, (int)wo, npix, ctx->Hpart.as<double>(), ctx->h_splits,
                                 stage_launch_events(ctx, FOBQ_STAGE_XXT)), "xxt (convolution)");
    }
    ctx->h_n += npix;
    return FOBQ_OK;
}

int fobq_hessian_form(fobq_ctx* ctx, int32_t* form)
{
    if (!ctx || !form) return FOBQ_EINVAL;
    *form = ctx->h_offsets ? FOBQ_FORM_INT8_TAP_OFFSETS : (ctx->h_i8_used ? FOBQ_FORM_INT8_SLICES : FOBQ_FORM_FP64);
    return FOBQ_OK;
}

int fobq_hessian_finalize(fobq_ctx* ctx, double* H_out)
{
    if (!ctx) return FOBQ_EINVAL;
    if (ctx->h_d == 0) return set_err(ctx, FOBQ_ESTATE, "hessian_finalize needs hessian_begin first");
    if (ctx->h_n == 0) return set_err(ctx, FOBQ_ESTATE, "no calibration columns were accumulated");
    DeviceGuard g(ctx->device);
    if (!g.ok) return set_err(ctx, FOBQ_EHIP, "cannot select device %d", ctx->device);
    const int d = (int)ctx->h_d;
    if (ctx->h_final) {
        // already finalized (the slabs are consumed by then): H is in the context
        if (H_out)
            FOBQ_TRY(hipMemcpyAsync(H_out, ctx->H.p, (size_t)d * d * sizeof(double), hipMemcpyDeviceToDevice, ctx->stream), "copy H");
        return FOBQ_OK;
    }
    {
        StageScope sc(ctx, FOBQ_STAGE_FINALIZE);
        const int* poison = ctx->h_i8_used ? ctx->flags.as<int>() + FLAG_WORD_NONFINITE : nullptr;
        if (ctx->h_offsets)
            FOBQ_TRY(launch_hessian_finalize_offsets(ctx->stream, ctx->Hpart.as<double>(), ctx->h_zeroed, d, 2.0 / (double)ctx->h_n,
                                                     ctx->H.as<double>(), ctx->h_conv_c, ctx->h_conv_k, ctx->hcorr.as<double>(),
                                                     poison), "hessian finalize (tap offsets)");
        else
            FOBQ_TRY(launch_hessian_finalize(ctx->stream, ctx->Hpart.as<double>(), ctx->h_zeroed, d,
                                             2.0 / (double)ctx->h_n, ctx->H.as<double>(), ctx->h_conv_c > 0 ? ctx->h_conv_c : 0,
                                             ctx->h_conv_k * ctx->h_conv_k, poison), "hessian finalize");
        if (H_out)
            FOBQ_TRY(hipMemcpyAsync(H_out, ctx->H.p, (size_t)d * d * sizeof(double), hipMemcpyDeviceToDevice,
                                    ctx->stream), "copy H");
    }
    ctx->h_final = true;
    return FOBQ_OK;
}

int fobq_spd_inverse(fobq_ctx* ctx, const double* H, int64_t d64, double* Hinv)
{
    if (!ctx) return FOBQ_EINVAL;
    if (ctx->pending) return set_err(ctx, FOBQ_ESTATE, "an enqueued layer is waiting for fobq_finish");
    if (!H || !Hinv) return set_err(ctx, FOBQ_EINVAL, "H or Hinv is NULL");
    if (d64 < 1 || d64 > MAX_DCOL) return set_err(ctx, FOBQ_EINVAL, "d must be in 1..%lld", (long long)MAX_DCOL);
    DeviceGuard g(ctx->device);
    if (!g.ok) return set_err(ctx, FOBQ_EHIP, "cannot select device %d", ctx->device);
    const int d = (int)d64;
    int rc = ensure_factor_ws(ctx, d);
    if (rc) return rc;
    rc = [&]() -> int {
        FOBQ_TRY(launch_clear_words(ctx->stream, ctx->flags.p, FLAG_COUNT, nullptr, 0), "clear flags");
        int r = enqueue_inverse(ctx, H, d, 0.0, 0.0);
        if (r) return r;
        // full symmetric copy out of the upper tiles
        FOBQ_TRY(launch_hinv_work(ctx->stream, ctx->Hinv.as<double>(), d, 0, Hinv), "copy Hinv");
        return read_flags(ctx);
    }();
    return (rc && rc != FOBQ_ENOTPD) ? drain_after_failure(ctx, rc) : rc;
}

// argument checks shared by fobq_sensitivity and fobq_sensitivity_static
static int check_sensitivity_args(fobq_ctx* ctx, const float* W, int64_t d_row, int64_t d_col, const double* Hinv,
                                  const fobq_opts* opts, const int32_t* perm)
{
    if (ctx->pending) return set_err(ctx, FOBQ_ESTATE, "an enqueued layer is waiting for fobq_finish");
    if (!W || !Hinv) return set_err(ctx, FOBQ_EINVAL, "W or Hinv is NULL");
    int rc = check_shape(ctx, d_row, d_col);
    if (rc) return rc;
    rc = check_opts(ctx, opts, d_col);
    if (rc) return rc;
    if (perm && opts->order == FOBQ_ORDER_SENSI_DYNAMIC)
        return set_err(ctx, FOBQ_EINVAL, "the dynamic order is only known after the column loop (fobq_quantize_layer returns it)");
    return FOBQ_OK;
}

// launches of the ordering stage on the context's stream with scratch `b`, results copied out by a kernel-free
// device-to-device copy; synchronises and reports the flags
static int run_sensitivity(fobq_ctx* ctx, const float* W, int R, int d, const double* Hinv, const fobq_opts* opts,
                           const OrderBufs& b, double* S, int32_t* perm)
{
    FOBQ_TRY(launch_clear_words(ctx->stream, b.flags, FLAG_COUNT, nullptr, 0), "clear flags");
    int rc = enqueue_grid_scores(ctx, ctx->stream, W, R, d, opts, b, nullptr, nullptr);
    if (rc) return rc;
    rc = enqueue_order(ctx, R, d, opts, Hinv, b);
    if (rc) return rc;
    if (S) FOBQ_TRY(hipMemcpyAsync(S, b.S, (size_t)d * sizeof(double), hipMemcpyDeviceToDevice, ctx->stream), "copy S");
    if (perm) FOBQ_TRY(hipMemcpyAsync(perm, b.perm, (size_t)d * sizeof(int), hipMemcpyDeviceToDevice, ctx->stream), "copy perm");
    return read_flags(ctx, b.flags);
}

int fobq_sensitivity(fobq_ctx* ctx, const float* W, int64_t d_row, int64_t d_col, const double* Hinv,
                     const fobq_opts* opts, double* S, int32_t* perm)
{
    if (!ctx) return FOBQ_EINVAL;
    int rc = check_sensitivity_args(ctx, W, d_row, d_col, Hinv, opts, perm);
    if (rc) return rc;
    DeviceGuard g(ctx->device);
    if (!g.ok) return set_err(ctx, FOBQ_EHIP, "cannot select device %d", ctx->device);
    const int R = (int)d_row, d = (int)d_col;
    OrderBufs b;
    rc = ensure_order_bufs(ctx, R, d, opts->group > 0 ? d / opts->group : 1, &b);
    if (rc) return rc;
    rc = run_sensitivity(ctx, W, R, d, Hinv, opts, b, S, perm);
    return (rc && rc != FOBQ_EINVAL && rc != FOBQ_ENOTPD) ? drain_after_failure(ctx, rc) : rc;
}

int fobq_sensitivity_static(fobq_ctx* ctx, const float* W, int64_t d_row, int64_t d_col, const double* Hinv,
                            const fobq_opts* opts, double* S, int32_t* perm)
{
    if (!ctx) return FOBQ_EINVAL;
    int rc = check_sensitivity_args(ctx, W, d_row, d_col, Hinv, opts, perm);
    if (rc) return rc;
    const int64_t G = opts->group > 0 ? d_col / opts->group : 1;
    if (d_col > STATIC_MAX_DCOL || d_row * G > STATIC_MAX_GRIDS || (int64_t)sens_chunks((int)d_row) * d_col > STATIC_MAX_SPART)
        return set_err(ctx, FOBQ_EINVAL,
                       "fobq_sensitivity_static: shape beyond the static scratch (needs d_col <= %lld, d_row * groups <= %lld, "
                       "ceil(d_row / 64) * d_col <= %lld); use fobq_sensitivity",
                       (long long)STATIC_MAX_DCOL, (long long)STATIC_MAX_GRIDS, (long long)STATIC_MAX_SPART);
    if (ctx->profiling) return set_err(ctx, FOBQ_ESTATE, "fobq_sensitivity_static: stage timing creates events; turn it off");
    unsigned char* base = ctx->static_scratch;
    if (!base) return set_err(ctx, FOBQ_ESTATE, "no static scratch array on device %d", ctx->device);
    DeviceGuard g(ctx->device);
    if (!g.ok) return set_err(ctx, FOBQ_EHIP, "cannot select device %d", ctx->device);
    const OrderBufs b{reinterpret_cast<double*>(base + STATIC_OFF_SCALE), reinterpret_cast<double*>(base + STATIC_OFF_ZERO),
                      reinterpret_cast<double*>(base + STATIC_OFF_SPART), reinterpret_cast<double*>(base + STATIC_OFF_S),
                      reinterpret_cast<int*>(base + STATIC_OFF_PERM), reinterpret_cast<int*>(base + STATIC_OFF_INVPERM),
                      reinterpret_cast<int*>(base + STATIC_OFF_FLAGS)};
    rc = run_sensitivity(ctx, W, (int)d_row, (int)d_col, Hinv, opts, b, S, perm);
    return (rc && rc != FOBQ_EINVAL && rc != FOBQ_ENOTPD) ? drain_after_failure(ctx, rc) : rc;
}

int fobq_obq_rows(fobq_ctx* ctx, const float* W, int64_t d_row, int64_t d_col, const double* Hinv, const fobq_opts* opts,
                  int64_t row_begin, int64_t row_end, uint8_t* codes, float* Q, int32_t* order, double* lossrow)
{
    if (!ctx) return FOBQ_EINVAL;
    if (ctx->pending) return set_err(ctx, FOBQ_ESTATE, "an enqueued layer is waiting for fobq_finish");
    if (!W || !Hinv || !codes || !Q || !lossrow) return set_err(ctx, FOBQ_EINVAL, "W, Hinv, codes, Q or lossrow is NULL");
    int rc = check_shape(ctx, d_row, d_col);
    if (rc) return rc;
    rc = check_opts(ctx, opts, d_col);
    if (rc) return rc;
    if (d_col > OBQ_MAX_D)
        return set_err(ctx, FOBQ_EINVAL, "fobq_obq_rows is a baseline for small layers: d_col <= %d (got %lld)", OBQ_MAX_D, (long long)d_col);
    if (row_begin < 0 || row_end > d_row || row_begin > row_end)
        return set_err(ctx, FOBQ_EINVAL, "rows %lld..%lld are not inside 0..%lld", (long long)row_begin, (long long)row_end, (long long)d_row);
    if (row_begin == row_end) return FOBQ_OK;
    DeviceGuard g(ctx->device);
    if (!g.ok) return set_err(ctx, FOBQ_EHIP, "cannot select device %d", ctx->device);
    const int R = (int)d_row, d = (int)d_col, G = opts->group > 0 ? d / opts->group : 1;
    // rows per launch: at most 4 GiB of running inverses at a time
    const size_t per_row = obq_scratch_per_row(d);
    const int64_t rows_total = row_end - row_begin;
    int64_t batch = per_row ? (int64_t)(((size_t)4 << 30) / per_row) : rows_total;
    batch = batch < 1 ? 1 : (batch > rows_total ? rows_total : batch);
    FOBQ_TRY(ctx->scale.ensure((size_t)R * G * sizeof(double)), "workspace scale");
    FOBQ_TRY(ctx->zero.ensure((size_t)R * G * sizeof(double)), "workspace zero");
    FOBQ_TRY(ctx->obq.ensure(per_row ? per_row * (size_t)batch : 256), "workspace of the per-row inverses");
    rc = ensure_flags(ctx);
    if (rc) return rc;
    hipStream_t s = ctx->stream;
    int* flags = ctx->flags.as<int>();
    rc = [&]() -> int {
        FOBQ_TRY(launch_clear_words(s, flags, FLAG_COUNT, nullptr, 0), "clear flags");
        FOBQ_TRY(launch_grid(s, W, R, d, opts->bits, opts->group, ctx->scale.as<double>(), ctx->zero.as<double>(), nullptr, nullptr), "grid");
        for (int64_t r0 = row_begin; r0 < row_end; r0 += batch) {
            const int rows = (int)(row_end - r0 < batch ? row_end - r0 : batch);
            FOBQ_TRY(launch_obq_rows(s, W, d, opts->bits, opts->group, Hinv, ctx->scale.as<double>(), ctx->zero.as<double>(), (int)r0,
                                     rows, ctx->obq.as<double>(), codes, Q, order, lossrow, flags + FLAG_NOTPD_HINV), "per-row baseline");
        }
        return read_flags(ctx);
    }();
    if (rc == FOBQ_ENOTPD) return set_err(ctx, FOBQ_ENOTPD, "a row's own inverse Hessian met a pivot <= 0 (is Hinv positive definite?)");
    return (rc && rc != FOBQ_EINVAL) ? drain_after_failure(ctx, rc) : rc;
}

int fobq_debug_offset_tables(int32_t k, int32_t pad, int64_t h, int64_t w, int32_t* out, int64_t cap, int64_t* used)
{
    if (!out || !used || k < 1 || pad < 0 || h < 1 || w < 1 || h > (1 << 20) || w > (1 << 20) || pad > (1 << 10))
        return FOBQ_EINVAL;
    OffsetTables tab;
    if (!offset_tables_build(k, pad, (int)h, (int)w, &tab)) return FOBQ_ESTATE;
    const int64_t need = 3 + 6 * (int64_t)tab.njobs + 4 * (int64_t)tab.npairs + 2 * (int64_t)tab.nterms;
    *used = need;
    if (need > cap) return FOBQ_EINVAL;
    int32_t* o = out;
    *o++ = tab.njobs; *o++ = tab.npairs; *o++ = tab.nterms;
    for (int j = 0; j < tab.njobs; ++j) {
        const OffsetJob& b = tab.jobs[j];
        *o++ = b.kind; *o++ = b.coord; *o++ = b.start; *o++ = b.len; *o++ = b.dy; *o++ = b.dx;
    }
    for (int p = 0; p < tab.npairs; ++p) {
        *o++ = tab.pair_ta[p]; *o++ = tab.pair_tb[p]; *o++ = tab.pair_begin[p]; *o++ = tab.pair_begin[p + 1];
    }
    for (int t = 0; t < tab.nterms; ++t) { *o++ = tab.term_job[t]; *o++ = tab.term_sign[t]; }
    return FOBQ_OK;
}

int fobq_debug_fail_after(fobq_ctx* ctx, int n)
{
    if (!ctx || n < 0) return FOBQ_EINVAL;
    ctx->fail_countdown = n;
    return FOBQ_OK;
}

// What one layer's launches need, fixed before the first of them is enqueued.
struct LayerPlan {
    const float* W; const double* H; const fobq_opts* opts; const fobq_out* out;
    int R, d, G, steps, block, Rp, nblocks;
    bool dynamic;
    OrderBufs ob;
};

// events of a layer in ctx->sync_ev: the fork / join pair that sends the grid and the W-only part of the
// scores to the side stream and back, then one "pivot rows ready" event per column block, then the start
// and the end of the column loop.  No event serves two purposes within a layer.
enum { EV_FORK = 0, EV_JOIN = 1, EV_ROWS0 = 2 };

// All launches of a layer (no allocation in here: a failure leaves work in flight, see quantize_enqueue).
static int enqueue_layer_launches(fobq_ctx* ctx, const LayerPlan& p)
{
    hipStream_t s = ctx->stream;
    const fobq_opts* opts = p.opts;
    const fobq_out* out = p.out;
    const int R = p.R, d = p.d, G = p.G, steps = p.steps, block = p.block, Rp = p.Rp, nblocks = p.nblocks;
    // grid and the W-only part of the column scores: on the side stream, beside the factorization.  The
    // events that order the streams ride on launches (see gemm64's `done`), here on the clearing kernel.
    FOBQ_TRY(launch_clear_words(s, ctx->flags.p, FLAG_COUNT, ctx->lossrow.p, 2 * (int64_t)R, ctx->sync_ev[EV_FORK]),
             "clear flags and loss");
    FOBQ_TRY(hipStreamWaitEvent(ctx->side, ctx->sync_ev[EV_FORK], 0), "stream wait");
    int rc = enqueue_grid_scores(ctx, ctx->side, p.W, R, d, opts, p.ob, out->scales, out->zeros, ctx->sync_ev[EV_JOIN]);
    if (rc) return rc;
    // damp, Cholesky, inverse
    rc = enqueue_inverse(ctx, p.H, d, opts->damp, opts->damp_abs);
    if (rc) return rc;
    FOBQ_TRY(hipStreamWaitEvent(s, ctx->sync_ev[EV_JOIN], 0), "stream wait");
    // column scores, order
    rc = enqueue_order(ctx, R, d, opts, ctx->Hinv.as<double>(), p.ob);
    if (rc) return rc;
    // blocked path: the event that lets the column loop's stream start rides on the gather launch
    hipEvent_t ev_start = block != 1 ? ctx->sync_ev[EV_ROWS0 + nblocks] : nullptr;
    hipEvent_t ev_done = block != 1 ? ctx->sync_ev[EV_ROWS0 + nblocks + 1] : nullptr;
    {
        StageScope sc(ctx, FOBQ_STAGE_PERMUTE);
        FOBQ_TRY(launch_gather(s, p.W, R, d, p.ob.perm, ctx->Hinv.as<double>(), ctx->Wp.as<double>(),
                               ctx->A.as<double>(), ev_start), "permute");
    }
    double* A = ctx->A.as<double>();
    double* Wp = ctx->Wp.as<double>();
    const double* scale = p.ob.scale;
    const double* zero = p.ob.zero;
    int* perm = p.ob.perm;
    uint8_t* codesT = ctx->codesT.as<uint8_t>();
    double* lossrow = ctx->lossrow.as<double>();

    if (block == 1) {
        // Eq. 9 / 11 and Eq. 12 one column at a time
        StageScope sc(ctx, FOBQ_STAGE_COLUMNS);
        int* pivot_flag = ctx->flags.as<int>() + FLAG_NOTPD_HINV;
        for (int t = 0; t < steps; ++t) {
            if (p.dynamic)
                FOBQ_TRY(launch_dyn_select(s, Wp, R, d, t, A, scale, zero, G, opts->group, perm, opts->bits,
                                           p.ob.Spart, sens_chunks(R)), "column choice");
            FOBQ_TRY(launch_step(s, Wp, R, d, t, A, scale, zero, G, opts->group, perm, opts->bits, codesT, Rp, lossrow,
                                 pivot_flag), "column step");
        }
        if (p.dynamic) FOBQ_TRY(launch_invert_perm(s, perm, d, p.ob.invperm), "order");
    } else {
        double* U = ctx->U.as<double>();
        double* Un = ctx->Un.as<double>();
        double* DT = ctx->DT.as<double>();
        // Eq. 12 does not involve W: the elimination runs ahead on the context's stream and the
        // column loop follows on the side stream, block k as soon as the pivot rows of block k exist
        // (both are chains of short dependent launches that leave most of the GPU idle).
        hipStream_t side = ctx->side;
        std::vector<hipEvent_t> rows_ready(ctx->sync_ev.begin() + EV_ROWS0, ctx->sync_ev.begin() + EV_ROWS0 + nblocks);
        FOBQ_TRY(hipStreamWaitEvent(side, ev_start, 0), "stream wait");
        {
            StageScope sc(ctx, FOBQ_STAGE_ELIMINATE);
            FOBQ_TRY(eliminate_blocked(ctx, A, d, steps, block, U, Un, ctx->flags.as<int>() + FLAG_NOTPD_HINV,
                                       &rows_ready), "eliminate");
        }
        {
            // One launch per block: its chain, and beside it the deferred compensation of the block before
            // for the columns from the next block on (see col_block_kernel); the event that hands the
            // result back to the context's stream rides on the last launch.
            StageScope sc(ctx, FOBQ_STAGE_COLUMNS, side);
            double* corr[2] = {ctx->corr.as<double>(), ctx->corr.as<double>() + (size_t)R * 64};
            int k = 0;
            int po = 0, pnb = 0;                 // the block before
            for (int o = 0; o < steps; o += block, ++k) {
                const int nb = (block < steps - o) ? block : steps - o;
                const bool has_next = o + nb < steps;
                const int nb_next = has_next ? ((block < steps - o - nb) ? block : steps - o - nb) : 0;
                FOBQ_TRY(hipStreamWaitEvent(side, rows_ready[k], 0), "stream wait");
                // the last launch of the loop: this one, unless columns are left over right of the last block
                const bool last = !has_next && o + nb >= d;
                FOBQ_TRY(launch_col_block(side, Wp, R, d, o, nb, Un, U, scale, zero, G, opts->group, perm, opts->bits,
                                          codesT, DT, Rp, lossrow, k > 0 ? corr[(k - 1) & 1] : nullptr,
                                          has_next ? corr[k & 1] : nullptr, nb_next, po, pnb, o + nb,
                                          last ? ev_done : nullptr), "column block");
                po = o; pnb = nb;
            }
            // stop_after: the last processed block's compensation of all the columns that stay unprocessed
            if (k == 0 || po + pnb < d)
                FOBQ_TRY(launch_col_block(side, Wp, R, d, 0, 0, Un, U, scale, zero, G, opts->group, perm, opts->bits,
                                          codesT, DT, Rp, lossrow, nullptr, nullptr, 0, po, pnb, po + pnb, ev_done),
                         "column block update");
        }
        FOBQ_TRY(hipStreamWaitEvent(s, ev_done, 0), "stream wait");
    }
    {
        StageScope sc(ctx, FOBQ_STAGE_EMIT);
        if (out->codes || out->Q)
            FOBQ_TRY(launch_emit(s, codesT, Rp, R, d, steps, p.ob.invperm, scale, zero, G, opts->group,
                                 out->codes, out->Q, lossrow, out->loss), "emit");
        else if (out->loss) FOBQ_TRY(launch_loss(s, lossrow, R, out->loss), "loss");
        if (out->perm)
            FOBQ_TRY(hipMemcpyAsync(out->perm, perm, (size_t)d * sizeof(int), hipMemcpyDeviceToDevice, s), "copy perm");
        if (out->W_work)
            FOBQ_TRY(hipMemcpyAsync(out->W_work, Wp, (size_t)R * d * sizeof(double), hipMemcpyDeviceToDevice, s), "copy W_work");
        if (out->Hinv_work) FOBQ_TRY(launch_hinv_work(s, A, d, steps, out->Hinv_work), "copy Hinv_work");
    }
    return FOBQ_OK;
}

// everything of fobq_quantize_layer except the final synchronisation and status read
static int quantize_enqueue(fobq_ctx* ctx, const float* W, int64_t d_row, int64_t d_col, const double* H,
                            const fobq_opts* opts, const fobq_out* out)
{
    if (!ctx) return FOBQ_EINVAL;
    if (ctx->pending)
        return set_err(ctx, FOBQ_ESTATE, "a layer enqueued with fobq_quantize_layer_enqueue is waiting for fobq_finish");
    if (!W) return set_err(ctx, FOBQ_EINVAL, "W is NULL");
    if (!out) return set_err(ctx, FOBQ_EINVAL, "out is NULL");
    int rc = check_shape(ctx, d_row, d_col);
    if (rc) return rc;
    rc = check_opts(ctx, opts, d_col);
    if (rc) return rc;
    if (!H) {
        if (!ctx->h_final) return set_err(ctx, FOBQ_ESTATE, "H is NULL and no finalized Hessian is held by the context");
        if (ctx->h_d != d_col)
            return set_err(ctx, FOBQ_EINVAL, "accumulated Hessian has d_col=%lld, layer has %lld", (long long)ctx->h_d, (long long)d_col);
        H = ctx->H.as<double>();
    }
    DeviceGuard g(ctx->device);
    if (!g.ok) return set_err(ctx, FOBQ_EHIP, "cannot select device %d", ctx->device);
    ctx->err.clear();

    LayerPlan p;
    p.W = W; p.H = H; p.opts = opts; p.out = out;
    p.R = (int)d_row; p.d = (int)d_col;
    p.G = opts->group > 0 ? p.d / opts->group : 1;
    p.steps = opts->stop_after < 0 ? p.d : opts->stop_after;
    p.dynamic = opts->order == FOBQ_ORDER_SENSI_DYNAMIC;
    p.block = p.dynamic ? 1 : (opts->block == 0 ? 64 : opts->block);   // re-sorting needs W after every column
    p.Rp = (p.R + 63) / 64 * 64;
    p.nblocks = p.block == 1 ? 0 : (p.steps + p.block - 1) / p.block;
    const size_t dd = (size_t)p.d * p.d * sizeof(double);

    // Every allocation (scratch growth, streams, events) comes before the first launch: scratch growth may
    // free a buffer, and a failure in here leaves nothing in flight.
    rc = ensure_factor_ws(ctx, p.d);
    if (rc) return rc;
    FOBQ_TRY(ctx->A.ensure(dd), "workspace A");
    FOBQ_TRY(ctx->Un.ensure(dd), "workspace Un");
    FOBQ_TRY(ctx->Wp.ensure((size_t)p.R * p.d * sizeof(double)), "workspace Wp");
    FOBQ_TRY(ctx->DT.ensure((size_t)p.d * p.Rp * sizeof(double)), "workspace DT");
    FOBQ_TRY(ctx->corr.ensure(2 * (size_t)p.R * 64 * sizeof(double)), "workspace corr");
    FOBQ_TRY(ctx->codesT.ensure((size_t)p.d * p.Rp), "workspace codesT");
    FOBQ_TRY(ctx->lossrow.ensure((size_t)p.R * sizeof(double)), "workspace lossrow");
    rc = ensure_order_bufs(ctx, p.R, p.d, p.G, &p.ob);
    if (rc) return rc;
    rc = ensure_sync_events(ctx, (size_t)EV_ROWS0 + p.nblocks + 2);
    if (rc) return rc;

    rc = enqueue_layer_launches(ctx, p);
    // a failure past this point has work in flight on both streams that reads W / H and writes the outputs
    // and the context's scratch: wait for it, so that the caller may free its buffers and use the context again
    return rc ? drain_after_failure(ctx, rc) : FOBQ_OK;
}

// carve `bytes` (rounded up to 256) out of a pool laid out from `*off`; base == null: only the size is wanted
static void* pool_take(unsigned char* base, size_t* off, size_t bytes)
{
    void* p = base ? base + *off : nullptr;
    *off += (bytes + 255) & ~size_t(255);
    return p;
}

// scratch pointers of one batched layer (or, with base == null, just the size it needs)
static void batch_layout(BatchLayer* L, unsigned char* base, size_t* off)
{
    const size_t dd = (size_t)L->d * L->d * sizeof(double);
    double** mats[] = {&L->Hd, &L->Linv, &L->T, &L->Hinv, &L->A, &L->U, &L->Un};
    for (double** m : mats) *m = static_cast<double*>(pool_take(base, off, dd));
    L->Gs = static_cast<double*>(pool_take(base, off, 64 * 64 * sizeof(double)));
    L->rinv = static_cast<double*>(pool_take(base, off, 64 * sizeof(double)));
    L->Wp = static_cast<double*>(pool_take(base, off, (size_t)L->R * L->d * sizeof(double)));
    L->DT = static_cast<double*>(pool_take(base, off, (size_t)L->d * L->Rp * sizeof(double)));
    L->codesT = static_cast<uint8_t*>(pool_take(base, off, (size_t)L->d * L->Rp));
    L->scale = static_cast<double*>(pool_take(base, off, (size_t)L->R * L->G * sizeof(double)));
    L->zero = static_cast<double*>(pool_take(base, off, (size_t)L->R * L->G * sizeof(double)));
    L->S = static_cast<double*>(pool_take(base, off, (size_t)L->d * sizeof(double)));
    L->Spart = static_cast<double*>(pool_take(base, off, (size_t)L->chunks * L->d * sizeof(double)));
    L->lossrow = static_cast<double*>(pool_take(base, off, (size_t)L->R * sizeof(double)));
    L->perm = static_cast<int*>(pool_take(base, off, (size_t)L->d * sizeof(int)));
    L->invperm = static_cast<int*>(pool_take(base, off, (size_t)L->d * sizeof(int)));
    L->flags = static_cast<int*>(pool_take(base, off, 4 * sizeof(int)));
}

int fobq_quantize_layers_batched(fobq_ctx* ctx, int32_t n_layers, const fobq_layer* layers, const fobq_opts* opts)
{
    if (!ctx) return FOBQ_EINVAL;
    if (ctx->pending)
        return set_err(ctx, FOBQ_ESTATE, "a layer enqueued with fobq_quantize_layer_enqueue is waiting for fobq_finish");
    if (n_layers < 0 || n_layers > BATCH_MAX_LAYERS)
        return set_err(ctx, FOBQ_EINVAL, "n_layers must be in 0..%d (got %d)", BATCH_MAX_LAYERS, n_layers);
    if (n_layers == 0) return FOBQ_OK;
    if (!layers) return set_err(ctx, FOBQ_EINVAL, "layers is NULL");
    if (!opts) return set_err(ctx, FOBQ_EINVAL, "opts is NULL");
    if (opts->order == FOBQ_ORDER_SENSI_DYNAMIC || opts->order == FOBQ_ORDER_CUSTOM)
        return set_err(ctx, FOBQ_EINVAL, "a batched call takes the orders that are computed from W and Hinv or NATURAL "
                                         "(one perm_in cannot serve layers of different d_col; the dynamic order runs one column per launch)");
    if (opts->block != 0 && opts->block != 64) return set_err(ctx, FOBQ_EINVAL, "a batched call uses the default block width");
    if (opts->stop_after != -1) return set_err(ctx, FOBQ_EINVAL, "a batched call processes all columns (stop_after must be -1)");
    for (int l = 0; l < n_layers; ++l) {
        const fobq_layer& in = layers[l];
        if (!in.W || !in.H) return set_err(ctx, FOBQ_EINVAL, "layer %d: W or H is NULL", l);
        int rc = check_shape(ctx, in.d_row, in.d_col);
        if (!rc) rc = check_opts(ctx, opts, in.d_col);
        if (rc) { ctx->err = "layer " + std::to_string(l) + ": " + ctx->err; return rc; }
        if (in.d_col > BATCH_MAX_D)
            return set_err(ctx, FOBQ_EINVAL, "layer %d: d_col = %lld; a batched call takes layers of up to %d columns", l,
                           (long long)in.d_col, BATCH_MAX_D);
        if (in.out.W_work || in.out.Hinv_work)
            return set_err(ctx, FOBQ_EINVAL, "layer %d: W_work / Hinv_work are not available from a batched call", l);
    }
    DeviceGuard g(ctx->device);
    if (!g.ok) return set_err(ctx, FOBQ_EHIP, "cannot select device %d", ctx->device);
    ctx->err.clear();

    // descriptors: pinned host staging (also receives the status words), device copy, scratch pool
    const size_t desc_bytes = (size_t)BATCH_MAX_LAYERS * sizeof(BatchLayer), flag_bytes = (size_t)BATCH_MAX_LAYERS * 4 * sizeof(int);
    if (!ctx->h_batch && hipHostMalloc(&ctx->h_batch, desc_bytes + flag_bytes, hipHostMallocDefault) != hipSuccess) {
        ctx->h_batch = nullptr;
        return set_err(ctx, FOBQ_ENOMEM, "cannot allocate pinned host memory for the batch descriptors");
    }
    FOBQ_TRY(ctx->batch_desc.ensure(desc_bytes + flag_bytes), "workspace batch descriptors");
    BatchLayer* hd = static_cast<BatchLayer*>(ctx->h_batch);
    int max_pairs = 1, max_chunks = 1, max_rows = 1;
    size_t pool = 0;
    for (int l = 0; l < n_layers; ++l) {
        const fobq_layer& in = layers[l];
        BatchLayer& L = hd[l];
        L = BatchLayer{};
        L.W = in.W; L.H = in.H;
        L.R = (int)in.d_row; L.d = (int)in.d_col;
        L.G = opts->group > 0 ? L.d / opts->group : 1;
        L.gs = opts->group > 0 ? opts->group : L.d;
        L.Rp = (L.R + 63) / 64 * 64;
        L.chunks = sens_chunks(L.R);
        L.maxq = (double)((1 << opts->bits) - 1);
        L.damp = opts->damp; L.damp_abs = opts->damp_abs;
        L.order = opts->order; L.kind = order_kind(opts);
        L.ascending = opts->order >= FOBQ_ORDER_SENSI_ASC && opts->order <= FOBQ_ORDER_W_ASC;
        L.codes = in.out.codes; L.scales = in.out.scales; L.zeros = in.out.zeros; L.Q = in.out.Q;
        L.perm_out = in.out.perm; L.loss = in.out.loss;
        batch_layout(&L, nullptr, &pool);
        max_pairs = std::max(max_pairs, L.R * L.G);
        max_chunks = std::max(max_chunks, L.chunks);
        max_rows = std::max(max_rows, L.R);
    }
    FOBQ_TRY(ctx->batch_pool.ensure(pool), "workspace batch pool");
    size_t off = 0;
    for (int l = 0; l < n_layers; ++l) batch_layout(&hd[l], ctx->batch_pool.as<unsigned char>(), &off);

    hipStream_t s = ctx->stream;
    const BatchLayer* dl = ctx->batch_desc.as<BatchLayer>();
    int rc = [&]() -> int {
        FOBQ_TRY(hipMemcpyAsync(ctx->batch_desc.p, hd, (size_t)n_layers * sizeof(BatchLayer), hipMemcpyHostToDevice, s),
                 "upload batch descriptors");
        FOBQ_TRY(launch_batch_grid(s, dl, n_layers, max_pairs), "grid (batch)");
        FOBQ_TRY(launch_batch_sens_partial(s, dl, n_layers, max_chunks), "sensitivity (batch)");
        FOBQ_TRY(launch_batch_inverse(s, dl, n_layers), "inverse (batch)");
        FOBQ_TRY(launch_batch_order(s, dl, n_layers), "order (batch)");
        FOBQ_TRY(launch_batch_eliminate(s, dl, n_layers), "eliminate (batch)");
        FOBQ_TRY(launch_batch_columns(s, dl, n_layers, max_rows), "column loop (batch)");
        FOBQ_TRY(launch_batch_loss(s, dl, n_layers), "loss (batch)");
        // status words of every layer, gathered by one strided copy into the staging area behind the descriptors
        int* hflags = reinterpret_cast<int*>(static_cast<unsigned char*>(ctx->h_batch) + desc_bytes);
        for (int l = 0; l < n_layers; ++l)
            FOBQ_TRY(hipMemcpyAsync(hflags + 4 * l, hd[l].flags, 4 * sizeof(int), hipMemcpyDeviceToHost, s), "read status flags");
        FOBQ_TRY(hipStreamSynchronize(s), "synchronize");
        for (int l = 0; l < n_layers; ++l) {
            if (hflags[4 * l + FLAG_NOTPD_H])
                return set_err(ctx, FOBQ_ENOTPD, "layer %d: damped Hessian is not positive definite (Cholesky pivot <= 0)", l);
            if (hflags[4 * l + FLAG_NOTPD_HINV])
                return set_err(ctx, FOBQ_ENOTPD, "layer %d: shared inverse Hessian lost positive definiteness (elimination pivot <= 0)", l);
        }
        return FOBQ_OK;
    }();
    return (rc && rc != FOBQ_ENOTPD) ? drain_after_failure(ctx, rc) : rc;
}

int fobq_quantize_layer(fobq_ctx* ctx, const float* W, int64_t d_row, int64_t d_col, const double* H,
                        const fobq_opts* opts, const fobq_out* out)
{
    int rc = quantize_enqueue(ctx, W, d_row, d_col, H, opts, out);
    if (rc) return rc;
    return read_flags(ctx);
}

int fobq_quantize_layer_enqueue(fobq_ctx* ctx, const float* W, int64_t d_row, int64_t d_col, const double* H,
                                const fobq_opts* opts, const fobq_out* out)
{
    int rc = quantize_enqueue(ctx, W, d_row, d_col, H, opts, out);
    if (rc) return rc;
    ctx->pending = true;
    return FOBQ_OK;
}

int fobq_finish(fobq_ctx* ctx)
{
    if (!ctx) return FOBQ_EINVAL;
    DeviceGuard g(ctx->device);
    if (!g.ok) return set_err(ctx, FOBQ_EHIP, "cannot select device %d", ctx->device);
    if (!ctx->pending) {
        FOBQ_TRY(hipStreamSynchronize(ctx->stream), "synchronize");
        return FOBQ_OK;
    }
    ctx->pending = false;
    return read_flags(ctx);
}

int fobq_profile_enable(fobq_ctx* ctx, int on)
{
    if (!ctx) return FOBQ_EINVAL;
    ctx->profiling = on == 1 ? ~0u : (unsigned)on >> 1;
    return FOBQ_OK;
}

int fobq_profile_get(fobq_ctx* ctx, int stage, double* ms, int64_t* intervals)
{
    if (!ctx) return FOBQ_EINVAL;
    if (stage < 0 || stage >= FOBQ_STAGE_COUNT) return set_err(ctx, FOBQ_EINVAL, "unknown stage %d", stage);
    DeviceGuard g(ctx->device);
    FOBQ_TRY(hipStreamSynchronize(ctx->stream), "synchronize");
    fold_events(ctx);
    if (ms) *ms = ctx->timer.ms[stage];
    if (intervals) *intervals = ctx->timer.launches[stage];
    return FOBQ_OK;
}

int fobq_profile_reset(fobq_ctx* ctx)
{
    if (!ctx) return FOBQ_EINVAL;
    DeviceGuard g(ctx->device);
    FOBQ_TRY(hipStreamSynchronize(ctx->stream), "synchronize");
    fold_events(ctx);
    for (int st = 0; st < FOBQ_STAGE_COUNT; ++st) {
        ctx->timer.ms[st] = 0.0;
        ctx->timer.launches[st] = 0;
    }
    return FOBQ_OK;
}

}  // extern "C"
