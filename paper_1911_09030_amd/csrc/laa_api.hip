// C-ABI layer of the Local AdaAlter library: handle, argument checks, the step counter t' of
// Algorithm 3 (arXiv 1911.09030) and kernel dispatch.  No arithmetic of the method lives here
// except the scalars handed to the kernels (eta_t, t' eps^2).
#include "../../include/laa.h"
#include "laa_kernels.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <vector>

struct laa_ctx {
    int64_t d = 0, pitch = 0;
    int32_t W = 0, H = 0;
    double eta = 0, eps = 0, b0 = 1.0;
    int64_t warmup_steps = 0;
    int32_t algo = LAA_ALGO_LOCAL_ADAALTER;
    float *x = nullptr, *acc = nullptr, *snap = nullptr;
    hipStream_t stream = nullptr;
    bool attached = false, vec4 = false, gen_aligned16 = true;
    int32_t wt = 1;
    bool split = false;     // one worker per thread block in non-sync steps (laa_set_tile(h, 0))
    bool lazy = false;      // keep the post-sync state once (row 0 of x, snap) until the next step
    bool collapsed = false; // rows 1.. of x and all of acc are stale; row 0 of x and snap hold the common state
    int64_t t = 0;          // iterations done
    int32_t s = 0;          // local steps since the last sync (t' - 1 before a step)
    // generator
    int32_t gen_mode = 0, off_mode = 0;
    uint64_t seed = 0;
    int64_t col0 = 0;                 // global indices of column 0 and worker 0 (generator counters)
    int32_t w0 = 0;
    const float *a = nullptr, *xstar = nullptr, *off = nullptr;
    float noise_scale = 0, off_scale = 0;
    // sparse bookkeeping (library-owned device memory)
    int64_t n_rows = 0;
    int32_t row_len = 0;
    uint32_t *dirty = nullptr;
    int32_t *dirty_list = nullptr;
    bool coalesce = false;            // sparse steps add up rows that a worker lists more than once
    uint64_t *sort_keys = nullptr;    // [W][k] sorted (row, position) keys of the coalescing step
    int64_t sort_cap = 0;             // keys allocated
    float *partials = nullptr;        // partial sums of rows listed many times
    int64_t partial_cap = 0;          // floats allocated
    uint32_t *dirty_count = nullptr, *scan_scratch = nullptr;
    unsigned long long *touched = nullptr;    // per table row: the workers that stepped it since the last sync (W <= 64)
    unsigned long long *bad = nullptr;    // [0] out-of-range indices skipped; sparse syncs: [1] rows averaged, [2] worker rows read per matrix
    double *diag_scratch = nullptr;   // block partials + results of laa_diagnostics
    bool sparse_only_since_sync = true;   // every step since the last sync was a sparse one
    uint64_t bytes = 0;                   // bytes the launches enqueued so far read and write (collapsed state counted as such)
    uint64_t bytes_literal = 0;           // the same iterations as separate step and Synchronize passes over full replicas
    // replayed periods (laa_run_periods_gen): one captured graph per state the period can start in
    struct PeriodGraph {
        hipGraph_t graph = nullptr;
        hipGraphExec_t exec = nullptr;
        uint64_t epoch = 0;               // configuration the graph was captured for
        bool warmed = false;              // an eager period of this kind has run (kernels loaded) at that epoch
        uint64_t warmed_epoch = 0;
        bool end_collapsed = false;
        uint64_t bytes = 0, bytes_literal = 0;   // byte counters of one period
    } period[2];                          // [0]: starts from full replicas, [1]: from the collapsed state
    uint64_t epoch = 1;                   // bumped whenever something a captured kernel argument depends on changes
    uint32_t *t_dev = nullptr;            // device word: iteration count at the start of the period being replayed
    bool capturing = false;
    int64_t replays = 0;                  // periods run by graph replay so far
};

// Scratch of laa_sync_static: the row list, its length and the block counts of the bitmap compaction, for tables of
// up to STATIC_MAX_ROWS rows.  One copy per GPU, held until the process ends; its address on a device comes from
// hipGetSymbolAddress (the array's name is not a device address in host code).
static constexpr int64_t STATIC_MAX_ROWS = 1 << 20;
static constexpr size_t STATIC_LIST_BYTES = (size_t)STATIC_MAX_ROWS * sizeof(int32_t);
static constexpr size_t STATIC_COUNT_AT = STATIC_LIST_BYTES;              // one uint32
static constexpr size_t STATIC_SCAN_AT = STATIC_LIST_BYTES + 256;         // one uint32 per 1024 bitmap words, + 1
static constexpr size_t STATIC_SCRATCH_BYTES = STATIC_SCAN_AT + 256;      // 33 words needed at the maximum
static __device__ __align__(256) unsigned char laa_static_scratch[STATIC_SCRATCH_BYTES];

namespace {

thread_local char g_err[256] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int hip_fail(hipError_t e, const char *what)
{
    return fail(LAA_EHIP, "%s: %s", what, hipGetErrorString(e));
}

// Device address of laa_static_scratch on the current device, looked up once per device.
constexpr int MAX_DEVICES = 64;
std::mutex g_static_mutex;
unsigned char *g_static_ptr[MAX_DEVICES] = {};

int static_scratch(unsigned char **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= MAX_DEVICES) return fail(LAA_EINVAL, "device %d is outside the %d this library keeps scratch for", dev, MAX_DEVICES);
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(laa_static_scratch));
        if (e != hipSuccess || !p) return hip_fail(e, "hipGetSymbolAddress(static scratch)");
        g_static_ptr[dev] = static_cast<unsigned char *>(p);
    }
    *out = g_static_ptr[dev];
    return LAA_OK;
}

bool aligned(const void *p, size_t n) { return (reinterpret_cast<uintptr_t>(p) % n) == 0; }

int pick_wt(int32_t W) { return W % 8 == 0 ? 8 : W % 4 == 0 ? 4 : W % 2 == 0 ? 2 : 1; }

// eta_t = eta min(1, t / warmup_steps): Section 6.2, warm-up learning rates
float eta_at(const laa_ctx *h, int64_t t)
{
    if (h->warmup_steps <= 0) return (float)h->eta;
    const double r = (double)t / (double)h->warmup_steps;
    return (float)(h->eta * (r < 1.0 ? r : 1.0));
}

int check_ready(laa_handle h)
{
    if (!h) return fail(LAA_EINVAL, "null handle");
    if (!h->attached) return fail(LAA_ENOTATTACHED, "state buffers not attached (laa_attach)");
    return LAA_OK;
}

void drop_period_graphs(laa_ctx *h)
{
    for (auto &p : h->period) {
        if (p.exec) (void)hipGraphExecDestroy(p.exec);
        if (p.graph) (void)hipGraphDestroy(p.graph);
        p = laa_ctx::PeriodGraph();
    }
}

// Something a captured kernel argument depends on has changed: captured periods are stale.
void config_changed(laa_ctx *h) { h->epoch += 1; }

void free_sparse(laa_ctx *h)
{
    if (h->dirty) (void)hipFree(h->dirty);
    if (h->dirty_list) (void)hipFree(h->dirty_list);
    if (h->dirty_count) (void)hipFree(h->dirty_count);
    if (h->scan_scratch) (void)hipFree(h->scan_scratch);
    if (h->bad) (void)hipFree(h->bad);
    if (h->touched) (void)hipFree(h->touched);
    h->touched = nullptr;
    if (h->sort_keys) (void)hipFree(h->sort_keys);
    h->sort_keys = nullptr; h->sort_cap = 0;
    if (h->partials) (void)hipFree(h->partials);
    h->partials = nullptr; h->partial_cap = 0;
    h->dirty = nullptr; h->dirty_list = nullptr; h->dirty_count = nullptr; h->scan_scratch = nullptr; h->bad = nullptr;
    h->n_rows = 0; h->row_len = 0;
    config_changed(h);                    // the fused sync's bitmap clear is part of a captured period
}

int64_t n_dirty_words(int64_t n_rows) { return (n_rows + 31) / 32; }

int ensure_sparse(laa_ctx *h, int32_t row_len)
{
    if (h->dirty && h->row_len == row_len) return LAA_OK;
    if (h->dirty && h->s != 0)
        return fail(LAA_EINVAL, "row_len changed between syncs (%d -> %d)", h->row_len, row_len);
    free_sparse(h);
    const int64_t n_rows = h->d / row_len;
    if (n_rows > 0x7fffffffLL) return fail(LAA_EINVAL, "more than 2^31-1 rows");
    const int64_t nw = n_dirty_words(n_rows);
    hipError_t e;
    const char *what = "hipMalloc dirty bitmap";
    e = hipMalloc(&h->dirty, nw * sizeof(uint32_t));
    if (e == hipSuccess) { what = "hipMalloc sparse counters"; e = hipMalloc(&h->bad, 3 * sizeof(unsigned long long)); }
    if (e == hipSuccess && h->W <= 64) {  // one bit per worker in a 64-bit word per row; more workers: not recorded
        what = "hipMalloc touched-worker words";
        e = hipMalloc(&h->touched, (size_t)n_rows * sizeof(unsigned long long));
    }
    if (e == hipSuccess) { what = "clear dirty bitmap"; e = laa::launch_fill_u32(h->dirty, 0u, nw, h->stream); }
    if (e == hipSuccess && h->touched) {
        what = "clear touched-worker words";
        e = laa::launch_fill_u32(reinterpret_cast<uint32_t *>(h->touched), 0u, 2 * n_rows, h->stream);
    }
    if (e == hipSuccess) {
        what = "clear sparse counters";
        e = laa::launch_fill_u32(reinterpret_cast<uint32_t *>(h->bad), 0u, 6, h->stream);
    }
    if (e != hipSuccess) {
        free_sparse(h);                   // all or nothing: the next call starts from scratch
        return hip_fail(e, what);
    }
    h->n_rows = n_rows;
    h->row_len = row_len;
    config_changed(h);
    return LAA_OK;
}

// The handle's own row list for laa_sync and laa_get_dirty_rows (one int32 per table row, the count and the
// compaction's block counts), allocated when one of them first needs it; laa_sync_static never does.
int ensure_row_list(laa_ctx *h)
{
    if (h->dirty_list) return LAA_OK;
    hipError_t e;
    const char *what = "hipMalloc dirty list";
    e = hipMalloc(&h->dirty_list, h->n_rows * sizeof(int32_t));
    if (e == hipSuccess) { what = "hipMalloc dirty count"; e = hipMalloc(&h->dirty_count, sizeof(uint32_t)); }
    if (e == hipSuccess) { what = "hipMalloc scan scratch"; e = hipMalloc(&h->scan_scratch, (size_t)laa::compact_scratch_words(h->n_rows) * sizeof(uint32_t)); }
    if (e != hipSuccess) {
        if (h->dirty_list) (void)hipFree(h->dirty_list);
        if (h->dirty_count) (void)hipFree(h->dirty_count);
        if (h->scan_scratch) (void)hipFree(h->scan_scratch);
        h->dirty_list = nullptr; h->dirty_count = nullptr; h->scan_scratch = nullptr;
        return hip_fail(e, what);
    }
    return LAA_OK;
}

// Expand the collapsed post-sync state into every worker's row.
int materialize(laa_ctx *h)
{
    if (!h->collapsed) return LAA_OK;
    hipError_t e = laa::launch_materialize(h->x, h->acc, h->snap, h->d, h->pitch, h->W, h->stream);
    if (e != hipSuccess) return hip_fail(e, "materialize kernel launch");
    h->collapsed = false;
    h->bytes += (uint64_t)(8 + 8 * h->W - 4) * (uint64_t)h->d;      // reads row 0 of x and snap; writes the other rows of x, all of acc
    return LAA_OK;
}

int clear_dirty(laa_ctx *h)
{
    if (!h->dirty) return LAA_OK;
    hipError_t e = laa::launch_fill_u32(h->dirty, 0u, n_dirty_words(h->n_rows), h->stream);
    if (e == hipSuccess && h->touched)
        e = laa::launch_fill_u32(reinterpret_cast<uint32_t *>(h->touched), 0u, 2 * h->n_rows, h->stream);
    return e == hipSuccess ? LAA_OK : hip_fail(e, "clear dirty bitmap");
}

enum StepKind { STEP_DENSE, STEP_GEN };

// One local iteration (and, if fuse_sync, the averaging in the same pass).
int dense_step(laa_handle h, StepKind kind, const float *grads, bool allow_fused_sync)
{
    int rc = check_ready(h);
    if (rc != LAA_OK) return rc;
    if (kind == STEP_DENSE) {
        if (!grads) return fail(LAA_EINVAL, "null gradient pointer");
        if (!aligned(grads, 4)) return fail(LAA_EALIGN, "gradient pointer not 4-byte aligned");
    } else if (h->gen_mode == 0) {
        return fail(LAA_EMODE, "no gradient generator configured (laa_set_generator)");
    }
    const bool adagrad = h->algo == LAA_ALGO_DIST_ADAGRAD;
    if (h->algo != LAA_ALGO_LOCAL_ADAALTER && !allow_fused_sync)
        return fail(LAA_EMODE, "this update rule runs through laa_step_* only");
    if (!adagrad && h->s >= h->H)
        return fail(LAA_ESYNCDUE, "%d local steps since the last sync (H=%d): call laa_sync", h->s, h->H);
    // Algorithm 2 steps every worker's own row; Algorithm 1 has one iterate, which stays collapsed with lazy replicas
    const bool adagrad_row0 = adagrad && h->lazy;
    if (h->algo != LAA_ALGO_LOCAL_ADAALTER && !adagrad_row0 && (rc = materialize(h)) != LAA_OK) return rc;

    laa::StepArgs a{};
    a.x = h->x; a.acc = h->acc; a.snap = h->snap;
    a.grads = kind == STEP_DENSE ? grads : nullptr;
    a.a = h->a; a.xstar = h->xstar; a.off = h->off;
    a.grad_out = nullptr;
    a.d = h->d; a.pitch = h->pitch; a.W = h->W;
    a.eta = eta_at(h, h->t + 1);
    const float eps2 = (float)(h->eps * h->eps);
    a.eps2 = eps2;
    a.pad = (float)(h->s + 1) * eps2;                      // t' eps^2, t' = steps since sync + 1
    a.noise_scale = h->noise_scale; a.off_scale = h->off_scale;
    a.seed_lo = (uint32_t)h->seed; a.seed_hi = (uint32_t)(h->seed >> 32);
    a.col0 = h->col0; a.w0 = h->w0;
    a.t_lo = (uint32_t)(h->t + 1);
    a.t_dev = h->capturing ? h->t_dev : nullptr;
    a.grad_source = kind == STEP_DENSE ? laa::GRAD_EXPLICIT : h->gen_mode;
    a.off_source = kind == STEP_DENSE ? laa::OFFSET_NONE : h->off_mode;
    a.sync = adagrad || (allow_fused_sync && h->s + 1 == h->H);
    a.collapsed_in = h->collapsed;
    a.collapsed_out = a.sync && h->lazy && h->algo != LAA_ALGO_LOCAL_SGD;
    a.algo = h->algo;
    a.wt = h->wt;
    a.split = h->split;
    a.vec4 = h->vec4 && (kind == STEP_DENSE ? aligned(grads, 16) : h->gen_aligned16);

    hipError_t e = laa::launch_step(a, h->stream);
    if (e != hipSuccess) return hip_fail(e, "step kernel launch");

    // byte counters, per column: what this launch moves, and what the same iteration moves as a plain step over full
    // replicas followed (when it averages) by a separate Synchronize pass
    const uint64_t W = (uint64_t)h->W, d = (uint64_t)h->d;
    uint64_t inputs = 4 * W;                                // explicit gradients
    if (kind != STEP_DENSE)
        inputs = (h->gen_mode == LAA_GEN_QUADRATIC ? 8 : 4) + (h->off_mode == LAA_OFF_ARRAY ? 4 * W : 0);
    uint64_t moved, literal;
    if (h->algo == LAA_ALGO_LOCAL_ADAALTER) {
        const uint64_t in = a.collapsed_in ? 8 : 8 * W + 4;                  // x, acc of every worker and snap, or row 0 and snap
        const uint64_t out = !a.sync ? 8 * W : a.collapsed_out ? 8 : 8 * W + 4;
        moved = in + inputs + out;
        literal = 16 * W + 4 + inputs + (a.sync ? 16 * W + 4 : 0);
    } else if (adagrad) {                                   // one iterate: x rows and snap in, x, acc rows and snap out
        moved = (a.collapsed_out ? 8 : 4 * W + 4) + inputs + (a.collapsed_out ? 8 : 8 * W + 4);
        literal = 4 * W + 4 + inputs + 8 * W + 4;
    } else {                                                // Local SGD: x rows in and out
        moved = 8 * W + inputs;
        literal = 8 * W + inputs + (a.sync ? 8 * W : 0);
    }
    h->bytes += moved * d;
    h->bytes_literal += literal * d;
    h->t += 1;
    h->s += 1;
    h->sparse_only_since_sync = false;
    h->collapsed = a.collapsed_out;
    if (a.sync) {
        h->s = 0;
        h->sparse_only_since_sync = true;
        rc = clear_dirty(h);
    }
    return rc;
}

}  // namespace

extern "C" {

const char *laa_last_error(void) { return g_err; }

int laa_create(int64_t d, int32_t W, int32_t H, double eta, double eps, laa_handle *out)
{
    if (!out) return fail(LAA_EINVAL, "null out pointer");
    *out = nullptr;
    if (d <= 0) return fail(LAA_EINVAL, "d must be positive (got %lld)", (long long)d);
    if (W <= 0) return fail(LAA_EINVAL, "W must be positive (got %d)", W);
    if (H <= 0) return fail(LAA_EINVAL, "H must be positive (got %d)", H);
    if (!std::isfinite(eta)) return fail(LAA_EINVAL, "eta must be finite");
    if (!(eps >= 0.0) || !std::isfinite(eps)) return fail(LAA_EINVAL, "eps must be finite and >= 0");
    if ((double)d * (double)W > 9.0e18) return fail(LAA_EINVAL, "W*d overflows");
    laa_ctx *h = new (std::nothrow) laa_ctx();
    if (!h) return fail(LAA_EINVAL, "out of host memory");
    h->d = d; h->W = W; h->H = H; h->eta = eta; h->eps = eps;
    h->wt = pick_wt(W);
    *out = h;
    return LAA_OK;
}

int laa_destroy(laa_handle h)
{
    if (!h) return LAA_OK;
    free_sparse(h);
    drop_period_graphs(h);
    if (h->t_dev) (void)hipFree(h->t_dev);
    if (h->diag_scratch) (void)hipFree(h->diag_scratch);
    delete h;
    return LAA_OK;
}

int laa_set_b0(laa_handle h, double b0)
{
    if (!h) return fail(LAA_EINVAL, "null handle");
    if (!(b0 >= 0.0) || !std::isfinite(b0)) return fail(LAA_EINVAL, "b0 must be finite and >= 0");
    if (h->t != 0) return fail(LAA_EINVAL, "b0 can only be set before the first step");
    h->b0 = b0;
    config_changed(h);
    return LAA_OK;
}

int laa_set_warmup(laa_handle h, int64_t warmup_steps)
{
    if (!h) return fail(LAA_EINVAL, "null handle");
    if (warmup_steps < 0) return fail(LAA_EINVAL, "warmup_steps must be >= 0");
    h->warmup_steps = warmup_steps;
    config_changed(h);
    return LAA_OK;
}

int laa_set_algorithm(laa_handle h, int32_t algo)
{
    if (!h) return fail(LAA_EINVAL, "null handle");
    if (algo < LAA_ALGO_LOCAL_ADAALTER || algo > LAA_ALGO_LOCAL_SGD) return fail(LAA_EINVAL, "unknown update rule %d", algo);
    if (h->t != 0) return fail(LAA_EINVAL, "the update rule can only be chosen before the first step");
    h->algo = algo;
    config_changed(h);
    return LAA_OK;
}

int laa_set_tile(laa_handle h, int32_t workers_per_batch)
{
    if (!h) return fail(LAA_EINVAL, "null handle");
    const int32_t wt = workers_per_batch;
    if (wt == 0) {              // one worker per thread block in non-sync steps
        h->split = true;
        h->wt = pick_wt(h->W);
        config_changed(h);
        return LAA_OK;
    }
    if (!(wt == 1 || wt == 2 || wt == 4 || wt == 8) || h->W % wt != 0)
        return fail(LAA_EINVAL, "workers_per_batch must be 0, or 1, 2, 4 or 8 and divide W");
    h->wt = wt;
    h->split = false;
    config_changed(h);
    return LAA_OK;
}

int laa_set_lazy_replicas(laa_handle h, int32_t on)
{
    if (!h) return fail(LAA_EINVAL, "null handle");
    if (!on && h->collapsed) {
        int rc = check_ready(h);
        if (rc == LAA_OK) rc = materialize(h);
        if (rc != LAA_OK) return rc;
    }
    h->lazy = on != 0;
    config_changed(h);
    return LAA_OK;
}

int laa_set_sparse_coalesce(laa_handle h, int32_t on)
{
    if (!h) return fail(LAA_EINVAL, "null handle");
    h->coalesce = on != 0;
    return LAA_OK;
}

int laa_materialize(laa_handle h)
{
    int rc = check_ready(h);
    return rc != LAA_OK ? rc : materialize(h);
}

int laa_attach(laa_handle h, float *x, float *acc, float *snap, void *hip_stream)
{
    return laa_attach_pitched(h, x, acc, snap, h ? h->d : 0, hip_stream);
}

int laa_attach_pitched(laa_handle h, float *x, float *acc, float *snap, int64_t pitch, void *hip_stream)
{
    if (!h) return fail(LAA_EINVAL, "null handle");
    if (pitch < h->d) return fail(LAA_EINVAL, "pitch %lld is smaller than d %lld", (long long)pitch, (long long)h->d);
    if (!x || !acc || !snap) return fail(LAA_EINVAL, "null state pointer");
    if (!aligned(x, 4) || !aligned(acc, 4) || !aligned(snap, 4)) return fail(LAA_EALIGN, "state pointer not 4-byte aligned");
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || n <= 0) return fail(LAA_ENODEVICE, "no HIP device available");
    h->x = x; h->acc = acc; h->snap = snap;
    h->stream = static_cast<hipStream_t>(hip_stream);
    h->pitch = pitch;
    h->vec4 = h->d % 4 == 0 && pitch % 4 == 0 && aligned(x, 16) && aligned(acc, 16) && aligned(snap, 16);
    h->attached = true;
    if (h->s > 0) h->sparse_only_since_sync = false;   // other arrays in the middle of a period: which of their rows
                                                       // differ between workers is unknown, the next sync takes them all
    config_changed(h);
    return LAA_OK;
}

int laa_init_state(laa_handle h, const float *x0)
{
    int rc = check_ready(h);
    if (rc != LAA_OK) return rc;
    if (x0 && !aligned(x0, 4)) return fail(LAA_EALIGN, "x0 not 4-byte aligned");
    const float b0sq = (float)(h->b0 * h->b0);
    hipError_t e = laa::launch_init(h->x, h->acc, h->snap, x0, b0sq, h->d, h->pitch, h->W, h->stream);
    if (e != hipSuccess) return hip_fail(e, "init kernel launch");
    h->t = 0; h->s = 0; h->bytes = 0; h->bytes_literal = 0; h->sparse_only_since_sync = true; h->collapsed = false;
    if (h->bad && laa::launch_fill_u32(reinterpret_cast<uint32_t *>(h->bad + 1), 0u, 4, h->stream) != hipSuccess)
        return fail(LAA_EHIP, "clearing the sparse-sync row counter");
    return clear_dirty(h);
}

int laa_set_generator(laa_handle h, int32_t mode, uint64_t seed, const float *a, const float *xstar,
                      const float *off, int32_t off_mode, float noise_scale, float off_scale)
{
    if (!h) return fail(LAA_EINVAL, "null handle");
    if (mode != LAA_GEN_QUADRATIC && mode != LAA_GEN_NOISE) return fail(LAA_EMODE, "unknown generator mode %d", mode);
    if (!a) return fail(LAA_EINVAL, "null a");
    if (mode == LAA_GEN_QUADRATIC && !xstar) return fail(LAA_EINVAL, "null xstar");
    if (mode == LAA_GEN_NOISE) off_mode = LAA_OFF_NONE;
    if (off_mode < LAA_OFF_NONE || off_mode > LAA_OFF_PHILOX) return fail(LAA_EMODE, "unknown offset mode %d", off_mode);
    if (off_mode == LAA_OFF_ARRAY && !off) return fail(LAA_EINVAL, "null off with LAA_OFF_ARRAY");
    if (!(noise_scale >= 0.0f) || !(off_scale >= 0.0f) || !std::isfinite(noise_scale) || !std::isfinite(off_scale))
        return fail(LAA_EINVAL, "noise_scale and off_scale are standard deviations: finite and >= 0");
    const bool a16 = aligned(a, 16) && (!xstar || aligned(xstar, 16)) && (off_mode != LAA_OFF_ARRAY || aligned(off, 16));
    if (!aligned(a, 4) || (xstar && !aligned(xstar, 4)) || (off && !aligned(off, 4)))
        return fail(LAA_EALIGN, "generator array not 4-byte aligned");
    h->gen_aligned16 = a16;                                // else generator steps take the scalar path
    h->gen_mode = mode; h->off_mode = off_mode; h->seed = seed;
    h->a = a; h->xstar = xstar; h->off = off;
    h->noise_scale = noise_scale; h->off_scale = off_scale;
    config_changed(h);
    return LAA_OK;
}

int laa_set_shard(laa_handle h, int64_t first_column, int32_t first_worker)
{
    if (!h) return fail(LAA_EINVAL, "null handle");
    if (first_column < 0 || first_column % 4 != 0)
        return fail(LAA_EINVAL, "first_column must be a non-negative multiple of 4 (got %lld)", (long long)first_column);
    if (first_column > INT64_MAX - h->d) return fail(LAA_EINVAL, "first_column + d overflows");
    if (first_worker < 0 || first_worker > INT32_MAX - h->W) return fail(LAA_EINVAL, "bad first_worker %d", first_worker);
    h->col0 = first_column; h->w0 = first_worker;
    config_changed(h);
    return LAA_OK;
}

int laa_local_step_dense(laa_handle h, const float *grads) { return dense_step(h, STEP_DENSE, grads, false); }
int laa_local_step_gen(laa_handle h) { return dense_step(h, STEP_GEN, nullptr, false); }
int laa_step_dense(laa_handle h, const float *grads) { return dense_step(h, STEP_DENSE, grads, true); }
int laa_step_gen(laa_handle h) { return dense_step(h, STEP_GEN, nullptr, true); }

// One period = H generator steps, the last one with the averaging fused in.
static int eager_period(laa_handle h)
{
    for (int32_t k = 0; k < h->H; ++k) {
        const int rc = dense_step(h, STEP_GEN, nullptr, true);
        if (rc != LAA_OK) return rc;
    }
    return LAA_OK;
}

int laa_run_periods_gen(laa_handle h, int32_t n_periods)
{
    int rc = check_ready(h);
    if (rc != LAA_OK) return rc;
    if (n_periods < 0) return fail(LAA_EINVAL, "n_periods must be >= 0");
    if (h->gen_mode == 0) return fail(LAA_EMODE, "no gradient generator configured (laa_set_generator)");
    if (h->algo != LAA_ALGO_LOCAL_ADAALTER) return fail(LAA_EMODE, "replayed periods exist for Local AdaAlter only");
    if (h->s != 0) return fail(LAA_EINVAL, "%d local steps since the last sync: a period must start right after one", h->s);
    hipError_t e;
    for (int32_t n = 0; n < n_periods; ++n) {
        const int c = h->collapsed ? 1 : 0;
        laa_ctx::PeriodGraph &pg = h->period[c];
        // The learning rate is an argument of the captured kernels: periods inside the warm-up run eagerly.  So does
        // everything on the legacy default stream, which cannot be captured, and the first period of each kind,
        // so that no kernel is launched for the first time under capture.
        const bool in_warmup = h->warmup_steps > 0 && h->t < h->warmup_steps;
        const bool warmed = pg.warmed && pg.warmed_epoch == h->epoch;
        const bool vector_path = h->vec4 && h->gen_aligned16 && !h->split;   // the kernels with a device iteration word
        if (in_warmup || h->stream == nullptr || !warmed || !vector_path) {
            if ((rc = eager_period(h)) != LAA_OK) return rc;
            if (!in_warmup) { pg.warmed = true; pg.warmed_epoch = h->epoch; }
            continue;
        }
        if (!h->t_dev) {
            if ((e = hipMalloc(&h->t_dev, 2 * sizeof(uint32_t))) != hipSuccess) return hip_fail(e, "hipMalloc iteration word");
        }
        if (!pg.exec || pg.epoch != h->epoch) {
            if (pg.exec) (void)hipGraphExecDestroy(pg.exec);
            if (pg.graph) (void)hipGraphDestroy(pg.graph);
            pg.exec = nullptr; pg.graph = nullptr;
            // Record the H launches of one period with iteration numbers 1..H relative to the device word, which the
            // last node of the graph advances by H.  Nothing runs during capture; the host state is put back after.
            const int64_t t_saved = h->t, warm_saved = h->warmup_steps;
            const uint64_t bytes_saved = h->bytes, literal_saved = h->bytes_literal;
            const int32_t s_saved = h->s;
            const bool sparse_only_saved = h->sparse_only_since_sync;
            if ((e = hipStreamBeginCapture(h->stream, hipStreamCaptureModeThreadLocal)) != hipSuccess)
                return hip_fail(e, "hipStreamBeginCapture");
            h->capturing = true; h->t = 0; h->warmup_steps = 0;
            rc = eager_period(h);
            hipError_t e_bump = rc == LAA_OK ? laa::launch_add_u32(h->t_dev, (uint32_t)h->H, h->stream) : hipSuccess;
            h->capturing = false; h->t = t_saved; h->warmup_steps = warm_saved;
            pg.end_collapsed = h->collapsed;
            pg.bytes = h->bytes - bytes_saved;
            pg.bytes_literal = h->bytes_literal - literal_saved;
            // nothing ran: put back everything the recorded calls changed on the host, also when recording failed midway
            h->bytes = bytes_saved; h->bytes_literal = literal_saved;
            h->s = s_saved; h->sparse_only_since_sync = sparse_only_saved;
            h->collapsed = c != 0;
            e = hipStreamEndCapture(h->stream, &pg.graph);            // always leave capture mode
            if (rc != LAA_OK) { if (pg.graph) (void)hipGraphDestroy(pg.graph); pg.graph = nullptr; return rc; }
            if (e_bump != hipSuccess) e = e_bump;
            if (e == hipSuccess) e = hipGraphInstantiate(&pg.exec, pg.graph, nullptr, nullptr, 0);
            if (e != hipSuccess) {
                if (pg.graph) (void)hipGraphDestroy(pg.graph);
                pg.graph = nullptr; pg.exec = nullptr;
                return hip_fail(e, "capturing a period into a HIP graph");
            }
            pg.epoch = h->epoch;
        }
        // consecutive periods of the same kind: set the device word once, replay back to back
        if ((e = laa::launch_fill_u32(h->t_dev, (uint32_t)h->t, 1, h->stream)) != hipSuccess)
            return hip_fail(e, "setting the iteration word");
        while (true) {
            if ((e = hipGraphLaunch(pg.exec, h->stream)) != hipSuccess) return hip_fail(e, "hipGraphLaunch");
            h->t += h->H;
            h->replays += 1;
            h->bytes += pg.bytes;
            h->bytes_literal += pg.bytes_literal;
            h->collapsed = pg.end_collapsed;
            h->sparse_only_since_sync = true;
            const bool next_in_warmup = h->warmup_steps > 0 && h->t < h->warmup_steps;
            if (n + 1 < n_periods && (h->collapsed ? 1 : 0) == c && !next_in_warmup) ++n;
            else break;
        }
    }
    return LAA_OK;
}

int laa_get_replay_count(laa_handle h, int64_t *periods_replayed)
{
    if (!h || !periods_replayed) return fail(LAA_EINVAL, "null argument");
    *periods_replayed = h->replays;
    return LAA_OK;
}

int laa_generate_gradient(laa_handle h, float *out)
{
    int rc = check_ready(h);
    if (rc != LAA_OK) return rc;
    if (h->gen_mode == 0) return fail(LAA_EMODE, "no gradient generator configured (laa_set_generator)");
    if (!out) return fail(LAA_EINVAL, "null out");
    if (!aligned(out, 4)) return fail(LAA_EALIGN, "out not 4-byte aligned");
    laa::StepArgs a{};
    a.x = h->x; a.acc = h->acc; a.snap = h->snap;
    a.a = h->a; a.xstar = h->xstar; a.off = h->off;
    a.grad_out = out;
    a.d = h->d; a.pitch = h->pitch; a.W = h->W;
    a.noise_scale = h->noise_scale; a.off_scale = h->off_scale;
    a.seed_lo = (uint32_t)h->seed; a.seed_hi = (uint32_t)(h->seed >> 32);
    a.col0 = h->col0; a.w0 = h->w0;
    a.t_lo = (uint32_t)(h->t + 1);
    a.grad_source = h->gen_mode; a.off_source = h->off_mode;
    a.collapsed_in = h->collapsed;
    a.vec4 = h->vec4 && h->gen_aligned16 && aligned(out, 16);
    a.wt = h->wt;
    hipError_t e = laa::launch_step(a, h->stream);
    return e == hipSuccess ? LAA_OK : hip_fail(e, "gradient kernel launch");
}

int laa_local_step_sparse(laa_handle h, const int32_t *idx, const float *vals, int32_t k, int32_t row_len)
{
    int rc = check_ready(h);
    if (rc != LAA_OK) return rc;
    if (h->algo != LAA_ALGO_LOCAL_ADAALTER) return fail(LAA_EMODE, "sparse steps exist for Local AdaAlter only");
    if (k < 0) return fail(LAA_EINVAL, "k must be >= 0");
    if (row_len <= 0 || row_len % 4 != 0) return fail(LAA_EINVAL, "row_len must be a positive multiple of 4");
    if (h->d % row_len != 0) return fail(LAA_EINVAL, "d is not a multiple of row_len");
    if (k > 0 && (!idx || !vals)) return fail(LAA_EINVAL, "null idx/vals");
    if (!aligned(h->x, 16) || !aligned(h->acc, 16) || !aligned(h->snap, 16) || (k > 0 && !aligned(vals, 16)) ||
        h->pitch % 4 != 0)
        return fail(LAA_EALIGN, "sparse path needs 16-byte aligned x, acc, snap, vals");
    if (k > 0 && !aligned(idx, 4)) return fail(LAA_EALIGN, "idx not 4-byte aligned");
    if (h->s >= h->H)
        return fail(LAA_ESYNCDUE, "%d local steps since the last sync (H=%d): call laa_sync", h->s, h->H);
    if (h->coalesce && k > laa::coalesce_max_k())
        return fail(LAA_EINVAL, "k = %d exceeds the coalescing step's limit of %d rows per worker and step", k,
                    laa::coalesce_max_k());
    rc = ensure_sparse(h, row_len);
    if (rc != LAA_OK) return rc;
    if ((rc = materialize(h)) != LAA_OK) return rc;      // the row kernel reads every worker's own rows
    laa::SparseArgs a{};
    a.x = h->x; a.acc = h->acc; a.snap = h->snap;
    a.idx = idx; a.vals = vals; a.dirty = h->dirty; a.touched = h->touched; a.bad = h->bad;
    a.d = h->d; a.pitch = h->pitch; a.n_rows = h->n_rows; a.W = h->W; a.k = k; a.row_len = row_len;
    a.eta = eta_at(h, h->t + 1);
    a.pad = (float)(h->s + 1) * (float)(h->eps * h->eps);
    hipError_t e;
    if (h->coalesce && k > 0) {
        // Sized on first use for the longest list the coalescing step takes, so that no later step allocates: a
        // step that found its buffers too small would have to free them, and hipFree waits for the device.
        const int64_t need = (int64_t)h->W * laa::coalesce_max_k();
        if (need > h->sort_cap) {
            if (h->sort_keys) (void)hipFree(h->sort_keys);
            h->sort_keys = nullptr; h->sort_cap = 0;
            if ((e = hipMalloc(&h->sort_keys, (size_t)need * sizeof(uint64_t))) != hipSuccess)
                return hip_fail(e, "hipMalloc sort keys");
            h->sort_cap = need;
        }
        const int64_t need_p = laa::coalesce_partial_rows(h->W, laa::coalesce_max_k()) * row_len;
        if (need_p > h->partial_cap) {                      // only when row_len grew (ensure_sparse dropped the old ones)
            if (h->partials) (void)hipFree(h->partials);
            h->partials = nullptr; h->partial_cap = 0;
            if ((e = hipMalloc(&h->partials, (size_t)need_p * sizeof(float))) != hipSuccess)
                return hip_fail(e, "hipMalloc partial rows");
            h->partial_cap = need_p;
        }
        a.partials = h->partials;
        if ((e = laa::launch_sort_rows(idx, h->sort_keys, h->W, k, h->n_rows, h->stream)) != hipSuccess)
            return hip_fail(e, "row sort kernel launch");
        a.keys = h->sort_keys;
        if ((e = laa::launch_sparse_step_coalesce(a, h->stream)) != hipSuccess)
            return hip_fail(e, "coalescing sparse step kernel launch");
        h->bytes += (uint64_t)h->W * (uint64_t)k * 16;             // keys written, then read
        h->bytes_literal += (uint64_t)h->W * (uint64_t)k * 16;
    } else {
        if ((e = laa::launch_sparse_step(a, h->stream)) != hipSuccess) return hip_fail(e, "sparse step kernel launch");
    }
    h->bytes += (uint64_t)h->W * (uint64_t)k * ((uint64_t)row_len * 24 + 4);
    h->bytes_literal += (uint64_t)h->W * (uint64_t)k * ((uint64_t)row_len * 24 + 4);
    h->t += 1;
    h->s += 1;
    return LAA_OK;
}

// Synchronize.  static_scratch: the dirty-row list and the compaction's counters live in laa_static_scratch
// instead of the handle's own buffers.
static int sync_impl(laa_handle h, bool use_static)
{
    int rc = check_ready(h);
    if (rc != LAA_OK) return rc;
    if (h->algo == LAA_ALGO_DIST_ADAGRAD) return LAA_OK;     // every iteration is already synchronous
    if (h->s == 0) return LAA_OK;
    hipError_t e;
    const bool x_only = h->algo == LAA_ALGO_LOCAL_SGD;
    if (h->dirty && h->sparse_only_since_sync && !x_only) {
        int32_t *list = nullptr;
        uint32_t *count = nullptr, *scan = nullptr;
        if (use_static) {
            if (h->n_rows > STATIC_MAX_ROWS)
                return fail(LAA_EINVAL, "the table has %lld rows; laa_sync_static holds the list of at most %lld (use laa_sync)",
                            (long long)h->n_rows, (long long)STATIC_MAX_ROWS);
            if ((size_t)laa::compact_scratch_words(h->n_rows) * sizeof(uint32_t) > STATIC_SCRATCH_BYTES - STATIC_SCAN_AT)
                return fail(LAA_EINVAL, "the compaction's block counts do not fit the static scratch");
            unsigned char *base = nullptr;
            if ((rc = static_scratch(&base)) != LAA_OK) return rc;
            list = reinterpret_cast<int32_t *>(base);
            count = reinterpret_cast<uint32_t *>(base + STATIC_COUNT_AT);
            scan = reinterpret_cast<uint32_t *>(base + STATIC_SCAN_AT);
        } else {
            if ((rc = ensure_row_list(h)) != LAA_OK) return rc;
            list = h->dirty_list; count = h->dirty_count; scan = h->scan_scratch;     // only now allocated for sure
        }
        // every word the kernels read from the scratch is written by an earlier kernel of the same call (block counts,
        // their scan, the count, the first `count` list entries): nothing has to start at zero
        e = laa::launch_compact_dirty(h->dirty, h->n_rows, list, count, scan, h->stream);
        if (e != hipSuccess) return hip_fail(e, "dirty-row compaction launch");
        e = laa::launch_mean_rows(h->x, h->acc, h->snap, h->pitch, h->W, h->wt, h->row_len, list, count, h->touched,
                                  h->bad + 1, h->stream);
        if (e != hipSuccess) return hip_fail(e, "dirty-row mean launch");
    } else {
        const bool collapse = h->lazy && !x_only;
        e = laa::launch_mean(h->x, h->acc, h->snap, h->d, h->pitch, h->W, h->vec4, h->wt, x_only,
                             collapse, h->stream);
        if (e != hipSuccess) return hip_fail(e, "mean kernel launch");
        const uint64_t W = (uint64_t)h->W;
        h->bytes += (x_only ? 8 * W : 8 * W + (collapse ? 8 : 8 * W + 4)) * (uint64_t)h->d;
        h->bytes_literal += (x_only ? 8 * W : 16 * W + 4) * (uint64_t)h->d;
        h->collapsed = collapse;
    }
    h->s = 0;
    h->sparse_only_since_sync = true;
    return clear_dirty(h);
}

int laa_sync(laa_handle h) { return sync_impl(h, false); }
int laa_sync_static(laa_handle h) { return sync_impl(h, true); }

int laa_step_sparse(laa_handle h, const int32_t *idx, const float *vals, int32_t k, int32_t row_len)
{
    int rc = laa_local_step_sparse(h, idx, vals, k, row_len);
    if (rc == LAA_OK && h->s == h->H) rc = laa_sync(h);
    return rc;
}

int laa_get_counters(laa_handle h, int64_t *t, int32_t *steps_since_sync, int64_t *bad_indices)
{
    if (!h) return fail(LAA_EINVAL, "null handle");
    if (t) *t = h->t;
    if (steps_since_sync) *steps_since_sync = h->s;
    if (bad_indices) {
        *bad_indices = 0;
        if (h->bad) {
            unsigned long long v = 0;
            hipError_t e = hipMemcpyAsync(&v, h->bad, sizeof(v), hipMemcpyDeviceToHost, h->stream);
            if (e == hipSuccess) e = hipStreamSynchronize(h->stream);
            if (e != hipSuccess) return hip_fail(e, "reading the bad-index counter");
            *bad_indices = (int64_t)v;
        }
    }
    return LAA_OK;
}

int laa_set_counters(laa_handle h, int64_t t, int32_t steps_since_sync)
{
    if (!h) return fail(LAA_EINVAL, "null handle");
    if (t < 0 || steps_since_sync < 0 || steps_since_sync > h->H || steps_since_sync > t)
        return fail(LAA_EINVAL, "need 0 <= steps_since_sync <= min(H, t)");
    h->t = t;
    h->s = steps_since_sync;
    h->collapsed = false;                 // the caller has put full arrays in place
    h->sparse_only_since_sync = false;    // rows touched before the checkpoint are unknown: next sync is dense
    return h->attached ? clear_dirty(h) : LAA_OK;
}

int laa_get_dirty_rows(laa_handle h, int32_t *out, int64_t cap, int64_t *n)
{
    int rc = check_ready(h);
    if (rc != LAA_OK) return rc;
    if (!n) return fail(LAA_EINVAL, "null n");
    if (cap < 0 || (cap > 0 && !out)) return fail(LAA_EINVAL, "bad out/cap");
    *n = 0;
    if (!h->dirty) return LAA_OK;
    if ((rc = ensure_row_list(h)) != LAA_OK) return rc;
    hipError_t e = laa::launch_compact_dirty(h->dirty, h->n_rows, h->dirty_list, h->dirty_count, h->scan_scratch, h->stream);
    if (e != hipSuccess) return hip_fail(e, "dirty-row compaction launch");
    uint32_t cnt = 0;
    e = hipMemcpyAsync(&cnt, h->dirty_count, sizeof(cnt), hipMemcpyDeviceToHost, h->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(h->stream);
    if (e != hipSuccess) return hip_fail(e, "reading the dirty-row count");
    *n = cnt;
    const int64_t m = cnt < cap ? cnt : cap;
    if (m > 0) {
        e = hipMemcpyAsync(out, h->dirty_list, m * sizeof(int32_t), hipMemcpyDeviceToHost, h->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(h->stream);
        if (e != hipSuccess) return hip_fail(e, "copying the dirty-row list");
    }
    return LAA_OK;
}

int laa_diagnostics(laa_handle h, double *out)
{
    int rc = check_ready(h);
    if (rc != LAA_OK) return rc;
    if (!out) return fail(LAA_EINVAL, "null out");
    if (h->gen_mode != LAA_GEN_QUADRATIC) return fail(LAA_EMODE, "diagnostics need the quadratic generator (a, xstar)");
    hipError_t e;
    if (!h->diag_scratch) {
        e = hipMalloc(&h->diag_scratch, (size_t)laa::diag_scratch_doubles() * sizeof(double));
        if (e != hipSuccess) return hip_fail(e, "hipMalloc diagnostics scratch");
    }
    laa::StepArgs a{};
    a.x = h->x; a.acc = h->acc; a.snap = h->snap;
    a.a = h->a; a.xstar = h->xstar; a.off = h->off;
    a.d = h->d; a.pitch = h->pitch; a.W = h->W;
    a.off_scale = h->off_scale;
    a.seed_lo = (uint32_t)h->seed; a.seed_hi = (uint32_t)(h->seed >> 32);
    a.col0 = h->col0; a.w0 = h->w0;
    a.off_source = h->off_mode;
    a.collapsed_in = h->collapsed;
    a.vec4 = h->vec4 && h->gen_aligned16;
    e = laa::launch_diagnostics(a, h->diag_scratch, h->stream);
    if (e != hipSuccess) return hip_fail(e, "diagnostics kernel launch");
    e = hipMemcpyAsync(out, h->diag_scratch + laa::diag_scratch_doubles() - 3, 3 * sizeof(double), hipMemcpyDeviceToHost,
                       h->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(h->stream);
    if (e != hipSuccess) return hip_fail(e, "reading the diagnostics");
    return LAA_OK;
}

int laa_bytes_moved(laa_handle h, uint64_t *moved_bytes, uint64_t *literal_bytes)
{
    if (!h || (!moved_bytes && !literal_bytes)) return fail(LAA_EINVAL, "null argument");
    uint64_t sparse_sync = 0, sparse_sync_literal = 0;
    if (h->bad) {                       // what the sparse syncs averaged and read is counted on the device
        unsigned long long c[2] = {0, 0};   // rows averaged; worker rows read per matrix
        hipError_t e = hipMemcpyAsync(c, h->bad + 1, sizeof(c), hipMemcpyDeviceToHost, h->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(h->stream);
        if (e != hipSuccess) return hip_fail(e, "reading the sparse-sync counters");
        // per listed row: the touched workers' rows of x and acc and one untouched worker's are read, every worker's
        // rows and snap's are written; literally, every worker's rows are read
        sparse_sync = (2 * (uint64_t)c[1] + (uint64_t)c[0] * (uint64_t)(2 * h->W + 1)) * 4 * (uint64_t)h->row_len;
        sparse_sync_literal = (uint64_t)c[0] * (uint64_t)(16 * h->W + 4) * (uint64_t)h->row_len;
    }
    if (moved_bytes) *moved_bytes = h->bytes + sparse_sync;
    if (literal_bytes) *literal_bytes = h->bytes_literal + sparse_sync_literal;
    return LAA_OK;
}

// ---- spread allocation -------------------------------------------------------------------------------------
namespace {
struct SpreadAlloc {
    size_t chunk = 0, dist = 0;
    std::vector<hipMemGenericAllocationHandle_t> handles;
    size_t mapped = 0;          // how many chunks are mapped
    bool reserved = false;
};
std::mutex g_spread_mutex;
std::map<void *, SpreadAlloc> g_spread;

void spread_release(void *base, SpreadAlloc &sa)
{
    for (size_t i = 0; i < sa.mapped; ++i) (void)hipMemUnmap(static_cast<char *>(base) + i * sa.dist, sa.chunk);
    for (auto h : sa.handles) (void)hipMemRelease(h);
    if (sa.reserved) (void)hipMemAddressFree(base, sa.dist * sa.handles.size());
}
}  // namespace

int laa_spread_alloc(int32_t n_arrays, int64_t array_bytes, int64_t distance_bytes, void **base,
                     int64_t *actual_distance_bytes)
{
    if (!base) return fail(LAA_EINVAL, "null base");
    *base = nullptr;
    if (n_arrays <= 0 || array_bytes <= 0 || distance_bytes < array_bytes)
        return fail(LAA_EINVAL, "need n_arrays > 0 and 0 < array_bytes <= distance_bytes");
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(LAA_ENODEVICE, "no HIP device available");
    hipMemAllocationProp prop = {};
    prop.type = hipMemAllocationTypePinned;
    prop.location.type = hipMemLocationTypeDevice;
    prop.location.id = dev;
    size_t gran = 0;
    if ((e = hipMemGetAllocationGranularity(&gran, &prop, hipMemAllocationGranularityRecommended)) != hipSuccess)
        return hip_fail(e, "hipMemGetAllocationGranularity");
    if (gran < (size_t(2) << 20)) gran = size_t(2) << 20;      // 2 MiB blocks so that large pages can be used
    SpreadAlloc sa;
    sa.chunk = ((size_t)array_bytes + gran - 1) / gran * gran;
    sa.dist = ((size_t)distance_bytes + gran - 1) / gran * gran;
    // Physical placement: the driver hands out device memory in creation order, so a spacer created between two
    // arrays pushes them apart; the spacers are released again before returning.
    std::vector<hipMemGenericAllocationHandle_t> spacers;
    for (int32_t i = 0; i < n_arrays && e == hipSuccess; ++i) {
        hipMemGenericAllocationHandle_t h;
        if ((e = hipMemCreate(&h, sa.chunk, &prop, 0)) != hipSuccess) break;
        sa.handles.push_back(h);
        if (i + 1 < n_arrays && sa.dist > sa.chunk) {
            if ((e = hipMemCreate(&h, sa.dist - sa.chunk, &prop, 0)) != hipSuccess) break;
            spacers.push_back(h);
        }
    }
    for (auto h : spacers) (void)hipMemRelease(h);
    void *va = nullptr;
    if (e == hipSuccess && (e = hipMemAddressReserve(&va, sa.dist * (size_t)n_arrays, 0, nullptr, 0)) == hipSuccess)
        sa.reserved = true;
    hipMemAccessDesc access = {};
    access.location = prop.location;
    access.flags = hipMemAccessFlagsProtReadWrite;
    for (size_t i = 0; e == hipSuccess && i < sa.handles.size(); ++i) {
        char *p = static_cast<char *>(va) + i * sa.dist;
        if ((e = hipMemMap(p, sa.chunk, 0, sa.handles[i], 0)) != hipSuccess) break;
        sa.mapped = i + 1;
        e = hipMemSetAccess(p, sa.chunk, &access, 1);
    }
    if (e != hipSuccess) {
        spread_release(va, sa);
        return hip_fail(e, "spread allocation (HIP virtual memory management)");
    }
    {
        std::lock_guard<std::mutex> lock(g_spread_mutex);
        g_spread[va] = sa;
    }
    *base = va;
    if (actual_distance_bytes) *actual_distance_bytes = (int64_t)sa.dist;
    return LAA_OK;
}

int laa_spread_free(void *base)
{
    if (!base) return LAA_OK;
    SpreadAlloc sa;
    {
        std::lock_guard<std::mutex> lock(g_spread_mutex);
        auto it = g_spread.find(base);
        if (it == g_spread.end()) return fail(LAA_EINVAL, "not a pointer returned by laa_spread_alloc");
        sa = it->second;
        g_spread.erase(it);
    }
    hipError_t e = hipDeviceSynchronize();
    spread_release(base, sa);
    return e == hipSuccess ? LAA_OK : hip_fail(e, "hipDeviceSynchronize before freeing a spread allocation");
}

// ---- chunked pool ------------------------------------------------------------------------------------------
namespace {
struct Pool {
    size_t chunk = 0;
    std::vector<hipMemGenericAllocationHandle_t> handles;   // one per chunk; 0 once released
    std::vector<bool> mapped;
    size_t reserved = 0;                                    // bytes of address range
};
std::map<void *, Pool> g_pools;                             // guarded by g_spread_mutex

void pool_release(void *base, Pool &pl)
{
    for (size_t i = 0; i < pl.handles.size(); ++i) {
        if (pl.mapped[i]) (void)hipMemUnmap(static_cast<char *>(base) + i * pl.chunk, pl.chunk);
        if (pl.handles[i]) (void)hipMemRelease(pl.handles[i]);
    }
    if (pl.reserved) (void)hipMemAddressFree(base, pl.reserved);
}
}  // namespace

int laa_pool_create(int64_t bytes, int64_t chunk_bytes, void **base, int64_t *actual_bytes, int64_t *actual_chunk_bytes)
{
    if (!base) return fail(LAA_EINVAL, "null base");
    *base = nullptr;
    if (bytes <= 0 || chunk_bytes <= 0) return fail(LAA_EINVAL, "need bytes > 0 and chunk_bytes > 0");
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(LAA_ENODEVICE, "no HIP device available");
    hipMemAllocationProp prop = {};
    prop.type = hipMemAllocationTypePinned;
    prop.location.type = hipMemLocationTypeDevice;
    prop.location.id = dev;
    size_t gran = 0;
    if ((e = hipMemGetAllocationGranularity(&gran, &prop, hipMemAllocationGranularityRecommended)) != hipSuccess)
        return hip_fail(e, "hipMemGetAllocationGranularity");
    if (gran < (size_t(2) << 20)) gran = size_t(2) << 20;
    Pool pl;
    pl.chunk = ((size_t)chunk_bytes + gran - 1) / gran * gran;
    const size_t n = ((size_t)bytes + pl.chunk - 1) / pl.chunk;
    if (n > 65536) return fail(LAA_EINVAL, "more than 65536 chunks: use larger chunks");
    void *va = nullptr;
    if ((e = hipMemAddressReserve(&va, n * pl.chunk, 0, nullptr, 0)) != hipSuccess)
        return hip_fail(e, "hipMemAddressReserve for a pool");
    pl.reserved = n * pl.chunk;
    hipMemAccessDesc access = {};
    access.location = prop.location;
    access.flags = hipMemAccessFlagsProtReadWrite;
    for (size_t i = 0; i < n; ++i) {
        hipMemGenericAllocationHandle_t h;
        if ((e = hipMemCreate(&h, pl.chunk, &prop, 0)) != hipSuccess) break;
        pl.handles.push_back(h);
        pl.mapped.push_back(false);
        char *p = static_cast<char *>(va) + i * pl.chunk;
        if ((e = hipMemMap(p, pl.chunk, 0, h, 0)) != hipSuccess) break;
        pl.mapped[i] = true;
        if ((e = hipMemSetAccess(p, pl.chunk, &access, 1)) != hipSuccess) break;
    }
    if (e != hipSuccess) {
        pool_release(va, pl);
        return hip_fail(e, "creating a pool (HIP virtual memory management)");
    }
    {
        std::lock_guard<std::mutex> lock(g_spread_mutex);
        g_pools[va] = pl;
    }
    *base = va;
    if (actual_bytes) *actual_bytes = (int64_t)(n * pl.chunk);
    if (actual_chunk_bytes) *actual_chunk_bytes = (int64_t)pl.chunk;
    return LAA_OK;
}

int laa_pool_trim(void *base, int32_t n_ranges, const int64_t *offsets, const int64_t *lengths)
{
    if (!base || n_ranges < 0 || (n_ranges > 0 && (!offsets || !lengths))) return fail(LAA_EINVAL, "bad arguments");
    std::lock_guard<std::mutex> lock(g_spread_mutex);
    auto it = g_pools.find(base);
    if (it == g_pools.end()) return fail(LAA_EINVAL, "not a pointer returned by laa_pool_create");
    Pool &pl = it->second;
    std::vector<bool> keep(pl.handles.size(), false);
    for (int32_t r = 0; r < n_ranges; ++r) {
        if (offsets[r] < 0 || lengths[r] <= 0 || (size_t)offsets[r] + (size_t)lengths[r] > pl.reserved)
            return fail(LAA_EINVAL, "range %d lies outside the pool", r);
        for (size_t c = (size_t)offsets[r] / pl.chunk; c <= ((size_t)offsets[r] + (size_t)lengths[r] - 1) / pl.chunk; ++c) {
            if (!pl.mapped[c]) return fail(LAA_EINVAL, "range %d touches a chunk that was released earlier", r);
            keep[c] = true;
        }
    }
    hipError_t e = hipDeviceSynchronize();                  // nothing may still be using what goes away
    if (e != hipSuccess) return hip_fail(e, "hipDeviceSynchronize before trimming a pool");
    for (size_t c = 0; c < pl.handles.size(); ++c) {
        if (keep[c] || !pl.mapped[c]) continue;
        (void)hipMemUnmap(static_cast<char *>(base) + c * pl.chunk, pl.chunk);
        (void)hipMemRelease(pl.handles[c]);
        pl.mapped[c] = false;
        pl.handles[c] = hipMemGenericAllocationHandle_t();
    }
    return LAA_OK;
}

int laa_pool_free(void *base)
{
    if (!base) return LAA_OK;
    Pool pl;
    {
        std::lock_guard<std::mutex> lock(g_spread_mutex);
        auto it = g_pools.find(base);
        if (it == g_pools.end()) return fail(LAA_EINVAL, "not a pointer returned by laa_pool_create");
        pl = it->second;
        g_pools.erase(it);
    }
    hipError_t e = hipDeviceSynchronize();
    pool_release(base, pl);
    return e == hipSuccess ? LAA_OK : hip_fail(e, "hipDeviceSynchronize before freeing a pool");
}

int laa_debug_philox(const uint32_t ctr[4], const uint32_t key[2], uint32_t *out)
{
    if (!ctr || !key || !out) return fail(LAA_EINVAL, "null argument");
    hipError_t e = laa::debug_philox(ctr, key, out);
    return e == hipSuccess ? LAA_OK : hip_fail(e, "philox debug kernel");
}

int laa_debug_copy(float *dst, const float *src, int64_t n, void *hip_stream)
{
    if (!dst || !src || n <= 0 || n % 4 != 0 || !aligned(dst, 16) || !aligned(src, 16))
        return fail(LAA_EINVAL, "copy needs 16-byte aligned pointers and n a positive multiple of 4");
    hipError_t e = laa::launch_copy(dst, src, n, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? LAA_OK : hip_fail(e, "copy kernel launch");
}

}  // extern "C"
