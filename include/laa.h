/*
 * laa — Local AdaAlter optimizer hot path for AMD MI355X (gfx950): C ABI.
 *
 * Method: arXiv 1911.09030, Algorithm 3 ("Local AdaAlter").  W workers are
 * kept as a worker axis of replicas in one GPU's memory.  Each iteration every
 * worker takes a local step
 *     y   = x - eta * G / sqrt(B2_sync + t' * eps^2)        (Algorithm 3, update line)
 *     B2 += G o G                                            (same line, accumulator)
 * where B2_sync is the accumulator as it stood at the last synchronisation
 * (identical on all workers; Section 4.2, "Lazy update of the denominators")
 * and t' counts local steps since then.  Every H-th iteration x and B2 are
 * replaced by their means over the worker axis (Algorithm 3, Synchronize).
 *
 * Conventions for every call
 *   - Return value: LAA_OK (0) or a negative LAA_E* code; nothing throws.
 *     laa_last_error() gives a message for the calling thread's last failure.
 *   - "device" pointers are HIP device memory owned by the CALLER (allocated
 *     e.g. through PyTorch).  The library allocates only small bookkeeping
 *     buffers of its own, on first use (the dirty-row bitmap of the sparse
 *     steps and, for W <= 64, 8 bytes per table row naming the workers that
 *     stepped it; the row list of laa_sync after sparse steps and of
 *     laa_get_dirty_rows; sort keys and partial rows of the coalescing sparse step,
 *     48 KiB of reduction scratch for laa_diagnostics, 8 bytes for
 *     laa_run_periods_gen), freed by laa_destroy.
 *   - All kernels are enqueued on the stream given to laa_attach and return
 *     without waiting, except the getters that copy to host memory, which
 *     synchronise that stream.
 *   - Layout: x and acc are [W][d] row-major fp32 (worker-major, coordinate
 *     contiguous; optionally with a row pitch, see laa_attach_pitched); snap,
 *     a, xstar are [d] fp32.  64-bit indexing throughout.
 *     Rows must be 4-byte aligned; the vectorised kernels are used when all
 *     base pointers are 16-byte aligned and d % 4 == 0, a scalar path otherwise.
 *   - A handle is not thread-safe; use one handle from one thread at a time.
 */
#ifndef LAA_H
#define LAA_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct laa_ctx *laa_handle;

enum {
    LAA_OK = 0,
    LAA_EINVAL = -1,       /* bad argument (non-positive size, null pointer, ...) */
    LAA_ENOTATTACHED = -2, /* state buffers not attached yet                       */
    LAA_ESYNCDUE = -3,     /* H local steps taken since the last sync: call laa_sync */
    LAA_EALIGN = -4,       /* pointer not 4-byte aligned                            */
    LAA_EMODE = -5,        /* generator step without a generator, or bad mode       */
    LAA_EHIP = -6,         /* a HIP runtime call failed                             */
    LAA_ENODEVICE = -7     /* no usable GPU                                         */
};

/* Synthetic-gradient modes (a stand-in for the stochastic gradient of Algorithm 3,
 * evaluated at each worker's own iterate; see laa_set_generator). */
enum { LAA_GEN_QUADRATIC = 1, LAA_GEN_NOISE = 2 };
/* Where the per-worker shift of the optimum comes from in LAA_GEN_QUADRATIC. */
enum { LAA_OFF_NONE = 0, LAA_OFF_ARRAY = 1, LAA_OFF_PHILOX = 2 };
/* Update rules: Algorithm 3 (default), and the paper's two comparison methods. */
enum { LAA_ALGO_LOCAL_ADAALTER = 0, LAA_ALGO_DIST_ADAGRAD = 1, LAA_ALGO_LOCAL_SGD = 2 };

const char *laa_last_error(void);

/* Create a handle for d coordinates, W workers, sync period H, step size eta and
 * the eps of Algorithm 3 (the kernels use eps^2, rounded once to fp32).  The
 * initial accumulator b0 defaults to 1 (the paper's experiments; the theorem
 * needs b0 >= 1).  Needs no GPU.  Errors: LAA_EINVAL for d<=0, W<=0, H<=0,
 * eps<0, non-finite eta, null out. */
int laa_create(int64_t d, int32_t W, int32_t H, double eta, double eps, laa_handle *out);

/* Release the handle and the library's own bookkeeping buffers (never the
 * caller's arrays).  Null is accepted. */
int laa_destroy(laa_handle h);

/* b0 of Algorithm 3's Initialize line; only before the first step. b0 >= 0. */
int laa_set_b0(laa_handle h, double b0);

/* Section 6.2 warm-up: eta_t = eta * min(1, t / warmup_steps) for the 1-based
 * iteration t; 0 switches it off (constant eta, as in Algorithm 3). */
int laa_set_warmup(laa_handle h, int64_t warmup_steps);

/* Choose the update rule.  LAA_ALGO_DIST_ADAGRAD is Algorithm 1 (mean gradient,
 * freshly updated accumulator under the root; use b0 = 0 for the paper's
 * B2_0 = 0) and LAA_ALGO_LOCAL_SGD is Algorithm 2; both run through
 * laa_step_dense / laa_step_gen only.  Only before the first step. */
int laa_set_algorithm(laa_handle h, int32_t algo);

/* Tuning knob for the dense kernels.  1, 2, 4 or 8 (must divide W; default: the largest that
 * does): a thread handles all W workers of its column group and loads that many workers' rows
 * before it starts computing.  0: in steps that do not average, every thread block handles ONE
 * worker of a 256-column tile instead (two read-modify-write streams per thread; the W blocks of
 * a tile run on the same XCD so that snap, a, xstar are re-read from its L2, not from HBM);
 * steps that average still use the default batch.  Results do not depend on the choice except
 * through the order of the worker-axis sum when W exceeds the batch. */
int laa_set_tile(laa_handle h, int32_t workers_per_batch);

/* Lazy replicas (off by default).  Right after a Synchronize every worker holds the same x and
 * the same B2 (= snap), so with this option a step or laa_sync that averages writes that common
 * state once (row 0 of x, and snap) instead of into all W rows, and the next step reads it from
 * there for every worker: per column one sync period moves 2W floats less on the averaging pass
 * and 2(W-1) floats less on the pass after it.  While the state is collapsed, rows 1..W-1 of x
 * and all rows of acc are stale; call laa_materialize before reading them (the library does so
 * itself before a sparse step, an Algorithm 2 step, or when the option is switched off).
 * Algorithm 1 has a single iterate: with this option it is kept in row 0 of x and in snap
 * throughout.  Results are bit-identical to the default. */
int laa_set_lazy_replicas(laa_handle h, int32_t on);
int laa_materialize(laa_handle h);

/* Hand over the state arrays (device, caller-owned, must outlive the handle's
 * use): x [W][d], acc [W][d] (running B2 of each worker), snap [d] (B2 at the
 * last sync), and the HIP stream (hipStream_t, may be null for the default
 * stream) on which all work is enqueued.  Attaching other arrays in the middle
 * of a period is allowed; the next sync then averages the whole table even if
 * only sparse steps were taken (as after laa_set_counters). */
int laa_attach(laa_handle h, float *x, float *acc, float *snap, void *hip_stream);

/* The same with rows `pitch` >= d elements apart: x, acc (and every other [W][.] array handed to
 * this handle: explicit gradients, stored offsets, laa_generate_gradient's output) are [W][pitch]
 * with the first d entries of each row used; the padding is never read or written.  For callers
 * whose per-worker arrays are padded or are slices of a larger buffer.  The 16-byte path needs
 * pitch % 4 == 0. */
int laa_attach_pitched(laa_handle h, float *x, float *acc, float *snap, int64_t pitch, void *hip_stream);

/* Algorithm 3, Initialize: x[w] = x0 for every w (x0 device [d], or null for
 * zero), acc = snap = b0^2, counters reset, dirty rows cleared. */
int laa_init_state(laa_handle h, const float *x0);

/* One local step of every worker with explicit gradients grads [W][d] (device),
 * already evaluated at the workers' current x.  LAA_ESYNCDUE after H steps
 * without laa_sync. */
int laa_local_step_dense(laa_handle h, const float *grads);

/* Configure the fused synthetic gradient.  a, xstar [d] and off [W][d] are
 * device arrays owned by the caller and read on every generator step.
 *   LAA_GEN_QUADRATIC: g = a_j (x_wj - (xstar_j + off_wj)) + noise_scale * n_wjt
 *   LAA_GEN_NOISE    : g = a_j * n_wjt            (xstar, off unused, may be null)
 * n_wjt ~ N(0,1) from Philox4x32-10: counter (q mod 2^32, w, t, 3 + 16 (q div 2^32))
 * with q = j/4, key = seed, the four words mapped to u = ((r>>9)+0.5) 2^-23 and
 * Box-Muller pairs (u0,u1),(u2,u3) giving the normals of coordinates 4q..4q+3;
 * j and w are global indices (laa_set_shard), t the 1-based iteration.  off_mode
 * LAA_OFF_PHILOX regenerates off_wj = off_scale * normal from the same counter
 * with t = 0 and 2 in place of 3 instead of reading an array; LAA_OFF_ARRAY reads
 * off; LAA_OFF_NONE uses zero.  noise_scale and off_scale are standard deviations:
 * finite and >= 0 (LAA_EINVAL otherwise). */
int laa_set_generator(laa_handle h, int32_t mode, uint64_t seed, const float *a, const float *xstar,
                      const float *off, int32_t off_mode, float noise_scale, float off_scale);

/* This handle holds a shard of a larger problem: its column j is global column first_column + j
 * (first_column a multiple of 4, so that the four normals of one Philox block stay together) and its
 * worker w is global worker first_worker + w.  The generator's counters use the global indices, so
 * a run split by columns (each shard with all W workers; nothing is exchanged) or by workers (one
 * worker or a few per shard, the deployment of Algorithm 3; the local steps need no exchange and the
 * Synchronize step becomes an all-reduce outside this library) draws the random numbers of the unsplit
 * run.  Default 0, 0.  Explicit-gradient and sparse steps are not affected. */
int laa_set_shard(laa_handle h, int64_t first_column, int32_t first_worker);

/* One local step with the gradient generated in the kernel at iteration t+1. */
int laa_local_step_gen(laa_handle h);

/* n_periods whole periods of Algorithm 3 with the generator: each is H calls of laa_step_gen (the
 * last one averages).  Must be called right after a sync (or at the start).  The H kernel launches
 * of a period are recorded once into a HIP graph and replayed, which removes most of the launch cost
 * when d is small enough for the launches to dominate; the iteration number the generator needs is
 * read from a device word that the graph advances.  Results are bit-identical to the same number of
 * laa_step_gen calls.  Periods run as plain launches instead (same results) on the legacy default
 * stream (null), which cannot be captured, during the warm-up of the learning rate, when the arrays
 * are not 16-byte aligned or d is not a multiple of 4, with laa_set_tile(h, 0), and the first time
 * after the configuration changed.  Allocates 8 bytes of device memory on first use. */
int laa_run_periods_gen(laa_handle h, int32_t n_periods);

/* How many periods laa_run_periods_gen has run by graph replay (the others ran as plain launches). */
int laa_get_replay_count(laa_handle h, int64_t *periods_replayed);

/* Write the gradient the next generator step would use into out [W][d] (device),
 * without stepping.  For tests and for pre-computing gradient pools. */
int laa_generate_gradient(laa_handle h, float *out);

/* One local step with row-sparse gradients: the table is d / row_len rows of
 * row_len floats; worker w updates rows idx[w][0..k) (device int32, [W][k])
 * with values vals [W][k][row_len] (device).  Rows listed by one worker in one
 * call must be distinct unless laa_set_sparse_coalesce is on (different workers
 * may always list the same row).  Rows that are not listed are left untouched,
 * which is exactly Algorithm 3 with a zero gradient there.  Indices outside [0, d/row_len) are skipped and counted
 * (laa_get_counters bad_indices).  row_len must be a multiple of 4. */
int laa_local_step_sparse(laa_handle h, const int32_t *idx, const float *vals, int32_t k, int32_t row_len);

/* Allow one worker to list a row several times in one sparse step (a batch of tokens with repeated
 * words).  The row's gradient is then the sum of its entries, added in list order, and the step of
 * Algorithm 3 is taken once with that sum (so acc grows by the square of the sum).  Each worker's list
 * is sorted on the device first, which limits k to 8192 rows per worker and step (LAA_EINVAL beyond)
 * and costs a small extra pass; lists without repeats give bit-identical results either way.
 * The first coalescing step (and the first after row_len grew) allocates the sort keys and the partial rows
 * for that limit (8 W KiB and 2 KiB W row_len), which waits for the device like any hipMalloc; later
 * steps allocate nothing.  Off by default. */
int laa_set_sparse_coalesce(laa_handle h, int32_t on);

/* Algorithm 3, Synchronize: x[w] and acc[w] become the means over w, snap the
 * mean acc.  After only sparse steps just the rows touched since the last sync
 * are averaged (all other rows are already equal on every worker), and of such
 * a row only the rows of the workers that stepped it and of one that did not are
 * read (the others hold the same values; W <= 64): the result is bit for bit
 * the one that reading every worker's row gives.  A call with
 * no step since the last sync is a no-op; an early call (fewer than H steps) is
 * allowed and restarts t' at 1. */
int laa_sync(laa_handle h);

/* laa_sync for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the same result bit for bit, but the scratch of the averaging after sparse
 * steps (the ascending list of touched rows, its length, the block counts of the bitmap compaction) lives in
 * a static device array of the library, 4 MiB + 512 bytes per GPU, instead of buffers that laa_sync and
 * laa_get_dirty_rows allocate when they first need them.  Calls no hipMalloc / hipFree; the table may have at
 * most 1 048 576 rows (LAA_EINVAL beyond: nothing is enqueued and nothing changes, use laa_sync).  The
 * handle's device must be the current one.  Every call on a GPU uses that GPU's one array: calls whose
 * kernels can overlap (handles on different streams or threads) race; calls on one stream are ordered and
 * need nothing cleared in between.  A dense averaging needs no scratch and runs exactly as in laa_sync. */
int laa_sync_static(laa_handle h);

/* One whole iteration of Algorithm 3: the local step and, when it is the H-th
 * since the last sync, the averaging, fused into one pass over the state. */
int laa_step_dense(laa_handle h, const float *grads);
int laa_step_gen(laa_handle h);
int laa_step_sparse(laa_handle h, const int32_t *idx, const float *vals, int32_t k, int32_t row_len);

/* Host-side counters: iterations done, local steps since the last sync, and the
 * number of out-of-range sparse indices skipped so far (this one synchronises
 * the stream).  Any pointer may be null. */
int laa_get_counters(laa_handle h, int64_t *t, int32_t *steps_since_sync, int64_t *bad_indices);

/* Resume from a checkpoint: the caller restores x, acc, snap itself (they are its arrays; call
 * laa_materialize before saving them when lazy replicas are on) and then sets the iteration count
 * and the number of local steps since the last sync that laa_get_counters reported.  The generator
 * continues with the same random numbers as an uninterrupted run.  The next laa_sync averages the
 * whole table even if only sparse steps follow (the rows touched before the checkpoint are unknown). */
int laa_set_counters(laa_handle h, int64_t t, int32_t steps_since_sync);

/* Rows touched by sparse steps since the last sync, ascending, into out (HOST,
 * capacity cap); *n receives the total count even if it exceeds cap.
 * Synchronises the stream. */
int laa_get_dirty_rows(laa_handle h, int32_t *out, int64_t cap, int64_t *n);

/* Diagnostics of the quadratic workload at the mean iterate xbar = (1/W) sum_w x_w (the auxiliary
 * variable of Section 5, which the convergence theorem is stated for), into out (HOST, 3 doubles):
 *   out[0] = ||xbar - xstar||^2
 *   out[1] = ||grad F(xbar)||^2,  grad F(xbar)_j = a_j (xbar_j - xstar_j - mean_w off_wj)
 *   out[2] = (1/W) sum_w ||x_w - xbar||^2      (how far the workers have drifted apart)
 * Needs LAA_GEN_QUADRATIC.  Sums are accumulated in fp64 in a fixed order (wavefront shuffles,
 * LDS, then one block over the per-block partials).  Synchronises the stream; allocates a 48 KiB
 * scratch buffer on first use. */
int laa_diagnostics(laa_handle h, double *out);

/* Byte counters for bandwidth accounting, for everything enqueued since laa_init_state; either pointer may be null.
 *   *moved_bytes:   what the launches read and write: x, acc of every worker and snap once per column, the
 *                   generator's arrays or the explicit gradients, the averaged state; with lazy replicas the
 *                   collapsed state counts as what it is (row 0 of x and snap, 8 bytes per column), and so do
 *                   laa_materialize, the sort keys of the coalescing step and the rows averaged after sparse steps
 *                   (per averaged row: x and acc rows of the workers that stepped it and of one that did not
 *                   read, every worker's rows and snap's written).
 *                   Dividing it by the elapsed time gives the rate the memory system delivered.
 *   *literal_bytes: the same iterations as Algorithm 3 spells them out, a local step over full replicas
 *                   (16 W + 4 bytes per column and the gradient's inputs) and a separate Synchronize pass
 *                   (16 W + 4; after sparse steps: that many bytes per element of the averaged rows) whenever
 *                   one averaged: the traffic that fusing, lazy replicas and the shared read of untouched
 *                   workers' rows save is still in it.
 * After sparse steps the averaged rows and the rows read are counted on the device: the call then synchronises the
 * stream. */
int laa_bytes_moved(laa_handle h, uint64_t *moved_bytes, uint64_t *literal_bytes);

/* Optional allocation helper for the state arrays (the library never needs it: any device memory
 * can be attached).  Allocates n_arrays arrays of array_bytes each whose starts are distance_bytes
 * apart in virtual AND, as far as the driver's placement allows, in physical address space, using
 * HIP's virtual-memory management: only the arrays themselves occupy device memory, the address
 * range between them is reserved but unmapped (touching it faults).  *base receives the first
 * array's address, array i starts at *base + i * (*actual_distance_bytes) (distance rounded up to
 * the 2 MiB mapping granularity).
 * Why: on MI355X, kernels that stream many arrays at once (the 2W rows of x and acc) mostly run
 * faster when those arrays are spread over most of the HBM address range than when they are
 * packed into one compact region (measured at d = 4e8, W = 8 with arrays 10 GB apart: 0.78-0.80 of
 * the HBM peak against 0.71-0.79).  Spreading makes bad placements rare; laa_pool_create below lets a
 * caller find a good one by measurement.
 * Physical spreading is obtained by creating a temporary spacer block between consecutive arrays
 * and releasing all spacers before returning; it relies on the driver handing out memory in
 * creation order and silently degrades to an ordinary allocation otherwise.
 * laa_spread_free synchronises the device, unmaps and releases everything; pass the base pointer.
 * Errors: LAA_EINVAL (sizes, unknown pointer), LAA_EHIP (out of memory or address space). */
int laa_spread_alloc(int32_t n_arrays, int64_t array_bytes, int64_t distance_bytes, void **base,
                     int64_t *actual_distance_bytes);
int laa_spread_free(void *base);

/* A pool of device memory for choosing WHERE the state arrays live (optional, like laa_spread_alloc).
 * laa_pool_create maps `bytes` of device memory, created as separate physical chunks of chunk_bytes (both
 * rounded up to the mapping granularity), back to back into one address range starting at *base.
 * Why: on MI355X the rate of a kernel that streams 2W + 3 arrays at once depends on where those arrays sit in
 * physical memory relative to one another (measured at d = 4e8, W = 8: 0.69 to 0.80 of the HBM peak over
 * 235 placements inside one 260 GB range), and nothing but a measurement tells a good placement from a bad
 * one.  A caller takes a pool of most of the free memory, times the step on candidate placements inside it
 * (arrays are just offsets into the pool), keeps the best and gives the rest back:
 * laa_pool_trim unmaps and releases every chunk that none of the n_ranges byte ranges [offsets[r],
 * offsets[r] + lengths[r]) touches; the kept chunks stay where they are, physically and virtually, so the
 * measured placement is the one that is used; addresses in released chunks fault when touched.
 * laa_pool_free releases everything.  Both synchronise the device first.
 * Errors: LAA_EINVAL (sizes, unknown pointer, a range outside the pool or in a released chunk), LAA_EHIP
 * (out of memory or address space). */
int laa_pool_create(int64_t bytes, int64_t chunk_bytes, void **base, int64_t *actual_bytes, int64_t *actual_chunk_bytes);
int laa_pool_trim(void *base, int32_t n_ranges, const int64_t *offsets, const int64_t *lengths);
int laa_pool_free(void *base);

/* Test hook: four raw Philox4x32-10 words for one counter/key, computed on the
 * device, copied to out (HOST, 4 words). */
int laa_debug_philox(const uint32_t ctr[4], const uint32_t key[2], uint32_t *out);

/* A plain device-to-device copy kernel of n floats on the given stream; used to
 * calibrate profiler byte counters against a known volume. */
int laa_debug_copy(float *dst, const float *src, int64_t n, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* LAA_H */
