// Internal launcher interface between the C-ABI layer (laa_api.hip) and the
// gfx950 kernels (laa_kernels.hip).  Plain device pointers and sizes only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace laa {

enum GradSource { GRAD_EXPLICIT = 0, GRAD_QUADRATIC = 1, GRAD_NOISE = 2 };
enum OffsetSource { OFFSET_NONE = 0, OFFSET_ARRAY = 1, OFFSET_PHILOX = 2 };
enum Algo { ALGO_LOCAL_ADAALTER = 0, ALGO_DIST_ADAGRAD = 1, ALGO_LOCAL_SGD = 2 };

struct StepArgs {
    float *x;            // [W][pitch], the first d entries of each row used
    float *acc;          // [W][pitch]
    float *snap;         // [d]
    const float *grads;  // [W][d] explicit gradients, or null
    const float *a;      // [d]
    const float *xstar;  // [d]
    const float *off;    // [W][d]
    float *grad_out;     // [W][d]: write the generated gradient here instead of stepping
    int64_t d;
    int64_t pitch;       // elements between consecutive workers' rows of x, acc, grads, off, grad_out (>= d)
    int32_t W;
    float eta;           // eta_t of this iteration
    float pad;           // t' * eps^2
    float eps2;
    float noise_scale, off_scale;  // standard deviations of the noise and of the per-worker offsets (>= 0)
    float noise_c, off_c;          // -2 ln2 sigma^2 of each: the normals' radii come out scaled (set by launch_step)
    uint32_t seed_lo, seed_hi;
    int64_t col0;        // global index of column 0 (multiple of 4) and
    int32_t w0;          // global index of worker 0: the generator's counters are global
    uint32_t t_lo;       // iteration number of this step (low 32 bits), Philox counter word
    const uint32_t *t_dev; // if not null: a device word added to t_lo (iteration count at the start of a replayed graph)
    int32_t grad_source, off_source;
    bool sync;           // average over the worker axis in the same pass
    bool vec4;           // pointers 16-byte aligned and d % 4 == 0
    int32_t wt;          // workers loaded per batch (1, 2, 4 or 8; must divide W)
    bool split;          // non-sync steps: one worker per thread block instead of all W (see block_work)
    bool collapsed_in;   // the common post-sync state is held once: x in row 0, B2 in snap
    bool collapsed_out;  // with sync: write the means to row 0 of x and to snap only
    int32_t algo;
};

hipError_t launch_step(const StepArgs &a, hipStream_t s);
hipError_t launch_mean(float *x, float *acc, float *snap, int64_t d, int64_t pitch, int32_t W, bool vec4, int32_t wt,
                       bool x_only, bool collapse, hipStream_t s);
hipError_t launch_materialize(float *x, float *acc, const float *snap, int64_t d, int64_t pitch, int32_t W,
                              hipStream_t s);
hipError_t launch_init(float *x, float *acc, float *snap, const float *x0, float b0sq, int64_t d, int64_t pitch,
                       int32_t W, hipStream_t s);
hipError_t launch_fill_u32(uint32_t *p, uint32_t v, int64_t n, hipStream_t s);
// *p += v by one thread (the iteration counter of a replayed period)
hipError_t launch_add_u32(uint32_t *p, uint32_t v, hipStream_t s);

struct SparseArgs {
    float *x, *acc, *snap;
    const int32_t *idx;  // [W][k]
    const float *vals;   // [W][k][row_len]
    const uint64_t *keys; // [W][k] sorted (row << 32 | position in the list), coalescing step only
    float *partials;     // coalesce_partial_rows(W, k) rows of row_len floats, coalescing step only
    uint32_t *dirty;     // bitmap, one bit per row
    unsigned long long *touched; // one word per row: bit w set once worker w has stepped the row (null: not recorded)
    unsigned long long *bad; // count of skipped out-of-range indices
    int64_t d;
    int64_t pitch;
    int64_t n_rows;
    int32_t W, k, row_len;
    float eta, pad;
};
hipError_t launch_sparse_step(const SparseArgs &a, hipStream_t s);
// Largest k the coalescing step takes: one thread block sorts a worker's list in LDS.
int32_t coalesce_max_k();
// Rows of row_len floats the coalescing step needs for partial sums of long runs.
int64_t coalesce_partial_rows(int32_t W, int32_t k);
// Sort every worker's list by (row, position) into keys [W][k]; out-of-range rows go to the end.
hipError_t launch_sort_rows(const int32_t *idx, uint64_t *keys, int32_t W, int32_t k, int64_t n_rows, hipStream_t s);
// Row-sparse step on sorted lists: entries of one worker that list the same row are added up first.
hipError_t launch_sparse_step_coalesce(const SparseArgs &a, hipStream_t s);
// bitmap -> ascending row list (device) + count (device); scratch holds compact_scratch_words(n_rows) uint32
int64_t compact_scratch_words(int64_t n_rows);
hipError_t launch_compact_dirty(const uint32_t *dirty, int64_t n_rows, int32_t *list, uint32_t *count,
                                uint32_t *scratch, hipStream_t s);
// touched (may be null, must be null when W > 64): per row, the workers that stepped it since the last averaging; the
// others' rows still hold the last averaged state, so one of them is read in place of all of them.
// totals (may be null), for byte accounting: totals[0] += rows averaged, totals[1] += worker rows read per matrix.
hipError_t launch_mean_rows(float *x, float *acc, float *snap, int64_t pitch, int32_t W, int32_t wt, int32_t row_len,
                            const int32_t *list, const uint32_t *count, const unsigned long long *touched,
                            unsigned long long *totals, hipStream_t s);
int32_t diag_scratch_doubles();
hipError_t launch_diagnostics(const StepArgs &a, double *scratch, hipStream_t s);
hipError_t launch_copy(float *dst, const float *src, int64_t n, hipStream_t s);
hipError_t debug_philox(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

}  // namespace laa
