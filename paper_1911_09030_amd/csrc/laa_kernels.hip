// Local AdaAlter (arXiv 1911.09030, Algorithm 3) kernels for gfx950 (MI355X, CDNA4): this file holds the 16-byte
// instantiations of the dense kernels (templates in laa_dense.inl), state initialisation and expansion, the
// row-sparse step and its bookkeeping, the diagnostics reduction and all launchers.
#include "laa_dense.inl"

namespace laa {

// Undo the collapse: x[w] = x[0] for w >= 1, acc[w] = snap for every w.
__global__ __launch_bounds__(BLOCK) void materialize_kernel(float *__restrict__ x, float *__restrict__ acc,
                                                            const float *__restrict__ snap, int64_t d, int64_t pitch,
                                                            int32_t W)
{
    const int64_t j = (int64_t)blockIdx.x * BLOCK + threadIdx.x;
    if (j >= d) return;
    const float xv = x[j], bv = snap[j];
    acc[j] = bv;
    for (int32_t w = 1; w < W; ++w) {
        x[(int64_t)w * pitch + j] = xv;
        acc[(int64_t)w * pitch + j] = bv;
    }
}

// Algorithm 3, Initialize: x[w] = x0 (or 0), acc = snap = b0^2.
__global__ __launch_bounds__(BLOCK) void init_kernel(float *__restrict__ x, float *__restrict__ acc,
                                                     float *__restrict__ snap, const float *__restrict__ x0,
                                                     float b0sq, int64_t d, int64_t pitch, int32_t W)
{
    const int64_t j = (int64_t)blockIdx.x * BLOCK + threadIdx.x;
    if (j >= d) return;
    const float v = x0 ? x0[j] : 0.0f;
    for (int32_t w = 0; w < W; ++w) {
        x[(int64_t)w * pitch + j] = v;
        acc[(int64_t)w * pitch + j] = b0sq;
    }
    snap[j] = b0sq;
}

__global__ __launch_bounds__(BLOCK) void fill_u32_kernel(uint32_t *p, uint32_t v, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * BLOCK + threadIdx.x;
    if (i < n) p[i] = v;
}

__global__ void add_u32_kernel(uint32_t *p, uint32_t v)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) *p += v;
}

__global__ __launch_bounds__(BLOCK) void copy_kernel(v4f *__restrict__ dst, const v4f *__restrict__ src, int64_t n4)
{
    const int64_t i = (int64_t)blockIdx.x * BLOCK + threadIdx.x;
    if (i < n4) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// ------------------------------------------------------------------------------------------
// Row-sparse step: one wavefront per (worker, listed row).  Rows not listed are not touched: with a zero
// gradient Algorithm 3 leaves y = x and A2 = B2.  The row's bit in the dirty bitmap is set so the next
// sync averages only rows some worker changed.
static constexpr int WAVE = 64;
static constexpr int WAVES_PER_BLOCK = BLOCK / WAVE;
// (64-thread blocks: the same 0.129 ms on the embedding workload; non-temporal accesses to x and acc: 0.137-0.147 ms,
// the frequent rows are served from the caches.)
// Row r has been stepped by worker w: its bit in the bitmap, and the worker's bit in the row's word.
__device__ __forceinline__ void mark_row(const SparseArgs &a, int32_t r, int32_t w)
{
    atomicOr(&a.dirty[r >> 5], 1u << (r & 31));
    if (a.touched) atomicOr(&a.touched[r], 1ull << w);
}

__global__ __launch_bounds__(BLOCK) void sparse_step_kernel(const SparseArgs a)
{
    const int64_t pair = (int64_t)blockIdx.x * WAVES_PER_BLOCK + (threadIdx.x / WAVE);
    const int lane = threadIdx.x % WAVE;
    if (pair >= (int64_t)a.W * a.k) return;
    const int32_t w = (int32_t)(pair / a.k);
    const int32_t r = a.idx[pair];
    if (r < 0 || (int64_t)r >= a.n_rows) {
        if (lane == 0) atomicAdd(a.bad, 1ull);
        return;
    }
    const float *gv = a.vals + pair * a.row_len;
    const int64_t col = (int64_t)r * a.row_len;
    float *xr = a.x + (int64_t)w * a.pitch + col;
    float *br = a.acc + (int64_t)w * a.pitch + col;
    const float *sr = a.snap + col;
    for (int32_t e = lane * 4; e < a.row_len; e += WAVE * 4) {
        const Pack<4> g = ld<4, true>(gv + e);
        const Pack<4> s = ld<4, false>(sr + e);
        Pack<4> xv = ld<4, false>(xr + e), bv = ld<4, false>(br + e);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const float step = a.eta / sqrtf(s.v[c] + a.pad);
            xv.v[c] = fmaf(-g.v[c], step, xv.v[c]);
            bv.v[c] = fmaf(g.v[c], g.v[c], bv.v[c]);
        }
        st<4, false>(xr + e, xv);
        st<4, false>(br + e, bv);
    }
    if (lane == 0) mark_row(a, r, w);
}

// Row-sparse step for lists in which one worker may name a row several times (a batch of tokens with repeated
// words): the gradient of that row is the sum of its entries, and Algorithm 3 is applied once to the sum.
// Pass 1 sorts each worker's list by (row, position) in LDS, one thread block per worker (bitonic network on
// 64-bit keys); pass 2 gives one wavefront to every sorted position, the wavefront at the first entry of a row
// adds the entries of the run in list order and takes the step, the others leave at once.
static constexpr int SORT_THREADS = 1024;
static constexpr int SORT_MAX_K = 8192;                      // 64 KiB of LDS
static constexpr uint32_t ROW_INVALID = 0xFFFFFFFEu;         // out-of-range rows sort behind every valid row

__global__ __launch_bounds__(SORT_THREADS) void sort_rows_kernel(const int32_t *__restrict__ idx,
                                                                 uint64_t *__restrict__ keys, int32_t k, int32_t kp,
                                                                 int64_t n_rows)
{
    extern __shared__ uint64_t sort_sh[];                    // kp keys, kp a power of two >= k
    const int64_t base = (int64_t)blockIdx.x * k;
    for (int32_t i = threadIdx.x; i < kp; i += SORT_THREADS) {
        uint64_t key = ~0ull;                                // padding sorts last
        if (i < k) {
            const int32_t r = idx[base + i];
            const uint32_t rr = (r < 0 || (int64_t)r >= n_rows) ? ROW_INVALID : (uint32_t)r;
            key = ((uint64_t)rr << 32) | (uint32_t)i;
        }
        sort_sh[i] = key;
    }
    __syncthreads();
    for (int32_t size = 2; size <= kp; size <<= 1) {
        for (int32_t stride = size >> 1; stride > 0; stride >>= 1) {
            for (int32_t t = threadIdx.x; t < (kp >> 1); t += SORT_THREADS) {
                const int32_t lo = 2 * t - (t & (stride - 1));        // the pair (lo, lo + stride)
                const int32_t hi = lo + stride;
                const bool ascending = (lo & size) == 0;
                const uint64_t u = sort_sh[lo], v = sort_sh[hi];
                if ((u > v) == ascending) { sort_sh[lo] = v; sort_sh[hi] = u; }
            }
            __syncthreads();
        }
    }
    for (int32_t i = threadIdx.x; i < k; i += SORT_THREADS) keys[base + i] = sort_sh[i];
}

// Sorted entries that list one row form a run.  A run is cut at every SEG-th sorted position, so that a word that
// fills a large part of the batch is added up by many wavefronts:
//   phase 0: the wavefront at the first entry of a run, and at every position that is a multiple of SEG inside a run,
//            adds the entries from its position to the next multiple of SEG (or the end of the run) in list order.
//            If that is the whole run it takes the step; otherwise it stores the sum as a partial row.
//   phase 1: the wavefront at the first entry of a run that crosses a multiple of SEG adds the partial rows in
//            order and takes the step.
// Partial rows: two per bucket of SEG positions (the odd one for a run that starts in the bucket, the even one for the
// run that enters it from the left); at most one of each exists.
static constexpr int SEG = 32;
static constexpr int GATHER = 8;                                     // loads in flight while adding in order

__device__ __forceinline__ uint32_t key_row(uint64_t key) { return (uint32_t)(key >> 32); }

__device__ __forceinline__ void sparse_row_update(const SparseArgs &a, float *xr, float *br, const float *sr, int32_t e,
                                                  const Pack<4> &g)
{
    const Pack<4> s = ld<4, false>(sr + e);
    Pack<4> xv = ld<4, false>(xr + e), bv = ld<4, false>(br + e);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const float step = a.eta / sqrtf(s.v[c] + a.pad);
        xv.v[c] = fmaf(-g.v[c], step, xv.v[c]);
        bv.v[c] = fmaf(g.v[c], g.v[c], bv.v[c]);
    }
    st<4, false>(xr + e, xv);
    st<4, false>(br + e, bv);
}

template <int PHASE>
__global__ __launch_bounds__(BLOCK) void sparse_step_coalesce_kernel(const SparseArgs a)
{
    const int64_t pair = (int64_t)blockIdx.x * WAVES_PER_BLOCK + (threadIdx.x / WAVE);
    const int lane = threadIdx.x % WAVE;
    if (pair >= (int64_t)a.W * a.k) return;
    const int32_t w = (int32_t)(pair / a.k);
    const int32_t p = (int32_t)(pair - (int64_t)w * a.k);
    const uint64_t *kw = a.keys + (int64_t)w * a.k;
    const uint64_t key = kw[p];
    const uint32_t r = key_row(key);
    if (r == ROW_INVALID) {
        if (PHASE == 0 && lane == 0) atomicAdd(a.bad, 1ull);
        return;
    }
    const bool head = p == 0 || key_row(kw[p - 1]) != r;             // first entry of its run
    const int32_t bnd = (p / SEG + 1) * SEG;                         // next multiple of SEG
    const bool goes_on = bnd < a.k && key_row(kw[bnd]) == r;         // sorted: then all of [p, bnd] lists r
    const int64_t buckets = (a.k + SEG - 1) / SEG;                   // per worker
    const int64_t bucket = (int64_t)w * buckets + p / SEG;
    const int64_t col = (int64_t)r * a.row_len;
    float *xr = a.x + (int64_t)w * a.pitch + col;
    float *br = a.acc + (int64_t)w * a.pitch + col;
    const float *sr = a.snap + col;
    if constexpr (PHASE == 0) {
        if (!head && p % SEG != 0) return;
        int32_t n = 1;                                               // entries of this piece: p .. p + n - 1 < bnd
        {
            const int32_t q = p + 1 + lane;
            const bool same = q < bnd && q < a.k && key_row(kw[q]) == r;
            n += __builtin_ctzll(~__ballot(same));                   // SEG - 1 < 64: some lane is always false
        }
        const bool whole = head && !goes_on;
        const float *vw = a.vals + (int64_t)w * a.k * a.row_len;
        float *dst = a.partials + (2 * bucket + (head ? 1 : 0)) * a.row_len;
        for (int32_t e = lane * 4; e < a.row_len; e += WAVE * 4) {
            Pack<4> g = ld<4, true>(vw + (int64_t)(uint32_t)key * a.row_len + e);
            for (int32_t q = 1; q < n; q += GATHER) {
                Pack<4> v[GATHER];
#pragma unroll
                for (int u = 0; u < GATHER; ++u)
                    if (q + u < n) v[u] = ld<4, true>(vw + (int64_t)(uint32_t)kw[p + q + u] * a.row_len + e);
#pragma unroll
                for (int u = 0; u < GATHER; ++u)
                    if (q + u < n) {
#pragma unroll
                        for (int c = 0; c < 4; ++c) g.v[c] += v[u].v[c];
                    }
            }
            if (whole) sparse_row_update(a, xr, br, sr, e, g);
            else st<4, false>(dst + e, g);
        }
        if (whole && lane == 0) mark_row(a, r, w);
    } else {
        if (!head || !goes_on) return;
        int32_t m = 0;                                               // pieces after the first: at bnd, bnd + SEG, ...
        for (int32_t b0 = bnd; b0 < a.k; b0 += WAVE * SEG) {
            const int64_t b = (int64_t)b0 + (int64_t)lane * SEG;
            const bool same = b < a.k && key_row(kw[b]) == r;
            const unsigned long long mask = __ballot(same);
            if (mask != ~0ull) { m += __builtin_ctzll(~mask); break; }
            m += WAVE;
        }
        const float *first = a.partials + (2 * bucket + 1) * a.row_len;
        const float *rest = a.partials + 2 * (bucket + 1) * a.row_len;       // even rows of the following buckets
        for (int32_t e = lane * 4; e < a.row_len; e += WAVE * 4) {
            Pack<4> g = ld<4, false>(first + e);
            for (int32_t q = 0; q < m; q += GATHER) {
                Pack<4> v[GATHER];
#pragma unroll
                for (int u = 0; u < GATHER; ++u)
                    if (q + u < m) v[u] = ld<4, false>(rest + (int64_t)(q + u) * 2 * a.row_len + e);
#pragma unroll
                for (int u = 0; u < GATHER; ++u)
                    if (q + u < m) {
#pragma unroll
                        for (int c = 0; c < 4; ++c) g.v[c] += v[u].v[c];
                    }
            }
            sparse_row_update(a, xr, br, sr, e, g);
        }
        if (lane == 0) mark_row(a, r, w);
    }
}

// Dirty bitmap -> ascending list of rows.  Three passes: per-block bit counts, scan of the block
// counts by one block, then each block writes its rows at its offset.
static constexpr int WORDS_PER_THREAD = 4;
static constexpr int WORDS_PER_BLOCK = BLOCK * WORDS_PER_THREAD;

__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t *total)
{
    __shared__ uint32_t sh[BLOCK];
    const int t = threadIdx.x;
    sh[t] = v;
    __syncthreads();
    for (int o = 1; o < BLOCK; o <<= 1) {
        const uint32_t add = t >= o ? sh[t - o] : 0u;
        __syncthreads();
        sh[t] += add;
        __syncthreads();
    }
    const uint32_t incl = sh[t];
    *total = sh[BLOCK - 1];
    __syncthreads();
    return incl - v;
}

__global__ __launch_bounds__(BLOCK) void dirty_count_kernel(const uint32_t *__restrict__ dirty, int64_t n_words,
                                                            uint32_t *__restrict__ block_counts)
{
    const int64_t w0 = (int64_t)blockIdx.x * WORDS_PER_BLOCK + (int64_t)threadIdx.x * WORDS_PER_THREAD;
    uint32_t c = 0;
    for (int i = 0; i < WORDS_PER_THREAD; ++i)
        if (w0 + i < n_words) c += __popc(dirty[w0 + i]);
    uint32_t total;
    block_exclusive_scan(c, &total);
    if (threadIdx.x == 0) block_counts[blockIdx.x] = total;
}

__global__ __launch_bounds__(BLOCK) void dirty_scan_kernel(uint32_t *__restrict__ block_counts, int32_t n_blocks,
                                                           uint32_t *__restrict__ count)
{
    uint32_t running = 0;
    for (int32_t base = 0; base < n_blocks; base += BLOCK) {
        const int32_t i = base + threadIdx.x;
        const uint32_t v = i < n_blocks ? block_counts[i] : 0u;
        uint32_t total;
        const uint32_t ex = block_exclusive_scan(v, &total);
        if (i < n_blocks) block_counts[i] = running + ex;
        running += total;
    }
    if (threadIdx.x == 0) *count = running;
}

__global__ __launch_bounds__(BLOCK) void dirty_write_kernel(const uint32_t *__restrict__ dirty, int64_t n_words,
                                                            const uint32_t *__restrict__ block_offsets,
                                                            int32_t *__restrict__ list)
{
    const int64_t w0 = (int64_t)blockIdx.x * WORDS_PER_BLOCK + (int64_t)threadIdx.x * WORDS_PER_THREAD;
    uint32_t words[WORDS_PER_THREAD];
    uint32_t c = 0;
    for (int i = 0; i < WORDS_PER_THREAD; ++i) {
        words[i] = w0 + i < n_words ? dirty[w0 + i] : 0u;
        c += __popc(words[i]);
    }
    uint32_t total;
    uint32_t pos = block_offsets[blockIdx.x] + block_exclusive_scan(c, &total);
    for (int i = 0; i < WORDS_PER_THREAD; ++i) {
        uint32_t m = words[i];
        while (m) {
            const int b = __ffs(m) - 1;
            m &= m - 1;
            list[pos++] = (int32_t)((w0 + i) * 32 + b);
        }
    }
}

// Synchronize branch restricted to the listed rows.  The length of the list is only known on the device, so a fixed
// grid of one-wavefront blocks strides over the work items, an item being 256 consecutive floats of a listed row
// (16 bytes per lane) for all W workers: up to 2W non-temporal 16-byte loads in flight per lane, 2W + 1 stores.  The row
// number of the next item is fetched before the current item's loads are waited for.  Measured on the embedding
// workload (290 000 of 800 000 rows of 512 floats listed, W = 8; list compaction included) while every worker's
// row was read (with the shared read of untouched workers' rows below: 2.12 ms): 3.14 ms with 2 wavefronts
// per SIMD (8 blocks per CU), 3.18 with 3, 3.23 with 4, 3.17-3.21 uncapped with 32 blocks per CU; 3.35 with cached
// instead of non-temporal accesses, 3.33 with one block per item under a grid that covers the largest possible list
// (most of its blocks leave at once).
#ifndef LAA_ROWS_WAVES_PER_CU
#define LAA_ROWS_WAVES_PER_CU 8
#endif
#ifndef LAA_ROWS_NT
#define LAA_ROWS_NT true
#endif
static constexpr int N_CU = 256;                                     // MI355X
static constexpr bool ROWS_NT = LAA_ROWS_NT;

#ifndef LAA_ROWS_WAVES
#define LAA_ROWS_WAVES 2               // wavefronts per SIMD; the grid holds exactly that many per CU
#endif
// The workers that did not step a row since the last averaging all still hold that averaging's result in it, bit
// for bit; `touched` names the ones that did.  One untouched worker's row is read in place of every untouched
// worker's: the same values enter the same sum, so the mean is the one the full read gives.  (A row touched by a
// single worker costs 2 + 2 row reads instead of 2W; on the embedding workload a touched row has 1.97 touching
// workers on average.)
__device__ __forceinline__ uint64_t touched_workers(const unsigned long long *touched, int32_t row, int32_t W)
{
    const uint64_t all = W >= 64 ? ~0ull : (1ull << W) - 1;
    if (!touched) return all;
    const uint64_t m = touched[row];
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)m), hi = __builtin_amdgcn_readfirstlane((uint32_t)(m >> 32));
    const uint64_t u = (((uint64_t)hi << 32) | lo) & all;
    return u ? u : all;                    // a listed row with no worker recorded: read them all
}

template <int WT>
__global__ __launch_bounds__(WAVE) __attribute__((amdgpu_waves_per_eu(1, LAA_ROWS_WAVES))) void mean_rows_kernel(float *__restrict__ x, float *__restrict__ acc,
                                                         float *__restrict__ snap, int64_t pitch, int32_t W,
                                                         int32_t row_len, const int32_t *__restrict__ list,
                                                         const uint32_t *__restrict__ count,
                                                         const unsigned long long *__restrict__ touched,
                                                         unsigned long long *__restrict__ totals)
{
    const uint32_t n = *count;
    if (totals && blockIdx.x == 0 && threadIdx.x == 0) totals[0] += n;
    const uint32_t chunks = (uint32_t)(row_len + WAVE * 4 - 1) / (WAVE * 4);
    const uint64_t items = (uint64_t)n * chunks;
    uint64_t it = blockIdx.x;
    if (it >= items) return;
    const int lane = threadIdx.x;
    const MeanOf mean(W);
    const uint64_t all = W >= 64 ? ~0ull : (1ull << W) - 1;
    unsigned long long rows_read = 0;
    int32_t row = list[it / chunks];
    uint64_t m = touched_workers(touched, row, W);
    while (true) {
        const uint64_t nxt = it + gridDim.x;
        const bool more = nxt < items;
        const int32_t row_next = more ? list[nxt / chunks] : 0;
        const uint64_t m_next = more ? touched_workers(touched, row_next, W) : all;
        const int32_t chunk = (int32_t)(it % chunks);
        const int32_t e = chunk * (WAVE * 4) + lane * 4;
        const bool some_untouched = m != all;
        if (chunk == 0) rows_read += some_untouched ? (unsigned long long)__builtin_popcountll(m) + 1 : (unsigned long long)W;
        if (e < row_len) {
            const int64_t col = (int64_t)row * row_len + e;
            Pack<4> sx, sb, xu, bu;
#pragma unroll
            for (int c = 0; c < 4; ++c) sx.v[c] = sb.v[c] = xu.v[c] = bu.v[c] = 0.0f;
            if (some_untouched) {
                const int32_t u = __builtin_ctzll(~m & all);
                xu = ld<4, ROWS_NT>(x + (int64_t)u * pitch + col);
                bu = ld<4, ROWS_NT>(acc + (int64_t)u * pitch + col);
            }
            for (int32_t w0 = 0; w0 < W; w0 += WT) {
                Pack<4> xv[WT], bv[WT];
#pragma unroll
                for (int k = 0; k < WT; ++k) {
                    if (!some_untouched || ((m >> ((w0 + k) & 63)) & 1)) {
                        xv[k] = ld<4, ROWS_NT>(x + (int64_t)(w0 + k) * pitch + col);
                        bv[k] = ld<4, ROWS_NT>(acc + (int64_t)(w0 + k) * pitch + col);
                    } else {
                        xv[k] = xu;
                        bv[k] = bu;
                    }
                }
                const Pack<4> tx = tree_sum<4, WT>(xv), tb = tree_sum<4, WT>(bv);
#pragma unroll
                for (int c = 0; c < 4; ++c) { sx.v[c] += tx.v[c]; sb.v[c] += tb.v[c]; }
            }
#pragma unroll
            for (int c = 0; c < 4; ++c) { sx.v[c] = mean(sx.v[c]); sb.v[c] = mean(sb.v[c]); }
            for (int32_t w = 0; w < W; ++w) {
                st<4, ROWS_NT>(x + (int64_t)w * pitch + col, sx);
                st<4, ROWS_NT>(acc + (int64_t)w * pitch + col, sb);
            }
            st<4, false>(snap + col, sb);
        }
        if (!more) break;
        it = nxt;
        row = row_next;
        m = m_next;
    }
    if (totals && lane == 0 && rows_read) atomicAdd(totals + 1, rows_read);
}

// ------------------------------------------------------------------------------------------
// Diagnostics of the quadratic workload at the mean iterate xbar = (1/W) sum_w x_w (the auxiliary variable of
// Section 5): out[0] = ||xbar - xstar||^2, out[1] = ||grad F(xbar)||^2 with
// grad F(xbar)_j = a_j (xbar_j - xstar_j - mean_w off_wj), out[2] = (1/W) sum_w ||x_w - xbar||^2.
// Elementwise terms in fp32, sums in fp64: per thread, then across the wavefront with lane shuffles, across the
// block through LDS, one partial per block into `partial`; a second one-block kernel adds the partials in a fixed
// order, so the result does not depend on scheduling.
static constexpr int DIAG_BLOCKS = 2048;

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    return v;
}

// WT > 0: the table has exactly WT workers and a thread keeps their WT column groups in registers, so every row of x
// is read once (streaming loads); WT == 0: any W, the rows are read a second time for the deviations.  Both add in
// the same order.
template <int VEC, int OS, int WT>
__global__ __launch_bounds__(BLOCK) void diag_kernel(const StepArgs a, double *__restrict__ partial)
{
    double s0 = 0.0, s1 = 0.0, s2 = 0.0;
    const int64_t n_groups = (a.d + VEC - 1) / VEC;
    const float fw = (float)a.W;
    for (int64_t q = (int64_t)blockIdx.x * BLOCK + threadIdx.x; q < n_groups; q += (int64_t)gridDim.x * BLOCK) {
        const int64_t j = q * VEC;
        const Pack<VEC> av = ld<VEC, true>(a.a + j), xs = ld<VEC, true>(a.xstar + j);
        Pack<VEC> xbar, moff, dev;
#pragma unroll
        for (int e = 0; e < VEC; ++e) xbar.v[e] = moff.v[e] = dev.v[e] = 0.0f;
        if (a.collapsed_in) {                 // every worker holds row 0: the mean is that row, the deviations are zero
            xbar = ld<VEC, true>(a.x + j);
        } else if constexpr (WT > 0) {
            Pack<VEC> xv[WT];
#pragma unroll
            for (int w = 0; w < WT; ++w) xv[w] = ld<VEC, true>(a.x + (int64_t)w * a.pitch + j);
#pragma unroll
            for (int w = 0; w < WT; ++w)
#pragma unroll
                for (int e = 0; e < VEC; ++e) xbar.v[e] += xv[w].v[e];
#pragma unroll
            for (int e = 0; e < VEC; ++e) xbar.v[e] = xbar.v[e] / fw;
#pragma unroll
            for (int w = 0; w < WT; ++w)
#pragma unroll
                for (int e = 0; e < VEC; ++e) { const float t = xv[w].v[e] - xbar.v[e]; dev.v[e] = fmaf(t, t, dev.v[e]); }
        } else {
            for (int32_t w = 0; w < a.W; ++w) {
                const Pack<VEC> xv = ld<VEC, false>(a.x + (int64_t)w * a.pitch + j);
#pragma unroll
                for (int e = 0; e < VEC; ++e) xbar.v[e] += xv.v[e];
            }
#pragma unroll
            for (int e = 0; e < VEC; ++e) xbar.v[e] = xbar.v[e] / fw;
            for (int32_t w = 0; w < a.W; ++w) {
                const Pack<VEC> xv = ld<VEC, false>(a.x + (int64_t)w * a.pitch + j);
#pragma unroll
                for (int e = 0; e < VEC; ++e) { const float t = xv.v[e] - xbar.v[e]; dev.v[e] = fmaf(t, t, dev.v[e]); }
            }
        }
        if constexpr (OS != OFFSET_NONE) {
            for (int32_t w = 0; w < a.W; ++w) {
                if constexpr (OS == OFFSET_ARRAY) {
                    const Pack<VEC> o = ld<VEC, true>(a.off + (int64_t)w * a.pitch + j);
#pragma unroll
                    for (int e = 0; e < VEC; ++e) moff.v[e] += o.v[e];
                } else {
                    const uint64_t ja = (uint64_t)(j + a.col0);
                    const Normals4 m = normals4(a.seed_lo, a.seed_hi, STREAM_OFFSET, ja >> 2, (uint32_t)(w + a.w0), 0u, a.off_c);
                    const int lane0 = VEC == 4 ? 0 : (int)(ja & 3);
#pragma unroll
                    for (int e = 0; e < VEC; ++e) moff.v[e] += m.rad[(lane0 + e) >> 1] * m.trig[lane0 + e];
                }
            }
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const float dx = xbar.v[e] - xs.v[e];
            const float g = av.v[e] * (dx - moff.v[e] / fw);
            s0 += (double)dx * (double)dx;
            s1 += (double)g * (double)g;
            s2 += (double)(dev.v[e] / fw);
        }
    }
    __shared__ double sh[3][WAVES_PER_BLOCK];
    s0 = wave_sum(s0); s1 = wave_sum(s1); s2 = wave_sum(s2);
    const int lane = threadIdx.x % WAVE, wave = threadIdx.x / WAVE;
    if (lane == 0) { sh[0][wave] = s0; sh[1][wave] = s1; sh[2][wave] = s2; }
    __syncthreads();
    if (threadIdx.x < 3) {
        double t = 0.0;
        for (int k = 0; k < WAVES_PER_BLOCK; ++k) t += sh[threadIdx.x][k];
        partial[(int64_t)blockIdx.x * 3 + threadIdx.x] = t;
    }
}

// One wavefront per quantity: lane l adds the partials of blocks l, l + 64, ... in that order, then the lanes are
// added by the same shuffle tree as above: a fixed order again.
__global__ __launch_bounds__(3 * WAVE) void diag_final_kernel(const double *__restrict__ partial, int32_t n_blocks,
                                                             double *__restrict__ out)
{
    const int lane = threadIdx.x % WAVE, k = threadIdx.x / WAVE;
    double t = 0.0;
    for (int32_t b = lane; b < n_blocks; b += WAVE) t += partial[(int64_t)b * 3 + k];
    t = wave_sum(t);
    if (lane == 0) out[k] = t;
}

__global__ void philox_debug_kernel(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1,
                                    uint32_t *out)
{
    uint32_t r[4];
    philox4x32_10(c0, c1, c2, c3, k0, k1, r);
    if (threadIdx.x == 0 && blockIdx.x == 0)
        for (int i = 0; i < 4; ++i) out[i] = r[i];
}

// ------------------------------------------------------------------------------------------
// launchers
// -2 ln2 sigma^2, rounded once from double
static float normal_c(float sigma) { return (float)(-1.3862943611198906 * (double)sigma * (double)sigma); }

hipError_t launch_step(const StepArgs &a_in, hipStream_t s)
{
    StepArgs a = a_in;
    if (a.noise_scale < 0.0f || a.off_scale < 0.0f) return hipErrorInvalidValue;
    a.noise_c = normal_c(a.noise_scale);
    a.off_c = normal_c(a.off_scale);
    if (a.d <= 0 || a.W <= 0 || a.wt <= 0 || a.W % a.wt != 0 || !layout_ok(a.d, a.pitch, a.vec4)) return hipErrorInvalidValue;
    // one worker per block only for the plain Local AdaAlter step (no averaging in the same pass)
    a.split = a.split && a.vec4 && !a.sync && !a.grad_out && !a.collapsed_in && a.algo == ALGO_LOCAL_ADAALTER && a.W > 1;
    // Algorithm 1 keeps one iterate: with lazy replicas it lives in row 0 of x and in snap throughout
    if (a.algo == ALGO_LOCAL_SGD && (a.collapsed_in || a.collapsed_out)) return hipErrorInvalidValue;
    if (a.algo == ALGO_DIST_ADAGRAD && a.collapsed_in && !a.collapsed_out) return hipErrorInvalidValue;
    if (a.collapsed_out && !a.sync) return hipErrorInvalidValue;
    if (a.split) a.wt = 1;
    dim3 grid;
    if (a.vec4) {
        if (a.d % 4 != 0 || !dense_grid(a.d / 4, a.split, a.W, &grid)) return hipErrorInvalidValue;
        return launch_step_wt<4>(a, grid, s);
    }
    if (!dense_grid(a.d, false, a.W, &grid)) return hipErrorInvalidValue;
    // same batches as the vector path: the order of the worker-axis sum, and with it every bit of the result, does
    // not depend on alignment
    return launch_step_scalar(a, grid, s);
}

hipError_t launch_mean(float *x, float *acc, float *snap, int64_t d, int64_t pitch, int32_t W, bool vec4, int32_t wt,
                       bool x_only, bool collapse, hipStream_t s)
{
    if (d <= 0 || W <= 0 || wt <= 0 || W % wt != 0 || !layout_ok(d, pitch, vec4) || (x_only && collapse))
        return hipErrorInvalidValue;
    dim3 grid;
    if (vec4) {
        if (d % 4 != 0 || !dense_grid(d / 4, false, W, &grid)) return hipErrorInvalidValue;
        return launch_mean_wt<4>(x, acc, snap, d, pitch, W, wt, x_only, collapse, grid, s);
    }
    if (!dense_grid(d, false, W, &grid)) return hipErrorInvalidValue;
    return launch_mean_scalar(x, acc, snap, d, pitch, W, wt, x_only, collapse, grid, s);
}

hipError_t launch_init(float *x, float *acc, float *snap, const float *x0, float b0sq, int64_t d, int64_t pitch,
                       int32_t W, hipStream_t s)
{
    dim3 grid;
    if (!grid_for(d, &grid) || !layout_ok(d, pitch, false)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(init_kernel, grid, dim3(BLOCK), 0, s, x, acc, snap, x0, b0sq, d, pitch, W);
    return hipGetLastError();
}

hipError_t launch_materialize(float *x, float *acc, const float *snap, int64_t d, int64_t pitch, int32_t W,
                              hipStream_t s)
{
    dim3 grid;
    if (!grid_for(d, &grid) || pitch < d) return hipErrorInvalidValue;
    hipLaunchKernelGGL(materialize_kernel, grid, dim3(BLOCK), 0, s, x, acc, snap, d, pitch, W);
    return hipGetLastError();
}

hipError_t launch_add_u32(uint32_t *p, uint32_t v, hipStream_t s)
{
    if (!p) return hipErrorInvalidValue;
    hipLaunchKernelGGL(add_u32_kernel, dim3(1), dim3(WAVE), 0, s, p, v);
    return hipGetLastError();
}

hipError_t launch_fill_u32(uint32_t *p, uint32_t v, int64_t n, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    dim3 grid;
    if (!grid_for(n, &grid)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(fill_u32_kernel, grid, dim3(BLOCK), 0, s, p, v, n);
    return hipGetLastError();
}

int32_t diag_scratch_doubles() { return DIAG_BLOCKS * 3 + 3; }

// scratch: diag_scratch_doubles() doubles of device memory; the three results land in its last three entries
hipError_t launch_diagnostics(const StepArgs &a_in, double *scratch, hipStream_t s)
{
    StepArgs a = a_in;
    if (a.off_scale < 0.0f) return hipErrorInvalidValue;
    a.off_c = normal_c(a.off_scale);
    if (a.d <= 0 || a.W <= 0 || !a.a || !a.xstar || !scratch || !layout_ok(a.d, a.pitch, a.vec4)) return hipErrorInvalidValue;
    const int64_t n_groups = a.vec4 ? a.d / 4 : a.d;
    const int64_t want = (n_groups + BLOCK - 1) / BLOCK;
    const int32_t nb = (int32_t)(want < DIAG_BLOCKS ? want : DIAG_BLOCKS);
    double *out = scratch + DIAG_BLOCKS * 3;
    const dim3 grid((unsigned)nb), block(BLOCK);
#define LAA_DIAG_W(VEC, OS, WT) hipLaunchKernelGGL((diag_kernel<VEC, OS, WT>), grid, block, 0, s, a, scratch)
#define LAA_DIAG(VEC, OS)                                      \
    do {                                                       \
        if (a.W == 8) LAA_DIAG_W(VEC, OS, 8);                  \
        else if (a.W == 4) LAA_DIAG_W(VEC, OS, 4);             \
        else if (a.W == 2) LAA_DIAG_W(VEC, OS, 2);             \
        else LAA_DIAG_W(VEC, OS, 0);                           \
    } while (0)
    if (a.vec4) {
        if (a.d % 4 != 0) return hipErrorInvalidValue;
        if (a.off_source == OFFSET_ARRAY) LAA_DIAG(4, OFFSET_ARRAY);
        else if (a.off_source == OFFSET_PHILOX) LAA_DIAG(4, OFFSET_PHILOX);
        else LAA_DIAG(4, OFFSET_NONE);
    } else {
        if (a.off_source == OFFSET_ARRAY) LAA_DIAG(1, OFFSET_ARRAY);
        else if (a.off_source == OFFSET_PHILOX) LAA_DIAG(1, OFFSET_PHILOX);
        else LAA_DIAG(1, OFFSET_NONE);
    }
#undef LAA_DIAG_W
#undef LAA_DIAG
    hipLaunchKernelGGL(diag_final_kernel, dim3(1), dim3(3 * WAVE), 0, s, scratch, nb, out);
    return hipGetLastError();
}

hipError_t launch_copy(float *dst, const float *src, int64_t n, hipStream_t s)
{
    if (n <= 0 || n % 4 != 0) return hipErrorInvalidValue;
    dim3 grid;
    if (!grid_for(n / 4, &grid)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(copy_kernel, grid, dim3(BLOCK), 0, s, reinterpret_cast<v4f *>(dst),
                       reinterpret_cast<const v4f *>(src), n / 4);
    return hipGetLastError();
}

hipError_t launch_sparse_step(const SparseArgs &a, hipStream_t s)
{
    const int64_t pairs = (int64_t)a.W * a.k;
    if (pairs == 0) return hipSuccess;
    if (a.row_len <= 0 || a.row_len % 4 != 0 || a.n_rows * a.row_len != a.d || a.pitch < a.d || a.pitch % 4 != 0)
        return hipErrorInvalidValue;
    const int64_t nb = (pairs + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK;
    if (nb > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(sparse_step_kernel, dim3((unsigned)nb), dim3(BLOCK), 0, s, a);
    return hipGetLastError();
}

int32_t coalesce_max_k() { return SORT_MAX_K; }
int64_t coalesce_partial_rows(int32_t W, int32_t k) { return 2 * (int64_t)W * ((k + SEG - 1) / SEG); }

hipError_t launch_sort_rows(const int32_t *idx, uint64_t *keys, int32_t W, int32_t k, int64_t n_rows, hipStream_t s)
{
    if (W <= 0 || k < 0 || k > SORT_MAX_K || n_rows <= 0 || n_rows >= (int64_t)ROW_INVALID) return hipErrorInvalidValue;
    if (k == 0) return hipSuccess;
    int32_t kp = 2;
    while (kp < k) kp <<= 1;
    hipLaunchKernelGGL(sort_rows_kernel, dim3((unsigned)W), dim3(SORT_THREADS), (size_t)kp * sizeof(uint64_t), s, idx, keys,
                       k, kp, n_rows);
    return hipGetLastError();
}

hipError_t launch_sparse_step_coalesce(const SparseArgs &a, hipStream_t s)
{
    const int64_t pairs = (int64_t)a.W * a.k;
    if (pairs == 0) return hipSuccess;
    if (!a.keys || !a.partials || a.row_len <= 0 || a.row_len % 4 != 0 || a.n_rows * a.row_len != a.d || a.pitch < a.d || a.pitch % 4 != 0)
        return hipErrorInvalidValue;
    const int64_t nb = (pairs + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK;
    if (nb > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(sparse_step_coalesce_kernel<0>, dim3((unsigned)nb), dim3(BLOCK), 0, s, a);
    hipLaunchKernelGGL(sparse_step_coalesce_kernel<1>, dim3((unsigned)nb), dim3(BLOCK), 0, s, a);
    return hipGetLastError();
}

int64_t compact_scratch_words(int64_t n_rows)
{
    const int64_t n_words = (n_rows + 31) / 32;
    return (n_words + WORDS_PER_BLOCK - 1) / WORDS_PER_BLOCK + 1;
}

hipError_t launch_compact_dirty(const uint32_t *dirty, int64_t n_rows, int32_t *list, uint32_t *count,
                                uint32_t *scratch, hipStream_t s)
{
    if (!dirty || !list || !count || !scratch) return hipErrorInvalidValue;
    const int64_t n_words = (n_rows + 31) / 32;
    const int64_t nb = (n_words + WORDS_PER_BLOCK - 1) / WORDS_PER_BLOCK;
    if (nb <= 0 || nb > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(dirty_count_kernel, dim3((unsigned)nb), dim3(BLOCK), 0, s, dirty, n_words, scratch);
    hipLaunchKernelGGL(dirty_scan_kernel, dim3(1), dim3(BLOCK), 0, s, scratch, (int32_t)nb, count);
    hipLaunchKernelGGL(dirty_write_kernel, dim3((unsigned)nb), dim3(BLOCK), 0, s, dirty, n_words, scratch, list);
    return hipGetLastError();
}

hipError_t launch_mean_rows(float *x, float *acc, float *snap, int64_t pitch, int32_t W, int32_t wt, int32_t row_len,
                            const int32_t *list, const uint32_t *count, const unsigned long long *touched,
                            unsigned long long *totals, hipStream_t s)
{
    if (W <= 0 || wt <= 0 || W % wt != 0 || row_len <= 0 || row_len % 4 != 0) return hipErrorInvalidValue;
    if (!x || !acc || !snap || !list || !count || (touched && W > 64)) return hipErrorInvalidValue;
    const dim3 grid(N_CU * LAA_ROWS_WAVES_PER_CU), block(WAVE);
#define LAA_ROWS(WT) hipLaunchKernelGGL((mean_rows_kernel<WT>), grid, block, 0, s, x, acc, snap, pitch, W, row_len, list, count, touched, totals)
    switch (wt) {               // the same batches as the dense mean: one order of the worker-axis sum everywhere
    case 8: LAA_ROWS(8); break;
    case 4: LAA_ROWS(4); break;
    case 2: LAA_ROWS(2); break;
    case 1: LAA_ROWS(1); break;
    default: return hipErrorInvalidValue;
    }
#undef LAA_ROWS
    return hipGetLastError();
}

hipError_t debug_philox(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t *dev = nullptr;
    hipError_t e = hipMalloc(&dev, 4 * sizeof(uint32_t));
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(philox_debug_kernel, dim3(1), dim3(64), 0, 0, ctr[0], ctr[1], ctr[2], ctr[3], key[0], key[1], dev);
    e = hipGetLastError();
    if (e == hipSuccess) e = hipMemcpy(out, dev, 4 * sizeof(uint32_t), hipMemcpyDeviceToHost);
    (void)hipFree(dev);
    return e;
}

}  // namespace laa
