// Dense kernels of the Local AdaAlter path (arXiv 1911.09030, Algorithm 3) for gfx950 (MI355X, CDNA4) and their
// dispatch, as templates over the vector width: included by laa_kernels.hip (16-byte path, VEC = 4) and
// laa_kernels_scalar.hip (VEC = 1 for unaligned pointers or d % 4 != 0), which are compiled side by side.
//
// The path is elementwise and HBM-bound: no MFMA, no LDS for the dense kernels.
// Layout: x, acc are [W][pitch] (worker-major, pitch >= d); one thread owns a group
// of four consecutive coordinates for ALL W workers, so
//   * every global access is a 16-byte load/store, consecutive lanes touch
//     consecutive 16-byte words (1 KiB per wavefront per instruction),
//   * the quantities shared by the workers of a column (the lazily updated
//     denominator of Section 4.2, the quadratic's a and xstar) are read and the
//     square root / division are evaluated once per column, not once per worker,
//   * the worker-axis mean of the Synchronize branch is a register reduction
//     (a balanced tree over the W values the thread already holds); no
//     cross-lane traffic is needed with this layout.
// State is streamed once per step, so loads/stores of x, acc and gradients are
// non-temporal (measured: 4 % faster than cached loads when the arrays are spread
// over the HBM address range).
#pragma once
#include "laa_kernels.h"

namespace laa {

typedef float v4f __attribute__((ext_vector_type(4)));

#ifndef LAA_BLOCK
#define LAA_BLOCK 64         // threads per block of the dense streaming kernels
#endif
#ifndef LAA_NT_LOAD
#define LAA_NT_LOAD true     // non-temporal loads of streamed state and gradients
#endif
#ifndef LAA_NT_STORE
#define LAA_NT_STORE true    // non-temporal stores of streamed state
#endif
// Dense kernels run one wavefront per thread block: with 16 to 35 independent 16-byte streams per thread the
// finest dispatch granularity measured fastest (64 > 128 > 256 > 512 threads, about 5 % end to end at d = 4e8).
static constexpr int DBLOCK = LAA_BLOCK;
static constexpr int BLOCK = 256;   // bookkeeping kernels (init, fill, sparse rows, bitmap compaction)
static constexpr bool NT_LD = LAA_NT_LOAD, NT_ST = LAA_NT_STORE;

// ------------------------------------------------------------------------------------------
// small vector pack: VEC = 4 (16-byte accesses) or VEC = 1 (fallback for unaligned / d % 4 != 0)
template <int VEC> struct Pack { float v[VEC]; };

template <int VEC, bool NT> __device__ __forceinline__ Pack<VEC> ld(const float *p)
{
    Pack<VEC> r;
    if constexpr (VEC == 4) {
        v4f t = NT ? __builtin_nontemporal_load(reinterpret_cast<const v4f *>(p)) : *reinterpret_cast<const v4f *>(p);
        r.v[0] = t.x; r.v[1] = t.y; r.v[2] = t.z; r.v[3] = t.w;
    } else {
        r.v[0] = NT ? __builtin_nontemporal_load(p) : *p;
    }
    return r;
}
template <int VEC, bool NT> __device__ __forceinline__ void st(float *p, const Pack<VEC> &r)
{
    if constexpr (VEC == 4) {
        v4f t = {r.v[0], r.v[1], r.v[2], r.v[3]};
        if (NT) __builtin_nontemporal_store(t, reinterpret_cast<v4f *>(p));
        else *reinterpret_cast<v4f *>(p) = t;
    } else {
        if (NT) __builtin_nontemporal_store(r.v[0], p);
        else *p = r.v[0];
    }
}

// The same with the address split into a part that is uniform over the wavefront (kernel arguments, block index,
// worker row: computed once on the scalar unit) and a small per-lane element offset.  The compiler then uses the
// scalar-base addressing form or, for the non-temporal accesses, forms the address with a single 64-bit add of the
// scalar base and the lane offset, instead of per-lane 64-bit multiply-adds for every stream.
template <int VEC, bool NT> __device__ __forceinline__ Pack<VEC> ld(const float *base, uint32_t lane_off)
{
    return ld<VEC, NT>(base + lane_off);
}
template <int VEC, bool NT> __device__ __forceinline__ void st(float *base, uint32_t lane_off, const Pack<VEC> &r)
{
    st<VEC, NT>(base + lane_off, r);
}

// ------------------------------------------------------------------------------------------
// Thread block -> work.  A tile is DBLOCK * VEC consecutive columns (one group per thread).
//   joint: block b owns tile b for all W workers (needed when the step also averages over the workers).
//   split: block b owns ONE worker of a tile, so a thread has two read-modify-write streams instead of 2W.
//          The W blocks of a tile re-read snap, a, xstar; they are given block ids 8 apart, which the
//          hardware's round-robin deal of consecutive block ids over the 8 XCDs puts on the same XCD close
//          in time, so those re-reads hit that XCD's L2 and HBM traffic stays at the algorithmic bytes:
//              b -> lo = b mod 8, w = (b div 8) mod W, hi = b div 8W, tile = 8 hi + lo.
template <int VEC, bool SPLIT>
__device__ __forceinline__ bool block_work(int64_t d, int32_t W, int64_t *jb, uint32_t *jl, int32_t *w_begin, int32_t *w_end)
{
    int64_t tile;
    if constexpr (SPLIT) {
        const int64_t b = blockIdx.x, n_tiles = (d / VEC + DBLOCK - 1) / DBLOCK;
        tile = (b / (8 * (int64_t)W)) * 8 + (b & 7);
        *w_begin = (int32_t)((b >> 3) % W);
        *w_end = *w_begin + 1;
        if (tile >= n_tiles) return false;
    } else {
        tile = blockIdx.x;
        *w_begin = 0;
        *w_end = W;
    }
    *jb = tile * (DBLOCK * VEC);                 // first column of the block: uniform
    *jl = threadIdx.x * VEC;                     // this thread's column group within it
    return *jb + *jl < d;
}

// ------------------------------------------------------------------------------------------
// a ^ b ^ c in one VALU operation (three-input bitwise op with truth table 0x96)
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c)
{
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

// Philox4x32-10 (Salmon et al., SC'11): per round hi0:lo0 = M0*c0, hi1:lo1 = M1*c2,
// (c0,c1,c2,c3) <- (hi1^c1^k0, lo1, hi0^c3^k1, lo0); the key advances by the Weyl constants.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                              uint32_t k1, uint32_t (&r)[4])
{
#pragma unroll
    for (int i = 0; i < 10; ++i) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = xor3((uint32_t)(p1 >> 32), c1, k0);
        const uint32_t n2 = xor3((uint32_t)(p0 >> 32), c3, k1);
        c1 = (uint32_t)p1; c3 = (uint32_t)p0; c0 = n0; c2 = n2;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    r[0] = c0; r[1] = c1; r[2] = c2; r[3] = c3;
}

// u = ((r >> 9) + 0.5) * 2^-23: 23 random bits, never 0 or 1, exact in fp32.  Two operations: the funnel shift
// (0x7F : r) >> 9 is the bit pattern of 1 + (r >> 9) 2^-23 in [1, 2), and subtracting 1 - 2^-24 from it is exact.
__device__ __forceinline__ float u01(uint32_t r)
{
    return __uint_as_float(__builtin_amdgcn_alignbit(0x7Fu, r, 9u)) - 0x1.fffffep-1f;
}

// Four normals for the coordinates 4*qa .. 4*qa+3 of worker w at iteration word t on a stream, scaled by sigma and
// left in factored form: normal e is rad[e / 2] * trig[e] (Box-Muller on (u0,u1) and (u2,u3): radius times cosine,
// radius times sine), so that the caller can put the product into a multiply-add.  c = -2 ln2 sigma^2:
// sigma sqrt(-2 ln u0) = sqrt(c log2 u0) for sigma >= 0, which saves the multiplication by sigma.
struct Normals4 { float rad[2], trig[4]; };

static constexpr float UNIT_NORMAL_C = -1.3862943611198906f;         // -2 ln 2

__device__ __forceinline__ Normals4 normals4(uint32_t seed_lo, uint32_t seed_hi, uint32_t stream, uint64_t qa, uint32_t w,
                                             uint32_t t, float c)
{
    uint32_t r[4];
    philox4x32_10((uint32_t)qa, w, t, stream + (uint32_t)(qa >> 32) * 16u, seed_lo, seed_hi, r);
    Normals4 n;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const float u0 = u01(r[2 * p]), u1 = u01(r[2 * p + 1]);
        // u0 >= 2^-24 is a normal number, so the bare hardware log2 / sqrt apply (relative error 1.4e-7 over all 2^23
        // inputs); the hardware sine and cosine take their argument in turns, which is u1 itself (absolute error
        // 1.3e-7 over all 2^23 inputs).
        n.rad[p] = __builtin_amdgcn_sqrtf(__builtin_amdgcn_logf(u0) * c);
        n.trig[2 * p] = __builtin_amdgcn_cosf(u1);
        n.trig[2 * p + 1] = __builtin_amdgcn_sinf(u1);
    }
    return n;
}

static constexpr uint32_t STREAM_OFFSET = 2, STREAM_NOISE = 3;

// Gradient of worker w for the VEC coordinates starting at j = jb + jl, evaluated at xv (the worker's x before the
// step); rowb = w * pitch + jb is the uniform part of the element's index in the [W][pitch] arrays.
//   quadratic: g = a (x - (xstar + off)) + noise_scale n        noise: g = a n
// evaluated as a ((x - xstar) - off) + noise_scale n with the scales folded into the normals' radii.
// TDEV: the iteration number is t_lo plus a device word (periods replayed from a graph).
template <int VEC, int GS, int OS, bool TDEV = false>
__device__ __forceinline__ Pack<VEC> gradient(const StepArgs &a, int64_t jb, uint32_t jl, int64_t rowb, int32_t w,
                                              const Pack<VEC> &xv, const Pack<VEC> &av, const Pack<VEC> &xs)
{
    Pack<VEC> g;
    if constexpr (GS == GRAD_EXPLICIT) {
        g = ld<VEC, NT_LD>(a.grads + rowb, jl);
    } else {
        const uint64_t ja = (uint64_t)(jb + jl + a.col0);    // col0 % 4 == 0: ja & 3 is the lane within the Philox block
        const uint64_t qa = ja >> 2;
        const uint32_t wg = (uint32_t)(w + a.w0);
        uint32_t t = a.t_lo;
        if constexpr (TDEV) t += *a.t_dev;                       // uniform: one scalar load
        const Normals4 n = normals4(a.seed_lo, a.seed_hi, STREAM_NOISE, qa, wg, t, GS == GRAD_NOISE ? UNIT_NORMAL_C : a.noise_c);
        const int lane0 = VEC == 4 ? 0 : (int)(ja & 3);
        if constexpr (GS == GRAD_NOISE) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) g.v[e] = av.v[e] * (n.rad[(lane0 + e) >> 1] * n.trig[lane0 + e]);
        } else {
            Pack<VEC> diff;                                      // x - xstar - off
#pragma unroll
            for (int e = 0; e < VEC; ++e) diff.v[e] = xv.v[e] - xs.v[e];
            if constexpr (OS == OFFSET_ARRAY) {
                const Pack<VEC> o = ld<VEC, NT_LD>(a.off + rowb, jl);
#pragma unroll
                for (int e = 0; e < VEC; ++e) diff.v[e] = diff.v[e] - o.v[e];
            } else if constexpr (OS == OFFSET_PHILOX) {
                const Normals4 m = normals4(a.seed_lo, a.seed_hi, STREAM_OFFSET, qa, wg, 0u, a.off_c);
#pragma unroll
                for (int e = 0; e < VEC; ++e) diff.v[e] = fmaf(-m.rad[(lane0 + e) >> 1], m.trig[lane0 + e], diff.v[e]);
            }
#pragma unroll
            for (int e = 0; e < VEC; ++e)
                g.v[e] = fmaf(av.v[e], diff.v[e], n.rad[(lane0 + e) >> 1] * n.trig[lane0 + e]);
        }
    }
    return g;
}

// sum / W.  For W a power of two the product with 1/W is the same correctly rounded value as the quotient (scaling by a
// power of two is exact, and rounds identically when the result is subnormal), so the IEEE division's ten or so
// instructions per element are spent only for the other W.  The choice is uniform over the grid.
struct MeanOf {
    float w, inv;
    bool pow2;
    __device__ __forceinline__ explicit MeanOf(int32_t W) : w((float)W), inv(1.0f / (float)W), pow2((W & (W - 1)) == 0) {}
    __device__ __forceinline__ float operator()(float sum) const { return pow2 ? sum * inv : sum / w; }
};

// balanced tree over the WT packs of one batch; batches are added in ascending order
template <int VEC, int WT> __device__ __forceinline__ Pack<VEC> tree_sum(const Pack<VEC> (&v)[WT])
{
    Pack<VEC> r;
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        if constexpr (WT == 1) r.v[e] = v[0].v[e];
        else if constexpr (WT == 2) r.v[e] = v[0].v[e] + v[1].v[e];
        else if constexpr (WT == 4) r.v[e] = (v[0].v[e] + v[1].v[e]) + (v[2].v[e] + v[3].v[e]);
        else r.v[e] = ((v[0].v[e] + v[1].v[e]) + (v[2].v[e] + v[3].v[e])) +
                      ((v[4].v[e] + v[5].v[e]) + (v[6].v[e] + v[7].v[e]));
    }
    return r;
}

// ------------------------------------------------------------------------------------------
// One iteration of Algorithm 3 for every worker of a column group.
//   den   = sqrt(B2_sync + t' eps^2)   (value of the accumulator at the last sync, shared by all workers)
//   y     = x - eta g / den ;  A2 = B2 + g o g
//   SYNC: x, B2 <- mean over workers of y, A2; B2_sync <- that mean      (Synchronize branch)
//   GRAD_ONLY: write g and change nothing (used to materialise gradients)
// Right after a Synchronize every worker holds the same x and B2 = B2_sync.  With lazy replicas that common
// state is kept once (x in row 0, B2 in snap):
//   CIN : the state is collapsed on entry: read x from row 0 and B2 from snap for every worker
//   COUT: (with SYNC) leave it collapsed: write the means to row 0 of x and to snap only
template <int VEC, int WT, int GS, int OS, bool SYNC, bool GRAD_ONLY, bool CIN, bool COUT, bool TDEV>
__device__ __forceinline__ void step_body(const StepArgs &a, const int64_t jb, const uint32_t jl, const int32_t w_begin,
                                          const int32_t w_end)
{
    // column j = jb + jl: jb is uniform over the block, jl the lane's offset (addresses = scalar base + lane offset)
    Pack<VEC> av, xs, step, sn, x0;
    if constexpr (GS != GRAD_EXPLICIT) av = ld<VEC, false>(a.a + jb, jl);
    if constexpr (GS == GRAD_QUADRATIC) xs = ld<VEC, false>(a.xstar + jb, jl);
    if constexpr (!GRAD_ONLY) {
        sn = ld<VEC, false>(a.snap + jb, jl);
#pragma unroll
        for (int e = 0; e < VEC; ++e) step.v[e] = a.eta / sqrtf(sn.v[e] + a.pad);
    }
    if constexpr (CIN) x0 = ld<VEC, false>(a.x + jb, jl);

    Pack<VEC> sx, sb;
#pragma unroll
    for (int e = 0; e < VEC; ++e) sx.v[e] = sb.v[e] = 0.0f;

    for (int32_t w0 = w_begin; w0 < w_end; w0 += WT) {
        Pack<VEC> xv[WT], bv[WT];
#pragma unroll
        for (int i = 0; i < WT; ++i) {
            const int64_t rowb = (int64_t)(w0 + i) * a.pitch + jb;
            if constexpr (CIN) {
                xv[i] = x0;
                if constexpr (!GRAD_ONLY) bv[i] = sn;
            } else {
                if constexpr (GS == GRAD_QUADRATIC || !GRAD_ONLY) xv[i] = ld<VEC, NT_LD>(a.x + rowb, jl);
                if constexpr (!GRAD_ONLY) bv[i] = ld<VEC, NT_LD>(a.acc + rowb, jl);
            }
        }
#pragma unroll
        for (int i = 0; i < WT; ++i) {
            const int64_t rowb = (int64_t)(w0 + i) * a.pitch + jb;
            const Pack<VEC> g = gradient<VEC, GS, OS, TDEV>(a, jb, jl, rowb, w0 + i, xv[i], av, xs);
            if constexpr (GRAD_ONLY) {
                st<VEC, NT_ST>(a.grad_out + rowb, jl, g);
            } else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    xv[i].v[e] = fmaf(-g.v[e], step.v[e], xv[i].v[e]);
                    bv[i].v[e] = fmaf(g.v[e], g.v[e], bv[i].v[e]);
                }
                if constexpr (!SYNC) {
                    st<VEC, NT_ST>(a.x + rowb, jl, xv[i]);
                    st<VEC, NT_ST>(a.acc + rowb, jl, bv[i]);
                }
            }
        }
        if constexpr (SYNC && !GRAD_ONLY) {
            const Pack<VEC> tx = tree_sum<VEC, WT>(xv), tb = tree_sum<VEC, WT>(bv);
#pragma unroll
            for (int e = 0; e < VEC; ++e) { sx.v[e] += tx.v[e]; sb.v[e] += tb.v[e]; }
        }
    }
    if constexpr (SYNC && !GRAD_ONLY) {
        const MeanOf mean(a.W);
#pragma unroll
        for (int e = 0; e < VEC; ++e) { sx.v[e] = mean(sx.v[e]); sb.v[e] = mean(sb.v[e]); }
        if constexpr (COUT) {
            st<VEC, false>(a.x + jb, jl, sx);
        } else {
            for (int32_t w = 0; w < a.W; ++w) {
                const int64_t rowb = (int64_t)w * a.pitch + jb;
                st<VEC, NT_ST>(a.x + rowb, jl, sx);
                st<VEC, NT_ST>(a.acc + rowb, jl, sb);
            }
        }
        st<VEC, false>(a.snap + jb, jl, sb);
    }
}

// Most wavefronts per SIMD for the steps that stream all 2W rows in and out (no averaging, state not collapsed): they
// need 122 (generated gradient) and 108 (explicit gradient) vector registers, which would allow 4, but fewer
// wavefronts with the same loads in flight run faster on a saturated memory system.  Measured at d = 4e8 / 1e8, W = 8,
// same process sequence: generated gradient 8.69 ms with 3, 8.75 with 4, 8.76 with 2; explicit gradient 2.56 ms
// with 2, 2.59 with 4, 2.60 with 3.
#ifndef LAA_PLAIN_WAVES
#define LAA_PLAIN_WAVES 3
#endif
#ifndef LAA_EXPLICIT_WAVES
#define LAA_EXPLICIT_WAVES 2
#endif
// The steps around an averaging (fewer bytes, bound by the generator's arithmetic as much as by memory) showed no
// consistent preference between 2 and 5 wavefronts per SIMD and are left to the register count.
static constexpr int step_waves(int gs, bool sync, bool grad_only, bool cin)
{
    return (sync || grad_only || cin) ? 8 : gs == GRAD_EXPLICIT ? LAA_EXPLICIT_WAVES : LAA_PLAIN_WAVES;
}

template <int VEC, int WT, int GS, int OS, bool SYNC, bool GRAD_ONLY, bool SPLIT, bool CIN, bool COUT, bool TDEV = false>
__global__ __launch_bounds__(DBLOCK)
__attribute__((amdgpu_waves_per_eu(1, step_waves(GS, SYNC, GRAD_ONLY, CIN))))
void step_kernel(const StepArgs a)
{
    static_assert(!SPLIT || (WT == 1 && !SYNC), "a split block owns one worker and cannot average");
    static_assert(!COUT || SYNC, "only a step that averages can leave the state collapsed");
    int64_t jb;
    uint32_t jl;
    int32_t w_begin, w_end;
    if (block_work<VEC, SPLIT>(a.d, a.W, &jb, &jl, &w_begin, &w_end))
        step_body<VEC, WT, GS, OS, SYNC, GRAD_ONLY, CIN, COUT, TDEV>(a, jb, jl, w_begin, w_end);
}

// Algorithm 1 (Distributed AdaGrad): G = mean_i G_i; B2 += G o G; x -= eta G / sqrt(B2 + eps^2), one
// shared iterate kept in every worker's row.  Algorithm 2 (Local SGD): y = x - eta G per worker.
// ROW0 (Algorithm 1 with lazy replicas): the one iterate is read from and written to row 0 of x only, B2 to snap only.
template <int VEC, int WT, int GS, int OS, int ALGO, bool SYNC, bool ROW0>
__device__ __forceinline__ void baseline_body(const StepArgs &a, const int64_t jb, const uint32_t jl)
{
    static_assert(!ROW0 || ALGO == ALGO_DIST_ADAGRAD, "only Algorithm 1 has a single iterate");
    Pack<VEC> av, xs;
    if constexpr (GS != GRAD_EXPLICIT) av = ld<VEC, false>(a.a + jb, jl);
    if constexpr (GS == GRAD_QUADRATIC) xs = ld<VEC, false>(a.xstar + jb, jl);
    Pack<VEC> sg, sx;
#pragma unroll
    for (int e = 0; e < VEC; ++e) sg.v[e] = sx.v[e] = 0.0f;
    Pack<VEC> x0;
    for (int32_t w0 = 0; w0 < a.W; w0 += WT) {
        Pack<VEC> xv[WT], gv[WT];
#pragma unroll
        for (int i = 0; i < WT; ++i) {
            if constexpr (ROW0) xv[i] = (w0 == 0 && i == 0) ? ld<VEC, false>(a.x + jb, jl) : x0;
            else xv[i] = ld<VEC, NT_LD>(a.x + ((int64_t)(w0 + i) * a.pitch + jb), jl);
            if (w0 == 0 && i == 0) x0 = xv[0];
        }
#pragma unroll
        for (int i = 0; i < WT; ++i) {
            const int64_t rowb = (int64_t)(w0 + i) * a.pitch + jb;
            gv[i] = gradient<VEC, GS, OS>(a, jb, jl, rowb, w0 + i, xv[i], av, xs);
            if constexpr (ALGO == ALGO_LOCAL_SGD) {
#pragma unroll
                for (int e = 0; e < VEC; ++e) xv[i].v[e] = fmaf(-a.eta, gv[i].v[e], xv[i].v[e]);
                if constexpr (!SYNC) st<VEC, NT_ST>(a.x + rowb, jl, xv[i]);
            }
        }
        if constexpr (ALGO == ALGO_DIST_ADAGRAD) {
            const Pack<VEC> t = tree_sum<VEC, WT>(gv);
#pragma unroll
            for (int e = 0; e < VEC; ++e) sg.v[e] += t.v[e];
        } else if constexpr (SYNC) {
            const Pack<VEC> t = tree_sum<VEC, WT>(xv);
#pragma unroll
            for (int e = 0; e < VEC; ++e) sx.v[e] += t.v[e];
        }
    }
    const MeanOf mean(a.W);
    if constexpr (ALGO == ALGO_DIST_ADAGRAD) {
        Pack<VEC> b2 = ld<VEC, false>(a.snap + jb, jl);
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const float g = mean(sg.v[e]);
            b2.v[e] = fmaf(g, g, b2.v[e]);
            x0.v[e] = x0.v[e] - (a.eta * g) / sqrtf(b2.v[e] + a.eps2);
        }
        if constexpr (ROW0) {
            st<VEC, false>(a.x + jb, jl, x0);
        } else {
            for (int32_t w = 0; w < a.W; ++w) {
                st<VEC, NT_ST>(a.x + ((int64_t)w * a.pitch + jb), jl, x0);
                st<VEC, NT_ST>(a.acc + ((int64_t)w * a.pitch + jb), jl, b2);
            }
        }
        st<VEC, false>(a.snap + jb, jl, b2);
    } else if constexpr (SYNC) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) sx.v[e] = mean(sx.v[e]);
        for (int32_t w = 0; w < a.W; ++w) st<VEC, NT_ST>(a.x + ((int64_t)w * a.pitch + jb), jl, sx);
    }
}

// Wavefronts per SIMD of the two comparison algorithms, measured at d = 4e8, W = 8 with the generated gradient: Local SGD
// 4.53 ms with 2, 4.75 with 3, 4.84 with 4, 5.08 uncapped (7); Distributed AdaGrad on W replicas 6.83 with 2, 6.86 with 3,
// 6.87 uncapped. The single-iterate AdaGrad step is bound by the generator's arithmetic and wants every wavefront it
// can get (3.09-3.12 ms uncapped, 3.24 with 2).
#ifndef LAA_BASELINE_WAVES
#define LAA_BASELINE_WAVES 2
#endif
static constexpr int baseline_waves(bool row0) { return row0 ? 8 : LAA_BASELINE_WAVES; }

template <int VEC, int WT, int GS, int OS, int ALGO, bool SYNC, bool ROW0 = false>
__global__ __launch_bounds__(DBLOCK) __attribute__((amdgpu_waves_per_eu(1, baseline_waves(ROW0))))
void baseline_kernel(const StepArgs a)
{
    int64_t jb;
    uint32_t jl;
    int32_t w_begin, w_end;
    if (block_work<VEC, false>(a.d, a.W, &jb, &jl, &w_begin, &w_end)) baseline_body<VEC, WT, GS, OS, ALGO, SYNC, ROW0>(a, jb, jl);
}

// Synchronize branch on its own: x[w], acc[w] <- mean over w; snap <- mean acc.
template <int VEC, int WT, bool X_ONLY, bool COUT>
__device__ __forceinline__ void mean_body(float *__restrict__ x, float *__restrict__ acc, float *__restrict__ snap,
                                          int64_t pitch, int32_t W, const int64_t jb, const uint32_t jl)
{
    Pack<VEC> sx, sb;
#pragma unroll
    for (int e = 0; e < VEC; ++e) sx.v[e] = sb.v[e] = 0.0f;
    for (int32_t w0 = 0; w0 < W; w0 += WT) {
        Pack<VEC> xv[WT], bv[WT];
#pragma unroll
        for (int i = 0; i < WT; ++i) {
            xv[i] = ld<VEC, NT_LD>(x + ((int64_t)(w0 + i) * pitch + jb), jl);
            if constexpr (!X_ONLY) bv[i] = ld<VEC, NT_LD>(acc + ((int64_t)(w0 + i) * pitch + jb), jl);
        }
        const Pack<VEC> tx = tree_sum<VEC, WT>(xv);
#pragma unroll
        for (int e = 0; e < VEC; ++e) sx.v[e] += tx.v[e];
        if constexpr (!X_ONLY) {
            const Pack<VEC> tb = tree_sum<VEC, WT>(bv);
#pragma unroll
            for (int e = 0; e < VEC; ++e) sb.v[e] += tb.v[e];
        }
    }
    const MeanOf mean(W);
#pragma unroll
    for (int e = 0; e < VEC; ++e) { sx.v[e] = mean(sx.v[e]); sb.v[e] = mean(sb.v[e]); }
    if constexpr (COUT) {
        st<VEC, false>(x + jb, jl, sx);
    } else {
        for (int32_t w = 0; w < W; ++w) {
            st<VEC, NT_ST>(x + ((int64_t)w * pitch + jb), jl, sx);
            if constexpr (!X_ONLY) st<VEC, NT_ST>(acc + ((int64_t)w * pitch + jb), jl, sb);
        }
    }
    if constexpr (!X_ONLY) st<VEC, false>(snap + jb, jl, sb);
}

// At most 2 wavefronts per SIMD for the averaging kernels too (2W loads in flight per lane): the whole-table mean of a
// 409.6M-column table ran in 8.38 ms with 2, 8.48 with 3, 8.58 with 4, 8.45-8.54 uncapped (7).
#ifndef LAA_MEAN_WAVES
#define LAA_MEAN_WAVES 2
#endif
template <int VEC, int WT, bool X_ONLY, bool COUT>
__global__ __launch_bounds__(DBLOCK) __attribute__((amdgpu_waves_per_eu(1, LAA_MEAN_WAVES))) void mean_kernel(float *__restrict__ x, float *__restrict__ acc,
                                                     float *__restrict__ snap, int64_t d, int64_t pitch, int32_t W)
{
    int64_t jb;
    uint32_t jl;
    int32_t w_begin, w_end;
    if (block_work<VEC, false>(d, W, &jb, &jl, &w_begin, &w_end))
        mean_body<VEC, WT, X_ONLY, COUT>(x, acc, snap, pitch, W, jb, jl);
}

// ------------------------------------------------------------------------------------------
// launchers
// rows of x, acc (and explicit gradients, stored offsets) are pitch >= d elements apart
static inline bool layout_ok(int64_t d, int64_t pitch, bool vec4)
{
    return pitch >= d && (!vec4 || pitch % 4 == 0);
}

// grid of the dense kernels for n_groups thread-items (one per VEC columns); split: one block per (tile, worker)
static inline bool dense_grid(int64_t n_groups, bool split, int32_t W, dim3 *grid)
{
    if (n_groups <= 0) return false;
    const int64_t n_tiles = (n_groups + DBLOCK - 1) / DBLOCK;
    const int64_t nb = split ? (n_tiles + 7) / 8 * 8 * (int64_t)W : n_tiles;
    if (nb > 0x7fffffffLL) return false;
    *grid = dim3((unsigned)nb);
    return true;
}

static inline bool grid_for(int64_t n_threads, dim3 *grid)
{
    const int64_t nb = (n_threads + BLOCK - 1) / BLOCK;
    if (nb <= 0 || nb > 0x7fffffffLL) return false;
    *grid = dim3((unsigned)nb);
    return true;
}

template <int VEC, int WT, int GS, int OS>
static inline hipError_t launch_step_4(const StepArgs &a, dim3 grid, hipStream_t s)
{
#define LAA_STEP(SYNC, GONLY, SPLIT, CIN, COUT) \
    hipLaunchKernelGGL((step_kernel<VEC, WT, GS, OS, SYNC, GONLY, SPLIT, CIN, COUT>), grid, dim3(DBLOCK), 0, s, a)
#define LAA_STEP_T(SYNC, CIN, COUT) \
    hipLaunchKernelGGL((step_kernel<VEC, WT, GS, OS, SYNC, false, false, CIN, COUT, true>), grid, dim3(DBLOCK), 0, s, a)
    if (a.t_dev) {              // a step of a replayed period: vector path, generator, Local AdaAlter, all workers per block
        if constexpr (VEC == 4 && GS != GRAD_EXPLICIT) {
            if (a.grad_out || a.split || a.algo != ALGO_LOCAL_ADAALTER) return hipErrorInvalidValue;
            if (a.sync) {
                if (a.collapsed_in && a.collapsed_out) LAA_STEP_T(true, true, true);
                else if (a.collapsed_in) LAA_STEP_T(true, true, false);
                else if (a.collapsed_out) LAA_STEP_T(true, false, true);
                else LAA_STEP_T(true, false, false);
            } else if (a.collapsed_in) {
                LAA_STEP_T(false, true, false);
            } else {
                LAA_STEP_T(false, false, false);
            }
            return hipGetLastError();
        } else {
            return hipErrorInvalidValue;
        }
    }
#undef LAA_STEP_T
    if (a.grad_out) {
        if constexpr (GS == GRAD_EXPLICIT) return hipErrorInvalidValue;
        else if (a.collapsed_in) LAA_STEP(false, true, false, true, false);
        else LAA_STEP(false, true, false, false, false);
    } else if (a.algo == ALGO_LOCAL_ADAALTER) {
        if (a.sync) {
            if (a.collapsed_in && a.collapsed_out) LAA_STEP(true, false, false, true, true);
            else if (a.collapsed_in) LAA_STEP(true, false, false, true, false);
            else if (a.collapsed_out) LAA_STEP(true, false, false, false, true);
            else LAA_STEP(true, false, false, false, false);
        } else if (a.collapsed_in) {
            LAA_STEP(false, false, false, true, false);
        } else if (a.split) {
            if constexpr (WT == 1) LAA_STEP(false, false, true, false, false);
            else return hipErrorInvalidValue;
        } else {
            LAA_STEP(false, false, false, false, false);
        }
    } else if (a.algo == ALGO_DIST_ADAGRAD) {
        if (a.collapsed_out)
            hipLaunchKernelGGL((baseline_kernel<VEC, WT, GS, OS, ALGO_DIST_ADAGRAD, true, true>), grid, dim3(DBLOCK), 0, s, a);
        else
            hipLaunchKernelGGL((baseline_kernel<VEC, WT, GS, OS, ALGO_DIST_ADAGRAD, true>), grid, dim3(DBLOCK), 0, s, a);
    } else {
        if (a.sync)
            hipLaunchKernelGGL((baseline_kernel<VEC, WT, GS, OS, ALGO_LOCAL_SGD, true>), grid, dim3(DBLOCK), 0, s, a);
        else
            hipLaunchKernelGGL((baseline_kernel<VEC, WT, GS, OS, ALGO_LOCAL_SGD, false>), grid, dim3(DBLOCK), 0, s, a);
    }
#undef LAA_STEP
    return hipGetLastError();
}

template <int VEC, int WT> static inline hipError_t launch_step_2(const StepArgs &a, dim3 grid, hipStream_t s)
{
    switch (a.grad_source) {
    case GRAD_EXPLICIT: return launch_step_4<VEC, WT, GRAD_EXPLICIT, OFFSET_NONE>(a, grid, s);
    case GRAD_NOISE: return launch_step_4<VEC, WT, GRAD_NOISE, OFFSET_NONE>(a, grid, s);
    case GRAD_QUADRATIC:
        switch (a.off_source) {
        case OFFSET_NONE: return launch_step_4<VEC, WT, GRAD_QUADRATIC, OFFSET_NONE>(a, grid, s);
        case OFFSET_ARRAY: return launch_step_4<VEC, WT, GRAD_QUADRATIC, OFFSET_ARRAY>(a, grid, s);
        case OFFSET_PHILOX: return launch_step_4<VEC, WT, GRAD_QUADRATIC, OFFSET_PHILOX>(a, grid, s);
        }
    }
    return hipErrorInvalidValue;
}

template <int VEC, int WT>
static inline hipError_t launch_mean_2(float *x, float *acc, float *snap, int64_t d, int64_t pitch, int32_t W, bool x_only,
                                bool collapse, dim3 grid, hipStream_t s)
{
    if (x_only) hipLaunchKernelGGL((mean_kernel<VEC, WT, true, false>), grid, dim3(DBLOCK), 0, s, x, acc, snap, d, pitch, W);
    else if (collapse) hipLaunchKernelGGL((mean_kernel<VEC, WT, false, true>), grid, dim3(DBLOCK), 0, s, x, acc, snap, d, pitch, W);
    else hipLaunchKernelGGL((mean_kernel<VEC, WT, false, false>), grid, dim3(DBLOCK), 0, s, x, acc, snap, d, pitch, W);
    return hipGetLastError();
}

// The worker batch (1, 2, 4 or 8 workers loaded together) is a template argument: one switch per vector width.
template <int VEC> static inline hipError_t launch_step_wt(const StepArgs &a, dim3 grid, hipStream_t s)
{
    switch (a.wt) {
    case 1: return launch_step_2<VEC, 1>(a, grid, s);
    case 2: return launch_step_2<VEC, 2>(a, grid, s);
    case 4: return launch_step_2<VEC, 4>(a, grid, s);
    case 8: return launch_step_2<VEC, 8>(a, grid, s);
    }
    return hipErrorInvalidValue;
}

template <int VEC>
static inline hipError_t launch_mean_wt(float *x, float *acc, float *snap, int64_t d, int64_t pitch, int32_t W, int32_t wt,
                                        bool x_only, bool collapse, dim3 grid, hipStream_t s)
{
    switch (wt) {
    case 1: return launch_mean_2<VEC, 1>(x, acc, snap, d, pitch, W, x_only, collapse, grid, s);
    case 2: return launch_mean_2<VEC, 2>(x, acc, snap, d, pitch, W, x_only, collapse, grid, s);
    case 4: return launch_mean_2<VEC, 4>(x, acc, snap, d, pitch, W, x_only, collapse, grid, s);
    case 8: return launch_mean_2<VEC, 8>(x, acc, snap, d, pitch, W, x_only, collapse, grid, s);
    }
    return hipErrorInvalidValue;
}

// defined in laa_kernels_scalar.hip
hipError_t launch_step_scalar(const StepArgs &a, dim3 grid, hipStream_t s);
hipError_t launch_mean_scalar(float *x, float *acc, float *snap, int64_t d, int64_t pitch, int32_t W, int32_t wt,
                              bool x_only, bool collapse, dim3 grid, hipStream_t s);

}  // namespace laa
