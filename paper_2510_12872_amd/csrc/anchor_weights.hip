// kvcomm_anchor_weights: anchor matching.  l2 distance between the segment's base keys and
// each selected anchor's base keys, then the softmax of the negative distance across the
// anchor dimension (Eq. "pred", Eq. "ph_update" and the weight step of Algorithm 1; the
// appendix on long-context anchor matching gives the reduced shape [m,1,1,seq_len,1]).
//
// Two deterministic stages, no floating-point atomics:
//   1. dist_partial_kernel streams the key rows once (HBM-bound: (A+1) rows per
//      (layer, head, token)) and leaves, per block, the squared distance of its chunk of
//      (layer, head) pairs: partial[chunk][token][anchor] in double.
//   2. finalize_kernel adds the chunks in a fixed order, takes the square root and the
//      softmax in double, and writes fp32 weights, the nearest anchor and the selection.
// Squared differences are accumulated in double so that fp32 inputs keep ~1e-7 relative
// accuracy in the weights and the arg-min is decided in the precision the definition uses.
//
// kvcomm_anchor_weights_rule adds the two weighting variants of the appendix on the
// approximation method: "nearest" (same distances, one-hot at the arg-min) and "cosine"
// (cos_partial_kernel leaves <x,y>, |x|^2 and |y|^2 per chunk; the softmax runs over the
// similarities).  Both reuse the two-stage structure and the finalize kernels.
#include <math.h>

#include <mutex>

#include "kvcomm_device.h"

// Partial sums of kvcomm_anchor_weights_static: one array per GPU that has loaded the library, kept
// until the process ends.  In host code this name is only a handle for hipGetSymbolAddress; the
// kernels receive the address that call returns.
static __device__ __align__(256) unsigned char scratch[KVCOMM_STATIC_SCRATCH_BYTES];

namespace {

using namespace kvc;

#ifndef KVC_DIST_BLOCKS
#define KVC_DIST_BLOCKS 2048  // blocks the distance grid aims at (measured best on MI355X among 1024 ... 8192)
#endif

constexpr int kBlock = 256;
constexpr int kAnchorTile = 16;  // anchors whose accumulators one lane keeps in registers

// How a launch is cut into blocks.  Rows of one (layer, head) are LPR lanes wide; a block owns RPB
// consecutive tokens and a run of lh_per_block (layer, head) pairs ("chunk").
struct DistPlan {
    int lpr;            // lanes per row = D / EPV
    int rpb;            // rows (tokens) per block
    int lh_per_block;
    int n_chunks;
};

// seg_lens: the segments of the launch (one for the single-segment entry points).
DistPlan make_plan(const kvcomm_model *m, const int32_t *seg_lens, int n_jobs, int gran)
{
    DistPlan pl;
    const int epv = 16 / elem_size(m->dtype);
    pl.lpr = m->head_dim / epv;
    pl.rpb = kBlock / pl.lpr;
    const int LH = m->n_layers * m->n_kv_heads;
    if (gran == KVCOMM_W_LAYER_HEAD_TOKEN) {
        pl.lh_per_block = 1;
    } else {
        int64_t tiles = 0;
        for (int j = 0; j < n_jobs; ++j) tiles += (seg_lens[j] + pl.rpb - 1) / pl.rpb;
        const int64_t target_blocks = (int64_t)KVC_DIST_BLOCKS * n_jobs;
        int64_t n_chunks = (target_blocks + tiles - 1) / tiles;
        if (n_chunks > LH) n_chunks = LH;
        if (n_chunks < 1) n_chunks = 1;
        pl.lh_per_block = (int)((LH + n_chunks - 1) / n_chunks);
    }
    pl.n_chunks = (LH + pl.lh_per_block - 1) / pl.lh_per_block;
    return pl;
}

struct DistJob {
    const void *seg_k;
    Strides s_seg;
    double *partial;       // [component][n_chunks][S][n_sel]
    int64_t comp_stride;   // elements between components (cosine rule)
    int32_t S, n_token_tiles, block0;
    int16_t a0, n_sel;     // its selected anchors: entries [a0, a0 + n_sel) of anc
    // outputs of the fused form (per-(layer, head, token) weights straight from the distance kernel)
    float *weights;
    int32_t *nearest;
    int32_t *selected_out;
    uint64_t sel_mask;     // bit a = anchor a is selected
    int32_t n_anchors;
};

struct DistParams {
    DistJob job[KVCOMM_MAX_BATCH];
    Strides s_anc;
    int32_t H, LH, lh_per_block, n_jobs;
    int32_t fused, rule;   // fused: a row's distances are complete inside its lanes; write the weights here
    int32_t per_segment;   // one weight set per segment: a block also adds up its rows (partial[chunk][tile][anchor])
    double tau;
    const void *anc[KVCOMM_MAX_ANCHORS];  // selected anchors of all segments
    uint8_t col[KVCOMM_MAX_ANCHORS];      // original index of a selected anchor
};
static_assert(sizeof(DistParams) <= 4096, "kernel arguments are limited to 4 KB");

__device__ __forceinline__ int job_of_block(const DistParams &p)
{
    int ji = 0;
#pragma unroll
    for (int i = 1; i < KVCOMM_MAX_BATCH; ++i)
        if (i < p.n_jobs && (int)blockIdx.x >= p.job[i].block0) ji = i;
    return ji;
}

// Sum of squared differences of two 16-byte vectors, added to a double accumulator.
template <typename T>
__device__ __forceinline__ void sqdiff_acc(double &acc, const float (&x)[Elem<T>::EPV], const u32x4 raw)
{
    float y[Elem<T>::EPV];
    unpack<T>(raw, y);
#pragma unroll
    for (int e = 0; e < Elem<T>::EPV; ++e) {
        const double d = (double)x[e] - (double)y[e];
        acc = fma(d, d, acc);
    }
}

template <typename T, int LPR>
__global__ __launch_bounds__(kBlock) void dist_partial_kernel(const DistParams p)
{
    constexpr int EPV = Elem<T>::EPV;
    constexpr int RPB = kBlock / LPR;
    const DistJob &jb = p.job[job_of_block(p)];
    const int tid = threadIdx.x;
    const int row = tid / LPR, lir = tid % LPR;
    const int bx = blockIdx.x - jb.block0;
    const int tile = bx % jb.n_token_tiles;
    const int chunk = bx / jb.n_token_tiles;
    const int a0 = blockIdx.y * kAnchorTile;
    const int na = min(kAnchorTile, jb.n_sel - a0);
    if (na <= 0) return;  // the grid's anchor tiles cover the largest pool of the launch
    const int t = tile * RPB + row;
    const bool valid = t < jb.S;
    const int lh0 = chunk * p.lh_per_block;
    const int lh1 = min(lh0 + p.lh_per_block, p.LH);

    double acc[kAnchorTile];
#pragma unroll
    for (int j = 0; j < kAnchorTile; ++j) acc[j] = 0.0;

    if (valid) {
        const T *seg = static_cast<const T *>(jb.seg_k);
        for (int lh = lh0; lh < lh1; ++lh) {
            const int l = lh / p.H, h = lh % p.H;
            const u32x4 rs = load16_stream(seg + l * jb.s_seg.layer + h * jb.s_seg.head + t * jb.s_seg.token + lir * EPV);
            const int64_t aoff = l * p.s_anc.layer + h * p.s_anc.head + t * p.s_anc.token + lir * EPV;
            u32x4 ra[kAnchorTile];
#pragma unroll
            for (int j = 0; j < kAnchorTile; ++j)
                if (j < na) ra[j] = load16_stream(static_cast<const T *>(p.anc[jb.a0 + a0 + j]) + aoff);
            float x[EPV];
            unpack<T>(rs, x);
#pragma unroll
            for (int j = 0; j < kAnchorTile; ++j)
                if (j < na) sqdiff_acc<T>(acc[j], x, ra[j]);
        }
    }
    // Fixed-shape butterfly over the LPR lanes of a row (all inside one wavefront).
    __shared__ double rows[RPB][kAnchorTile];
#pragma unroll
    for (int j = 0; j < kAnchorTile; ++j) {
        if (j < na) {
            double v = acc[j];
#pragma unroll
            for (int off = LPR / 2; off >= 1; off >>= 1) v += __shfl_xor(v, off, LPR);
            if (p.per_segment) {
                if (lir == 0) rows[row][j] = valid ? v : 0.0;
            } else if (valid && lir == 0) {
                jb.partial[((int64_t)chunk * jb.S + t) * jb.n_sel + a0 + j] = v;
            }
        }
    }
    if (p.per_segment) {  // the block's rows in a fixed order: one partial per (chunk, token tile, anchor)
        __syncthreads();
        if (tid < na) {
            double v = 0.0;
            for (int r = 0; r < RPB; ++r) v += rows[r][tid];
            jb.partial[((int64_t)chunk * jb.n_token_tiles + tile) * jb.n_sel + a0 + tid] = v;
        }
    }
}

// Reduce-scatter of kAnchorTile per-lane sums over the LPR lanes of a row (LPR a power of two, lanes of a row are
// consecutive): afterwards lane `lir` holds the row's totals of its own anchors in acc[0 .. max(1, kAnchorTile /
// LPR)), anchor_of_lane() says which.  Lanes 16 and up of a wider row hold copies that anchor_of_lane() maps
// past the tile, so they are ignored.
template <int LPR>
__device__ __forceinline__ int anchor_of_lane(int lir, int k)
{
    if constexpr (LPR >= kAnchorTile)
        return lir + k * LPR;                       // k == 0: anchor lir (invalid from kAnchorTile on)
    else
        return (kAnchorTile / LPR) * lir + k;
}
template <int CNT, int OFF, int LPR>
__device__ __forceinline__ void reduce_scatter_round(double (&acc)[kAnchorTile], int lir)
{
    if constexpr (OFF >= 1 && CNT >= 2) {
        const bool up = lir & OFF;
#pragma unroll
        for (int i = 0; i < CNT / 2; ++i) {
            const double keep = up ? acc[i + CNT / 2] : acc[i];
            const double send = up ? acc[i] : acc[i + CNT / 2];
            acc[i] = keep + __shfl_xor(send, OFF, LPR);
        }
        reduce_scatter_round<CNT / 2, OFF / 2, LPR>(acc, lir);
    }
}
template <int LPR>
__device__ __forceinline__ void row_reduce_scatter(double (&acc)[kAnchorTile], int lir)
{
    static_assert(kAnchorTile == 16, "written for tiles of 16 anchors");
#pragma unroll
    for (int off = LPR / 2; off >= kAnchorTile; off >>= 1)
#pragma unroll
        for (int j = 0; j < kAnchorTile; ++j) acc[j] += __shfl_xor(acc[j], off, LPR);
    constexpr int OFF0 = (LPR < kAnchorTile ? LPR : kAnchorTile) / 2;
    reduce_scatter_round<kAnchorTile, OFF0, LPR>(acc, lir);
}

// One softmax per (layer, head, token), pools of up to kAnchorTile selected anchors: a row's distances are
// complete inside the LPR lanes that read the row, so this kernel finishes the softmax itself and writes the
// weights (no partial sums, no second kernel).
// Lane r of a row takes anchors r, r + LPR, ...; maximum, arg-max (lowest index among equals) and denominator
// are joined by fixed butterflies, so all lanes of a row agree bit for bit.  The exponent is formed in double
// (distances of a few hundred differ by fractions); the exponential and the normalisation are fp32, which is
// what the fp32 weights can resolve.
template <typename T, int LPR>
__global__ __launch_bounds__(kBlock) void dist_row_softmax_kernel(const DistParams p)
{
    constexpr int EPV = Elem<T>::EPV;
    constexpr int RPB = kBlock / LPR;
    constexpr int NPL = (kAnchorTile + LPR - 1) / LPR;  // anchors per lane
    const DistJob &jb = p.job[job_of_block(p)];
    const int tid = threadIdx.x;
    const int row = tid / LPR, lir = tid % LPR;
    const int bx = blockIdx.x - jb.block0;
    const int tile = bx % jb.n_token_tiles;
    const int chunk = bx / jb.n_token_tiles;
    const int na = jb.n_sel;  // 1 ... kAnchorTile (checked by the host)
    const int t = tile * RPB + row;
    const bool valid = t < jb.S;
    const int lh0 = chunk * p.lh_per_block;
    const int lh1 = min(lh0 + p.lh_per_block, p.LH);
    if (bx == 0 && jb.selected_out && tid < jb.n_anchors) jb.selected_out[tid] = (int32_t)((jb.sel_mask >> tid) & 1);

    const T *seg = static_cast<const T *>(jb.seg_k);
    for (int lh = lh0; lh < lh1; ++lh) {
        double acc[kAnchorTile];
#pragma unroll
        for (int j = 0; j < kAnchorTile; ++j) acc[j] = 0.0;
        if (valid) {
            const int l = lh / p.H, h = lh % p.H;
            const u32x4 rs = load16_stream(seg + l * jb.s_seg.layer + h * jb.s_seg.head + t * jb.s_seg.token + lir * EPV);
            const int64_t aoff = l * p.s_anc.layer + h * p.s_anc.head + t * p.s_anc.token + lir * EPV;
            u32x4 ra[kAnchorTile];
#pragma unroll
            for (int j = 0; j < kAnchorTile; ++j)
                if (j < na) ra[j] = load16_stream(static_cast<const T *>(p.anc[jb.a0 + j]) + aoff);
            float x[EPV];
            unpack<T>(rs, x);
#pragma unroll
            for (int j = 0; j < kAnchorTile; ++j)
                if (j < na) sqdiff_acc<T>(acc[j], x, ra[j]);
        }
        // Sum over the lanes of the row and hand each lane its own anchors in one go: in every round a lane keeps
        // one half of its values and adds the partner's copy of that half (15 exchanges for 16 anchors over 16
        // lanes instead of 64 for a butterfly per anchor).  Rows wider than 16 lanes first fold their upper lanes in.
        row_reduce_scatter<LPR>(acc, lir);
        double sc[NPL];
        double smax = -INFINITY;
        int best = kAnchorTile;
#pragma unroll
        for (int k = 0; k < NPL; ++k) {
            const int a = anchor_of_lane<LPR>(lir, k);
            sc[k] = a < na ? -sqrt(acc[k]) : -INFINITY;
            if (sc[k] > smax) {  // ascending a: the lowest index wins among equals
                smax = sc[k];
                best = a;
            }
        }
#pragma unroll
        for (int off = LPR / 2; off >= 1; off >>= 1) {
            const double om = __shfl_xor(smax, off, LPR);
            const int ob = __shfl_xor(best, off, LPR);
            if (om > smax || (om == smax && ob < best)) {
                smax = om;
                best = ob;
            }
        }
        float e[NPL], denom = 0.f;
#pragma unroll
        for (int k = 0; k < NPL; ++k) {
            const int a = anchor_of_lane<LPR>(lir, k);
            e[k] = a < na ? (p.rule == KVCOMM_RULE_NEAREST ? (a == best ? 1.f : 0.f)
                                                           : expf((float)((sc[k] - smax) / p.tau)))
                          : 0.f;
            denom += e[k];
        }
#pragma unroll
        for (int off = LPR / 2; off >= 1; off >>= 1) denom += __shfl_xor(denom, off, LPR);
        if (valid) {
            const int64_t slot = (int64_t)lh * jb.S + t;
            float *wrow = jb.weights + slot * jb.n_anchors;
#pragma unroll
            for (int k = 0; k < NPL; ++k) {
                const int a = anchor_of_lane<LPR>(lir, k);
                if (a < na) wrow[p.col[jb.a0 + a]] = e[k] / denom;
            }
            for (int c = lir; c < jb.n_anchors; c += LPR)
                if (!((jb.sel_mask >> c) & 1)) wrow[c] = 0.f;
            if (lir == 0 && jb.nearest) jb.nearest[slot] = p.col[jb.a0 + best];
        }
    }
}

constexpr int kCosTile = 8;  // anchors per lane in the cosine variant (two accumulators each)

// Cosine variant: per chunk, token and selected anchor the three sums <x,y>, |x|^2, |y|^2
// (x = segment key row, y = anchor key row), laid out [component][chunk][token][anchor].
template <typename T, int LPR>
__global__ __launch_bounds__(kBlock) void cos_partial_kernel(const DistParams p)
{
    constexpr int EPV = Elem<T>::EPV;
    constexpr int RPB = kBlock / LPR;
    const DistJob &jb = p.job[job_of_block(p)];
    const int tid = threadIdx.x;
    const int row = tid / LPR, lir = tid % LPR;
    const int bx = blockIdx.x - jb.block0;
    const int tile = bx % jb.n_token_tiles;
    const int chunk = bx / jb.n_token_tiles;
    const int a0 = blockIdx.y * kCosTile;
    const int na = min(kCosTile, jb.n_sel - a0);
    if (na <= 0) return;
    const int t = tile * RPB + row;
    const bool valid = t < jb.S;
    const int lh0 = chunk * p.lh_per_block;
    const int lh1 = min(lh0 + p.lh_per_block, p.LH);

    __shared__ double rows[RPB][kCosTile][3];
    double dot[kCosTile], ny[kCosTile], nx = 0.0;
#pragma unroll
    for (int j = 0; j < kCosTile; ++j) dot[j] = ny[j] = 0.0;

    if (valid) {
        const T *seg = static_cast<const T *>(jb.seg_k);
        for (int lh = lh0; lh < lh1; ++lh) {
            const int l = lh / p.H, h = lh % p.H;
            const u32x4 rs = load16_stream(seg + l * jb.s_seg.layer + h * jb.s_seg.head + t * jb.s_seg.token + lir * EPV);
            const int64_t aoff = l * p.s_anc.layer + h * p.s_anc.head + t * p.s_anc.token + lir * EPV;
            u32x4 ra[kCosTile];
#pragma unroll
            for (int j = 0; j < kCosTile; ++j)
                if (j < na) ra[j] = load16_stream(static_cast<const T *>(p.anc[jb.a0 + a0 + j]) + aoff);
            float x[EPV];
            unpack<T>(rs, x);
#pragma unroll
            for (int e = 0; e < EPV; ++e) nx = fma((double)x[e], (double)x[e], nx);
#pragma unroll
            for (int j = 0; j < kCosTile; ++j)
                if (j < na) {
                    float y[EPV];
                    unpack<T>(ra[j], y);
#pragma unroll
                    for (int e = 0; e < EPV; ++e) {
                        dot[j] = fma((double)x[e], (double)y[e], dot[j]);
                        ny[j] = fma((double)y[e], (double)y[e], ny[j]);
                    }
                }
        }
    }
#pragma unroll
    for (int off = LPR / 2; off >= 1; off >>= 1) nx += __shfl_xor(nx, off, LPR);
#pragma unroll
    for (int j = 0; j < kCosTile; ++j) {
        if (j < na) {
            double u = dot[j], v = ny[j];
#pragma unroll
            for (int off = LPR / 2; off >= 1; off >>= 1) {
                u += __shfl_xor(u, off, LPR);
                v += __shfl_xor(v, off, LPR);
            }
            if (p.per_segment) {
                if (lir == 0) {
                    rows[row][j][0] = valid ? u : 0.0;
                    rows[row][j][1] = valid ? nx : 0.0;
                    rows[row][j][2] = valid ? v : 0.0;
                }
            } else if (valid && lir == 0) {
                const int64_t i = ((int64_t)chunk * jb.S + t) * jb.n_sel + a0 + j;
                jb.partial[i] = u;
                jb.partial[jb.comp_stride + i] = nx;
                jb.partial[2 * jb.comp_stride + i] = v;
            }
        }
    }
    if (p.per_segment) {
        __syncthreads();
        if (tid < 3 * na) {
            const int j = tid / 3, c = tid % 3;
            double v = 0.0;
            for (int r = 0; r < RPB; ++r) v += rows[r][j][c];
            jb.partial[c * jb.comp_stride + ((int64_t)chunk * jb.n_token_tiles + tile) * jb.n_sel + a0 + j] = v;
        }
    }
}

struct FinalJob {
    const double *partial;
    float *weights;
    int32_t *nearest;
    int32_t *selected_out;
    int64_t comp_stride;   // cosine rule: elements between the three partial components
    uint64_t sel_mask;     // bit a = anchor a is selected
    int32_t S, n_slots, n_anchors, chunk_lanes, block0, n_token_tiles;
    int16_t a0, n_sel;     // its selected anchors: entries [a0, a0 + n_sel) of col
};

struct FinalParams {
    FinalJob job[KVCOMM_MAX_BATCH];
    int32_t n_chunks, gran, rule, n_jobs;
    double tau;
    uint8_t col[KVCOMM_MAX_ANCHORS];   // original index of a selected anchor
};

// Score whose softmax across anchors gives the weights: minus the l2 distance, or the cosine
// similarity <x,y> / (|x| |y|) (0 when a norm is 0).
__device__ __forceinline__ double score_of(const FinalParams &p, double s0, double s1, double s2)
{
    if (p.rule != KVCOMM_RULE_COSINE_SOFTMAX) return -sqrt(s0);
    const double den = sqrt(s1) * sqrt(s2);
    return den > 0.0 ? s0 / den : 0.0;
}

// Softmax over the selected anchors of one slot, evaluated identically by each of the
// slot's threads from the scores in `sc` (LDS): every thread walks the anchors in index
// order, so all agree bit for bit on the maximum, the arg-max and the denominator.
__device__ __forceinline__ void slot_softmax(const FinalParams &p, const FinalJob &jb, const double *sc, int a, int64_t slot)
{
    double smax = sc[0];
    int best = 0;
    for (int j = 1; j < jb.n_sel; ++j)
        if (sc[j] > smax) {
            smax = sc[j];
            best = j;
        }
    double w;
    if (p.rule == KVCOMM_RULE_NEAREST) {
        w = a == best ? 1.0 : 0.0;
    } else {
        double denom = 0.0;
        for (int j = 0; j < jb.n_sel; ++j) denom += exp((sc[j] - smax) / p.tau);
        w = exp((sc[a] - smax) / p.tau) / denom;
    }
    jb.weights[slot * jb.n_anchors + p.col[jb.a0 + a]] = (float)w;
    if (a == 0) {
        if (jb.nearest) jb.nearest[slot] = p.col[jb.a0 + best];
        for (int c = 0; c < jb.n_anchors; ++c)
            if (!((jb.sel_mask >> c) & 1)) jb.weights[slot * jb.n_anchors + c] = 0.f;
    }
}

// Per-token and per-(layer, head, token) granularity.  A (slot, selected anchor) pair is summed by CL threads:
// thread (c, slot, anchor) adds chunks c, c + CL, ... in increasing order (its loads all in flight at once; anchor,
// then slot, vary fastest over the threads, so a wavefront reads whole runs of a chunk's row), the CL sums meet in
// LDS and are added in increasing c, so the result does not depend on timing.
__global__ __launch_bounds__(kBlock) void finalize_kernel(const FinalParams p)
{
    __shared__ double dsh[kBlock];
    __shared__ double red[3][kBlock];
    int ji = 0;
#pragma unroll
    for (int i = 1; i < KVCOMM_MAX_BATCH; ++i)
        if (i < p.n_jobs && (int)blockIdx.x >= p.job[i].block0) ji = i;
    const FinalJob &jb = p.job[ji];
    const int bx = blockIdx.x - jb.block0;
    const int tid = threadIdx.x;
    if (bx == 0 && jb.selected_out && tid < jb.n_anchors) jb.selected_out[tid] = (int32_t)((jb.sel_mask >> tid) & 1);
    if (jb.n_sel == 0) {  // nothing selected: all weights 0, nearest -1
        const int64_t slot = (int64_t)bx * kBlock + tid;
        if (slot < jb.n_slots) {
            for (int c = 0; c < jb.n_anchors; ++c) jb.weights[slot * jb.n_anchors + c] = 0.f;
            if (jb.nearest) jb.nearest[slot] = -1;
        }
        return;
    }
    const int CL = jb.chunk_lanes;             // power of two, CL * n_sel <= kBlock
    const int spb = kBlock / (CL * jb.n_sel);  // slots per block
    const int per_lane = spb * jb.n_sel;       // (slot, anchor) pairs of a block
    const int a = tid % jb.n_sel, sl = (tid / jb.n_sel) % spb, cl = tid / per_lane;
    const int64_t slot = (int64_t)bx * spb + sl;
    const bool active = cl < CL && slot < jb.n_slots;
    const bool cosine = p.rule == KVCOMM_RULE_COSINE_SOFTMAX;
    double s0 = 0.0, s1 = 0.0, s2 = 0.0;
    if (active) {
        if (p.gran == KVCOMM_W_TOKEN) {
            for (int c = cl; c < p.n_chunks; c += CL) {
                const int64_t i = ((int64_t)c * jb.S + slot) * jb.n_sel + a;
                s0 += jb.partial[i];
                if (cosine) {
                    s1 += jb.partial[jb.comp_stride + i];
                    s2 += jb.partial[2 * jb.comp_stride + i];
                }
            }
        } else {  // one chunk per (layer, head): slot = chunk * S + t, CL == 1
            const int64_t i = slot * jb.n_sel + a;
            s0 = jb.partial[i];
            if (cosine) {
                s1 = jb.partial[jb.comp_stride + i];
                s2 = jb.partial[2 * jb.comp_stride + i];
            }
        }
    }
    if (CL > 1) {
        red[0][tid] = s0;
        if (cosine) {
            red[1][tid] = s1;
            red[2][tid] = s2;
        }
        __syncthreads();
        if (active && cl == 0) {
            for (int c = 1; c < CL; ++c) {
                s0 += red[0][c * per_lane + tid];
                if (cosine) {
                    s1 += red[1][c * per_lane + tid];
                    s2 += red[2][c * per_lane + tid];
                }
            }
        }
    }
    if (active && cl == 0) dsh[sl * jb.n_sel + a] = score_of(p, s0, s1, s2);
    __syncthreads();
    if (active && cl == 0) slot_softmax(p, jb, dsh + sl * jb.n_sel, a, slot);
}

// Per-segment granularity: one block per segment.  The distance kernel has left one partial per (chunk, token
// tile, anchor), n_rows = n_chunks * n_token_tiles rows of n_sel values.  Thread t adds the rows g, g + G, ... of
// anchor t % n_sel (g = t / n_sel, G = 256 / n_sel groups: consecutive threads read consecutive addresses) and a
// fixed-order sum over the groups closes each anchor, so the result does not depend on timing.
__global__ __launch_bounds__(kBlock) void finalize_segment_kernel(const FinalParams p)
{
    __shared__ double red[3][kBlock];
    __shared__ double dsh[KVCOMM_MAX_ANCHORS];
    const FinalJob &jb = p.job[blockIdx.x];
    const int tid = threadIdx.x;
    if (jb.selected_out && tid < jb.n_anchors) jb.selected_out[tid] = (int32_t)((jb.sel_mask >> tid) & 1);
    if (jb.n_sel == 0) {
        if (tid < jb.n_anchors) jb.weights[tid] = 0.f;
        if (tid == 0 && jb.nearest) jb.nearest[0] = -1;
        return;
    }
    const int n_sel = jb.n_sel, G = kBlock / n_sel;
    const int a = tid % n_sel, g = tid / n_sel;
    const int64_t n_rows = (int64_t)p.n_chunks * jb.n_token_tiles;
    const int n_comp = p.rule == KVCOMM_RULE_COSINE_SOFTMAX ? 3 : 1;
    double s[3][4] = {};   // four interleaved chains per component keep several loads in flight
    if (g < G) {
        for (int c = 0; c < n_comp; ++c) {
            const double *src = jb.partial + c * jb.comp_stride + a;
            int64_t r = g;
            for (; r + 3 * G < n_rows; r += 4 * G) {
#pragma unroll
                for (int u = 0; u < 4; ++u) s[c][u] += src[(r + u * G) * n_sel];
            }
            for (int u = 0; r < n_rows; r += G, ++u) s[c][u] += src[r * n_sel];
        }
    }
    for (int c = 0; c < n_comp; ++c) red[c][tid] = (s[c][0] + s[c][1]) + (s[c][2] + s[c][3]);
    __syncthreads();
    if (tid < n_sel) {
        double tot[3] = {0.0, 0.0, 0.0};
        for (int c = 0; c < n_comp; ++c)
            for (int gg = 0; gg < G; ++gg) tot[c] += red[c][gg * n_sel + tid];
        dsh[tid] = score_of(p, tot[0], tot[1], tot[2]);
    }
    __syncthreads();
    if (tid < n_sel) slot_softmax(p, jb, dsh, tid, 0);
}

template <typename T, int LPR>
int launch_dist(const DistParams &p, int n_blocks, int max_sel, bool cosine, hipStream_t stream)
{
    if (p.fused) return launch(dist_row_softmax_kernel<T, LPR>, dim3(n_blocks), dim3(kBlock), 0, stream, p);
    if (cosine) {
        const int a_tiles = (max_sel + kCosTile - 1) / kCosTile;
        return launch(cos_partial_kernel<T, LPR>, dim3(n_blocks, a_tiles), dim3(kBlock), 0, stream, p);
    }
    const int a_tiles = (max_sel + kAnchorTile - 1) / kAnchorTile;
    return launch(dist_partial_kernel<T, LPR>, dim3(n_blocks, a_tiles), dim3(kBlock), 0, stream, p);
}

int check_rule(int rule)
{
    return (rule == KVCOMM_RULE_L2_SOFTMAX || rule == KVCOMM_RULE_NEAREST || rule == KVCOMM_RULE_COSINE_SOFTMAX)
               ? KVCOMM_OK
               : KVCOMM_EINVAL;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Bytes of segment j's partial sums for a plan.
size_t job_partial_bytes(const DistPlan &pl, int32_t seg_len, int32_t n_anchors, int rule)
{
    const size_t n_comp = rule == KVCOMM_RULE_COSINE_SOFTMAX ? 3 : 1;
    return sizeof(double) * n_comp * (size_t)pl.n_chunks * seg_len * n_anchors;
}

}  // namespace

extern "C" size_t kvcomm_weight_slots(const kvcomm_model *model, int32_t seg_len, int32_t gran)
{
    if (check_model(model) || check_gran(gran) || seg_len <= 0) return 0;
    if (gran == KVCOMM_W_TOKEN) return (size_t)seg_len;
    if (gran == KVCOMM_W_SEGMENT) return 1;
    return (size_t)model->n_layers * model->n_kv_heads * seg_len;
}

extern "C" size_t kvcomm_anchor_weights_batch_workspace(const kvcomm_model *model, int32_t gran, int32_t rule,
                                                        const int32_t *seg_lens, const int32_t *n_anchors,
                                                        int32_t n_jobs)
{
    if (check_model(model) || check_gran(gran) || check_rule(rule) || !seg_lens || !n_anchors || n_jobs <= 0 ||
        n_jobs > KVCOMM_MAX_BATCH)
        return 0;
    for (int j = 0; j < n_jobs; ++j)
        if (seg_lens[j] <= 0 || n_anchors[j] <= 0 || n_anchors[j] > KVCOMM_MAX_ANCHORS) return 0;
    const DistPlan pl = make_plan(model, seg_lens, n_jobs, gran);
    size_t total = 0;
    for (int j = 0; j < n_jobs; ++j) total += align256(job_partial_bytes(pl, seg_lens[j], n_anchors[j], rule));
    return total;
}

extern "C" size_t kvcomm_anchor_weights_rule_workspace(const kvcomm_model *model, int32_t seg_len, int32_t n_anchors,
                                                       int32_t gran, int32_t rule)
{
    if (check_model(model) || check_gran(gran) || check_rule(rule) || seg_len <= 0 || n_anchors <= 0 ||
        n_anchors > KVCOMM_MAX_ANCHORS)
        return 0;
    const DistPlan pl = make_plan(model, &seg_len, 1, gran);
    return job_partial_bytes(pl, seg_len, n_anchors, rule);
}

extern "C" size_t kvcomm_anchor_weights_workspace(const kvcomm_model *model, int32_t seg_len, int32_t n_anchors,
                                                  int32_t gran)
{
    return kvcomm_anchor_weights_rule_workspace(model, seg_len, n_anchors, gran, KVCOMM_RULE_L2_SOFTMAX);
}

extern "C" int kvcomm_anchor_weights_batch(const kvcomm_model *model, int32_t gran, int32_t rule, float temperature,
                                           kvcomm_tensor anchor_layout, const kvcomm_weights_job *jobs,
                                           int32_t n_jobs, void *workspace, size_t workspace_bytes, void *stream)
{
    int st = check_model(model);
    if (st) return st;
    if ((st = check_gran(gran)) || (st = check_rule(rule))) return st;
    if (!jobs || n_jobs <= 0) return KVCOMM_EINVAL;
    if (n_jobs > KVCOMM_MAX_BATCH) return KVCOMM_EUNSUPPORTED;
    if (!(temperature > 0.f)) return KVCOMM_EINVAL;  // also rejects NaN
    const int dt = model->dtype;
    if ((st = check_tensor(anchor_layout, dt, false))) return st;
    int32_t seg_lens[KVCOMM_MAX_BATCH];
    for (int j = 0; j < n_jobs; ++j) {
        const kvcomm_weights_job &jd = jobs[j];
        if (jd.seg_len <= 0 || jd.n_anchors <= 0) return KVCOMM_EINVAL;
        if (jd.n_anchors > KVCOMM_MAX_ANCHORS) return KVCOMM_EUNSUPPORTED;
        if ((st = check_tensor(jd.seg_base_k, dt, true))) return st;
        if (!jd.anchor_base_k || !jd.anchor_len || !jd.weights_out) return KVCOMM_EINVAL;
        seg_lens[j] = jd.seg_len;
    }

    const DistPlan pl = make_plan(model, seg_lens, n_jobs, gran);
    const bool cosine = rule == KVCOMM_RULE_COSINE_SOFTMAX;
    DistParams dp{};
    FinalParams fp{};
    int n_sel_total = 0, max_sel = 0, min_sel = KVCOMM_MAX_ANCHORS;
    size_t need = 0;
    for (int j = 0; j < n_jobs; ++j) {
        const kvcomm_weights_job &jd = jobs[j];
        DistJob &dj = dp.job[j];
        FinalJob &fj = fp.job[j];
        dj.a0 = fj.a0 = (int16_t)n_sel_total;
        int n_sel = 0;
        for (int a = 0; a < jd.n_anchors; ++a) {
            if (jd.anchor_len[a] < 0) return KVCOMM_EINVAL;
            if (jd.anchor_len[a] < jd.seg_len) continue;
            if (!jd.anchor_base_k[a] || !aligned16(jd.anchor_base_k[a])) return KVCOMM_EINVAL;
            if (n_sel_total + n_sel >= KVCOMM_MAX_ANCHORS) return KVCOMM_EUNSUPPORTED;  // over all segments of the launch
            fp.col[n_sel_total + n_sel] = dp.col[n_sel_total + n_sel] = (uint8_t)a;
            fj.sel_mask |= (uint64_t)1 << a;
            dp.anc[n_sel_total + n_sel] = jd.anchor_base_k[a];
            ++n_sel;
        }
        dj.n_sel = fj.n_sel = (int16_t)n_sel;
        n_sel_total += n_sel;
        max_sel = n_sel > max_sel ? n_sel : max_sel;
        min_sel = n_sel < min_sel ? n_sel : min_sel;
        need += n_jobs == 1 ? job_partial_bytes(pl, jd.seg_len, jd.n_anchors, rule)
                            : align256(job_partial_bytes(pl, jd.seg_len, jd.n_anchors, rule));
    }
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return KVCOMM_EWORKSPACE;

    hipStream_t s = static_cast<hipStream_t>(stream);
    dp.s_anc = strides_of(anchor_layout);
    dp.H = model->n_kv_heads;
    dp.LH = model->n_layers * model->n_kv_heads;
    dp.lh_per_block = pl.lh_per_block;
    dp.n_jobs = n_jobs;
    // One softmax per (layer, head, token): a row's distances are complete inside the lanes that read the
    // row, so the distance kernel writes the weights itself (no partial sums, no second kernel) as long as
    // every segment's selected anchors fit one anchor tile.
    const bool fused = gran == KVCOMM_W_LAYER_HEAD_TOKEN && !cosine && min_sel >= 1 && max_sel <= kAnchorTile;
    // (one (layer, head) pair per block, as in the two-stage form: with runs of several pairs per block the
    // softmax of one pair delays the loads of the next, measured 6 % slower)
    dp.fused = fused ? 1 : 0;
    dp.per_segment = gran == KVCOMM_W_SEGMENT ? 1 : 0;
    dp.rule = rule;
    dp.tau = (double)temperature;
    fp.n_chunks = pl.n_chunks;
    fp.gran = gran;
    fp.rule = rule;
    fp.n_jobs = n_jobs;
    fp.tau = (double)temperature;
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    int64_t dist_blocks = 0, final_blocks = 0;
    for (int j = 0; j < n_jobs; ++j) {
        const kvcomm_weights_job &jd = jobs[j];
        DistJob &dj = dp.job[j];
        FinalJob &fj = fp.job[j];
        dj.seg_k = jd.seg_base_k.ptr;
        dj.s_seg = strides_of(jd.seg_base_k);
        dj.partial = reinterpret_cast<double *>(ws);
        ws += align256(job_partial_bytes(pl, jd.seg_len, jd.n_anchors, rule));
        dj.comp_stride = (int64_t)pl.n_chunks * jd.seg_len * dj.n_sel;  // <= a third of the segment's partials
        dj.S = jd.seg_len;
        dj.n_token_tiles = (jd.seg_len + pl.rpb - 1) / pl.rpb;
        dj.block0 = (int32_t)dist_blocks;
        dist_blocks += (int64_t)pl.n_chunks * dj.n_token_tiles;

        dj.weights = jd.weights_out;
        dj.nearest = jd.nearest_out;
        dj.selected_out = jd.selected_out;
        dj.sel_mask = fj.sel_mask;
        dj.n_anchors = jd.n_anchors;
        fj.partial = dj.partial;
        fj.weights = jd.weights_out;
        fj.nearest = jd.nearest_out;
        fj.selected_out = jd.selected_out;
        fj.comp_stride = dj.comp_stride;
        fj.n_token_tiles = dj.n_token_tiles;
        fj.S = jd.seg_len;
        fj.n_slots = (int32_t)kvcomm_weight_slots(model, jd.seg_len, gran);
        fj.n_anchors = jd.n_anchors;
        int cl = 1;
        if (gran == KVCOMM_W_TOKEN && dj.n_sel > 0)
            while (cl < 8 && 2 * cl * dj.n_sel <= kBlock && 2 * cl <= pl.n_chunks) cl *= 2;
        fj.chunk_lanes = cl;
        const int spb = dj.n_sel > 0 ? kBlock / (cl * dj.n_sel) : kBlock;
        fj.block0 = (int32_t)final_blocks;
        final_blocks += (fj.n_slots + spb - 1) / spb;
    }
    if (dist_blocks > 0x7fffffff || final_blocks > 0x7fffffff) return KVCOMM_EUNSUPPORTED;

    if (max_sel > 0) {
        st = KVCOMM_EUNSUPPORTED;
        const int nb = (int)dist_blocks;
        if (dt == KVCOMM_BF16) {
            switch (pl.lpr) {
                case 8: st = launch_dist<bf16_t, 8>(dp, nb, max_sel, cosine, s); break;
                case 16: st = launch_dist<bf16_t, 16>(dp, nb, max_sel, cosine, s); break;
                case 32: st = launch_dist<bf16_t, 32>(dp, nb, max_sel, cosine, s); break;
            }
        } else {
            switch (pl.lpr) {
                case 16: st = launch_dist<float, 16>(dp, nb, max_sel, cosine, s); break;
                case 32: st = launch_dist<float, 32>(dp, nb, max_sel, cosine, s); break;
                case 64: st = launch_dist<float, 64>(dp, nb, max_sel, cosine, s); break;
            }
        }
        if (st) return st;
    }
    if (fused) return KVCOMM_OK;
    if (gran == KVCOMM_W_SEGMENT)
        return launch(finalize_segment_kernel, dim3(n_jobs), dim3(kBlock), 0, s, fp);
    return launch(finalize_kernel, dim3((unsigned)final_blocks), dim3(kBlock), 0, s, fp);
}

extern "C" int kvcomm_anchor_weights_rule(const kvcomm_model *model, int32_t gran, int32_t rule, float temperature,
                                          kvcomm_tensor seg_base_k, int32_t seg_len,
                                          const void *const *anchor_base_k, kvcomm_tensor anchor_layout,
                                          const int32_t *anchor_len, int32_t n_anchors, float *weights_out,
                                          int32_t *nearest_out, int32_t *selected_out, void *workspace,
                                          size_t workspace_bytes, void *stream)
{
    kvcomm_weights_job job{};
    job.seg_base_k = seg_base_k;
    job.seg_len = seg_len;
    job.anchor_base_k = anchor_base_k;
    job.anchor_len = anchor_len;
    job.n_anchors = n_anchors;
    job.weights_out = weights_out;
    job.nearest_out = nearest_out;
    job.selected_out = selected_out;
    return kvcomm_anchor_weights_batch(model, gran, rule, temperature, anchor_layout, &job, 1, workspace,
                                       workspace_bytes, stream);
}

extern "C" int kvcomm_anchor_weights(const kvcomm_model *model, int32_t gran, float temperature,
                                     kvcomm_tensor seg_base_k, int32_t seg_len, const void *const *anchor_base_k,
                                     kvcomm_tensor anchor_layout, const int32_t *anchor_len, int32_t n_anchors,
                                     float *weights_out, int32_t *nearest_out, int32_t *selected_out, void *workspace,
                                     size_t workspace_bytes, void *stream)
{
    return kvcomm_anchor_weights_rule(model, gran, KVCOMM_RULE_L2_SOFTMAX, temperature, seg_base_k, seg_len,
                                      anchor_base_k, anchor_layout, anchor_len, n_anchors, weights_out, nearest_out,
                                      selected_out, workspace, workspace_bytes, stream);
}

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU, looked up once per GPU

// Address of the current device's copy of `scratch` (every GPU holds its own copy at its own address).
int static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return KVCOMM_EHIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return KVCOMM_EHIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return KVCOMM_OK;
}

}  // namespace

extern "C" size_t kvcomm_anchor_weights_static_capacity(void) { return KVCOMM_STATIC_SCRATCH_BYTES; }

extern "C" int kvcomm_anchor_weights_static(const kvcomm_model *model, int32_t gran, float temperature,
                                            kvcomm_tensor seg_base_k, int32_t seg_len,
                                            const void *const *anchor_base_k, kvcomm_tensor anchor_layout,
                                            const int32_t *anchor_len, int32_t n_anchors, float *weights_out,
                                            int32_t *nearest_out, int32_t *selected_out, void *stream)
{
    // Size first: a request that does not fit is refused before anything else is looked at.
    int st = check_model(model);
    if (st) return st;
    if ((st = check_gran(gran))) return st;
    if (seg_len <= 0 || n_anchors <= 0) return KVCOMM_EINVAL;
    if (n_anchors > KVCOMM_MAX_ANCHORS) return KVCOMM_EUNSUPPORTED;
    const size_t need = kvcomm_anchor_weights_workspace(model, seg_len, n_anchors, gran);
    if (need > KVCOMM_STATIC_SCRATCH_BYTES) return KVCOMM_EWORKSPACE;
    void *ws = nullptr;
    if ((st = static_scratch(&ws))) return st;
    // Nothing in the array has to start at zero: the distance kernel writes every partial sum that the
    // finalize kernel reads, whatever an earlier call left behind.
    return kvcomm_anchor_weights(model, gran, temperature, seg_base_k, seg_len, anchor_base_k, anchor_layout,
                                 anchor_len, n_anchors, weights_out, nearest_out, selected_out, ws,
                                 KVCOMM_STATIC_SCRATCH_BYTES, stream);
}
