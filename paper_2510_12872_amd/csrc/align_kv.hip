// kvcomm_align_kv: positional alignment fused with the offset approximation
// (Eq. "ph_update" / Eq. "pf_update" of the paper, keys first rotated to their new
// position as Sec. 3.1 "Positional Alignment" requires).
//
// The kernel is a single streaming pass bounded by HBM bandwidth: per cache row
// (layer, kv head, token) it reads the base K and V rows and one dK and one dV row per
// selected anchor, and writes one K and one V row: 2*(A+2) rows of D elements.
//
// Work split.  A row is covered by LPR = D / (2 * EPV) lanes (EPV = elements per 16-byte
// vector).  Lane r of a row owns channels [r*EPV, r*EPV+EPV) of the first half and the
// same channels of the second half, i.e. both members of each RoPE pair (i, i + D/2), so
// the rotation needs no cross-lane traffic and the kernel may run in place.  A block of
// 256 threads owns a tile of 256/LPR consecutive tokens of one (layer, head) and of ONE of
// the two tensors (blockIdx.y: 0 = keys, 1 = values): the two streams are independent, and
// splitting them halves the registers per lane so that many wavefronts per CU keep loads in
// flight.  Every access to a tensor is a run of whole 128-byte lines; the traffic is marked
// non-temporal.  Per-token anchor weights and the cos/sin tables load once per block (LDS).
// cos/sin: the angle delta * theta^(-2i/D) is formed and reduced modulo 2*pi in double from a
// host-computed frequency table (kernel argument); sine and cosine of the reduced angle are fp32.
#include "align_common.h"

namespace {

using namespace kvc;

#ifndef KVC_ALIGN_BLOCKS
#define KVC_ALIGN_BLOCKS 32768  // blocks per tensor the grid aims at (measured best on MI355X)
#endif

#ifndef KVC_ALIGN_INFLIGHT
#define KVC_ALIGN_INFLIGHT 2
#endif
#ifndef KVC_ALIGN_WPE
#define KVC_ALIGN_WPE 4   // wavefronts per SIMD the register budget is sized for (measured best: 4 with 2 anchors in flight)
#endif

constexpr int kBlock = kAlignBlock;
constexpr int kAnchorsInFlight = KVC_ALIGN_INFLIGHT;

struct AlignParams {
    AlignJob job[KVCOMM_MAX_BATCH];
    Strides s_anc;
    int32_t H, LH;             // kv heads, layers*heads
    int32_t gran, n_jobs;
    int32_t lh_per_block;
    int32_t tiles_total;       // token tiles of all segments
    int32_t tab_delta[kMaxTab];                 // position delta of each rotation table
    const void *anc[2][KVCOMM_MAX_ANCHORS];     // [0] dK, [1] dV of the selected anchors of all segments
    uint8_t col[KVCOMM_MAX_ANCHORS];            // weight column of a selected anchor
    uint8_t tab[KVCOMM_MAX_ANCHORS];            // its rotation table (index among the segment's tables) + 1, 0 = identity
    double inv_freq[kMaxHalf];                  // theta^(-2i/D), i < D/2
};
static_assert(sizeof(AlignParams) <= 4096, "kernel arguments are limited to 4 KB");

template <typename T, int LPR>
__global__ __launch_bounds__(kBlock, KVC_ALIGN_WPE) void align_kernel(const AlignParams p)
{
    constexpr int EPV = Elem<T>::EPV;
    constexpr int HALF = LPR * EPV;  // D / 2
    constexpr int RPB = kBlock / LPR;

    // Block order: (layer, head) chunk, then segment, then token tile, so that the blocks in flight
    // write neighbouring slices of the same cache rows when the segments of a launch are adjacent.
    const int chunk = blockIdx.x / p.tiles_total;
    const int r = blockIdx.x % p.tiles_total;
    const AlignJob &jb = p.job[job_of_tile(p, r)];
    const int n_sel = jb.n_sel, a0 = jb.a0;

    extern __shared__ __align__(16) unsigned char smem_raw[];
    float2 *cs = reinterpret_cast<float2 *>(smem_raw);                          // [n_tab][HALF] (cos, sin)
    float *w_lds = reinterpret_cast<float *>(smem_raw) + 2 * jb.n_tab * HALF;   // [RPB][n_sel]

    const int tid = threadIdx.x;
    const int row = tid / LPR;
    const int lir = tid % LPR;
    const int tile = r - jb.tile0;
    const int which = blockIdx.y;          // 0 = keys (rotated), 1 = values
    const bool is_k = which == 0;
    const int t = tile * RPB + row;
    const bool valid = t < jb.S;
    const int lh0 = chunk * p.lh_per_block;
    const int lh1 = min(lh0 + p.lh_per_block, p.LH);

    if (is_k) {
        // cos/sin of delta * theta^(-2i/D): product and reduction modulo 2*pi in double.
        for (int idx = tid; idx < jb.n_tab * HALF; idx += kBlock) {
            const int r = idx / HALF, i = idx % HALF;
            cs[idx] = rope_cos_sin(p.tab_delta[jb.t0 + r], p.inv_freq[i]);
        }
    }
    if (p.gran != KVCOMM_W_LAYER_HEAD_TOKEN) {
        for (int idx = tid; idx < RPB * n_sel; idx += kBlock) {
            const int r = idx / n_sel, a = idx % n_sel;
            const int tt = tile * RPB + r;
            const int64_t slot = p.gran == KVCOMM_W_TOKEN ? tt : 0;
            w_lds[idx] = tt < jb.S ? jb.weights[slot * jb.w_pitch + p.col[a0 + a]] : 0.f;
        }
    }
    __syncthreads();
    if (!valid) return;

    const bool rot_base = is_k && jb.base_tab != 0;
    float bc[EPV], bs[EPV];
    if (rot_base) {
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
            const float2 v = cs[(jb.base_tab - 1) * HALF + lir * EPV + e];
            bc[e] = v.x;
            bs[e] = v.y;
        }
    }

    const T *bp = static_cast<const T *>(jb.base[which]);
    T *op = static_cast<T *>(jb.out[which]);
    const Strides sb = jb.s_base[which], so = jb.s_out[which];
    const int64_t col0 = (int64_t)lir * EPV;

    for (int lh = lh0; lh < lh1; ++lh) {
        const int l = lh / p.H, h = lh % p.H;
        const T *xp = bp + l * sb.layer + h * sb.head + t * sb.token + col0;
        const u32x4 rlo = load16_stream(xp), rhi = load16_stream(xp + HALF);
        const int64_t aoff = l * p.s_anc.layer + h * p.s_anc.head + t * p.s_anc.token + col0;
        const float *wrow = p.gran == KVCOMM_W_LAYER_HEAD_TOKEN
                                ? jb.weights + ((int64_t)lh * jb.S + t) * jb.w_pitch
                                : nullptr;

        float lo[EPV], hi[EPV];
        unpack<T>(rlo, lo);
        unpack<T>(rhi, hi);
        if (rot_base) {
#pragma unroll
            for (int e = 0; e < EPV; ++e) {
                const float a = lo[e], b = hi[e];
                lo[e] = a * bc[e] - b * bs[e];
                hi[e] = b * bc[e] + a * bs[e];
            }
        }

        auto accumulate = [&](int a, const u32x4 &rdlo, const u32x4 &rdhi) {
            const float w = wrow ? wrow[p.col[a0 + a]] : w_lds[row * n_sel + a];
            float dlo[EPV], dhi[EPV];
            unpack<T>(rdlo, dlo);
            unpack<T>(rdhi, dhi);
            const int tb = is_k ? p.tab[a0 + a] : 0;
            if (tb) {
                const float2 *tcs = cs + (tb - 1) * HALF + lir * EPV;
#pragma unroll
                for (int e = 0; e < EPV; ++e) {
                    const float2 v = tcs[e];
                    const float x = dlo[e], y = dhi[e];
                    dlo[e] = x * v.x - y * v.y;
                    dhi[e] = y * v.x + x * v.y;
                }
            }
#pragma unroll
            for (int e = 0; e < EPV; ++e) {
                lo[e] += w * dlo[e];
                hi[e] += w * dhi[e];
            }
        };

        // kAnchorsInFlight anchors (twice as many independent 16-byte loads) are kept in flight.
        int a = 0;
        for (; a + kAnchorsInFlight <= n_sel; a += kAnchorsInFlight) {
            u32x4 x[kAnchorsInFlight][2];
#pragma unroll
            for (int u = 0; u < kAnchorsInFlight; ++u) {
                const T *d = static_cast<const T *>(p.anc[which][a0 + a + u]) + aoff;
                x[u][0] = load16_stream(d);
                x[u][1] = load16_stream(d + HALF);
            }
#pragma unroll
            for (int u = 0; u < kAnchorsInFlight; ++u) accumulate(a + u, x[u][0], x[u][1]);
        }
        for (; a < n_sel; ++a) {
            const T *d = static_cast<const T *>(p.anc[which][a0 + a]) + aoff;
            const u32x4 x0 = load16_stream(d), x1 = load16_stream(d + HALF);
            accumulate(a, x0, x1);
        }

        T *yp = op + l * so.layer + h * so.head + t * so.token + col0;
        store16_stream(yp, pack<T>(lo));
        store16_stream(yp + HALF, pack<T>(hi));
    }
}

template <typename T, int LPR>
int launch_align(const AlignParams &p, int n_blocks, int max_tab, int max_sel, hipStream_t stream)
{
    constexpr int HALF = LPR * Elem<T>::EPV;
    constexpr int RPB = kBlock / LPR;
    const size_t lds = sizeof(float2) * (size_t)max_tab * HALF + sizeof(float) * (size_t)RPB * max_sel;
    return launch(align_kernel<T, LPR>, dim3(n_blocks, 2), dim3(kBlock), lds, stream, p);
}

}  // namespace

extern "C" int kvcomm_align_kv_batch(const kvcomm_model *model, int32_t gran, kvcomm_tensor anchor_layout,
                                     const kvcomm_align_job *jobs, int32_t n_jobs, void *stream)
{
    AlignParams p{};
    AlignLaunch pl{};
    const int es = model ? elem_size(model->dtype) : 2;
    int st = plan_align(model, gran, anchor_layout, es, jobs, n_jobs, KVC_ALIGN_BLOCKS, p, pl,
                        [](int, const kvcomm_align_job &, int) { return (int)KVCOMM_OK; });
    if (st) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int nb = (int)pl.n_blocks;
    if (model->dtype == KVCOMM_BF16) {
        switch (pl.lpr) {
            case 4: return launch_align<bf16_t, 4>(p, nb, pl.max_tab, pl.max_sel, s);
            case 8: return launch_align<bf16_t, 8>(p, nb, pl.max_tab, pl.max_sel, s);
            case 16: return launch_align<bf16_t, 16>(p, nb, pl.max_tab, pl.max_sel, s);
        }
    } else {
        switch (pl.lpr) {
            case 8: return launch_align<float, 8>(p, nb, pl.max_tab, pl.max_sel, s);
            case 16: return launch_align<float, 16>(p, nb, pl.max_tab, pl.max_sel, s);
            case 32: return launch_align<float, 32>(p, nb, pl.max_tab, pl.max_sel, s);
        }
    }
    return KVCOMM_EUNSUPPORTED;
}

extern "C" int kvcomm_align_kv(const kvcomm_model *model, int32_t gran, kvcomm_tensor base_k, kvcomm_tensor base_v,
                               int32_t seg_len, const void *const *anchor_dk, const void *const *anchor_dv,
                               kvcomm_tensor anchor_layout, const int32_t *anchor_len, int32_t n_anchors,
                               const float *weights, int32_t delta_pos, const int32_t *anchor_delta_pos,
                               kvcomm_tensor out_k, kvcomm_tensor out_v, void *stream)
{
    kvcomm_align_job job{};
    job.base_k = base_k;
    job.base_v = base_v;
    job.out_k = out_k;
    job.out_v = out_v;
    job.seg_len = seg_len;
    job.delta_pos = delta_pos;
    job.anchor_dk = anchor_dk;
    job.anchor_dv = anchor_dv;
    job.anchor_len = anchor_len;
    job.anchor_delta_pos = anchor_delta_pos;
    job.n_anchors = n_anchors;
    job.weights = weights;
    job.weights_slots = check_model(model) || check_gran(gran) ? 0 : (int64_t)kvcomm_weight_slots(model, seg_len, gran);
    return kvcomm_align_kv_batch(model, gran, anchor_layout, &job, 1, stream);
}
