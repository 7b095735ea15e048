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
#include <math.h>

#include "kvcomm_device.h"

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

constexpr int kBlock = 256;
constexpr int kAnchorsInFlight = KVC_ALIGN_INFLIGHT;
constexpr int kMaxTab = KVCOMM_MAX_ANCHORS + 1;
constexpr int kMaxHalf = 128;  // head_dim / 2 for the largest supported head_dim

// One segment of a launch.  A launch covers up to KVCOMM_MAX_BATCH segments (all placeholders of an
// agent, and the prefix segments that follow them, are independent and are updated "in parallel").
struct AlignJob {
    const void *base[2];   // [0] keys, [1] values
    void *out[2];
    Strides s_base[2], s_out[2];
    const float *weights;
    int32_t S;                 // tokens
    int32_t w_pitch;           // anchors per weight row (n_anchors of the segment)
    int32_t n_token_tiles;
    int32_t tile0;             // first of the segment's tiles in the launch-wide tile list
    int16_t a0, n_sel;         // its selected anchors: entries [a0, a0 + n_sel) of anc / col / tab
    int16_t t0, n_tab;         // its rotation tables: entries [t0, t0 + n_tab) of tab_delta
    int16_t base_tab;          // table of the base keys' rotation (index among the segment's tables) + 1, 0 = identity
    int16_t pad_;
};

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
    int ji = 0;
#pragma unroll
    for (int i = 1; i < KVCOMM_MAX_BATCH; ++i)
        if (i < p.n_jobs && r >= p.job[i].tile0) ji = i;
    const AlignJob &jb = p.job[ji];
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
    hipLaunchKernelGGL((align_kernel<T, LPR>), dim3(n_blocks, 2), dim3(kBlock), lds, stream, p);
    return launch_status();
}

}  // namespace

extern "C" int kvcomm_align_kv_batch(const kvcomm_model *model, int32_t gran, kvcomm_tensor anchor_layout,
                                     const kvcomm_align_job *jobs, int32_t n_jobs, void *stream)
{
    int st = check_model(model);
    if (st) return st;
    if ((st = check_gran(gran))) return st;
    if (!jobs || n_jobs <= 0) return KVCOMM_EINVAL;
    if (n_jobs > KVCOMM_MAX_BATCH) return KVCOMM_EUNSUPPORTED;
    const int dt = model->dtype;
    bool any_anchor = false;
    for (int j = 0; j < n_jobs; ++j) {
        const kvcomm_align_job &jd = jobs[j];
        if (jd.seg_len <= 0 || jd.n_anchors < 0) return KVCOMM_EINVAL;
        if (jd.n_anchors > KVCOMM_MAX_ANCHORS) return KVCOMM_EUNSUPPORTED;
        if ((st = check_tensor(jd.base_k, dt, true)) || (st = check_tensor(jd.base_v, dt, true)) ||
            (st = check_tensor(jd.out_k, dt, true)) || (st = check_tensor(jd.out_v, dt, true)))
            return st;
        if (jd.n_anchors > 0) {
            if (!jd.anchor_dk || !jd.anchor_dv || !jd.anchor_len || !jd.weights) return KVCOMM_EINVAL;
            any_anchor = true;
        }
    }
    if (any_anchor && (st = check_tensor(anchor_layout, dt, false))) return st;

    AlignParams p{};
    p.s_anc = strides_of(anchor_layout);
    p.H = model->n_kv_heads;
    p.LH = model->n_layers * model->n_kv_heads;
    p.gran = gran;
    p.n_jobs = n_jobs;
    for (int i = 0; i < model->head_dim / 2; ++i)
        p.inv_freq[i] = pow(model->rope_theta, -2.0 * (double)i / (double)model->head_dim);

    const int es = elem_size(dt);
    const int lpr = model->head_dim / (2 * (16 / es));
    const int rpb = kBlock / lpr;
    int n_tab_total = 0, n_sel_total = 0, max_tab = 0, max_sel = 0;
    int64_t tiles_total = 0;
    for (int j = 0; j < n_jobs; ++j) {
        const kvcomm_align_job &jd = jobs[j];
        AlignJob &jb = p.job[j];
        jb.base[0] = jd.base_k.ptr;
        jb.base[1] = jd.base_v.ptr;
        jb.out[0] = jd.out_k.ptr;
        jb.out[1] = jd.out_v.ptr;
        jb.s_base[0] = strides_of(jd.base_k);
        jb.s_base[1] = strides_of(jd.base_v);
        jb.s_out[0] = strides_of(jd.out_k);
        jb.s_out[1] = strides_of(jd.out_v);
        jb.weights = jd.weights;
        jb.S = jd.seg_len;
        jb.w_pitch = jd.n_anchors;
        jb.a0 = (int16_t)n_sel_total;
        jb.t0 = (int16_t)n_tab_total;
        // Rotation tables of the segment: one per distinct non-zero position delta (base keys: delta_pos;
        // anchor a's deviation: delta_pos - anchor_delta_pos[a]).
        int n_tab = 0;
        bool overflow = false;
        auto table_of = [&](int32_t d) -> int {
            if (d == 0) return 0;
            for (int r = 0; r < n_tab; ++r)
                if (p.tab_delta[n_tab_total + r] == d) return r + 1;
            if (n_tab_total + n_tab >= kMaxTab) {
                overflow = true;
                return 0;
            }
            p.tab_delta[n_tab_total + n_tab] = d;
            return ++n_tab;
        };
        jb.base_tab = (int16_t)table_of(jd.delta_pos);
        int n_sel = 0;
        for (int a = 0; a < jd.n_anchors; ++a) {
            if (jd.anchor_len[a] < 0) return KVCOMM_EINVAL;
            if (jd.anchor_len[a] < jd.seg_len) continue;  // not selected: never read
            if (!jd.anchor_dk[a] || !jd.anchor_dv[a] || !aligned16(jd.anchor_dk[a]) || !aligned16(jd.anchor_dv[a]))
                return KVCOMM_EINVAL;
            if (n_sel_total + n_sel >= KVCOMM_MAX_ANCHORS) return KVCOMM_EUNSUPPORTED;  // over all segments of the launch
            const int s = n_sel_total + n_sel++;
            p.anc[0][s] = jd.anchor_dk[a];
            p.anc[1][s] = jd.anchor_dv[a];
            p.col[s] = (uint8_t)a;
            p.tab[s] = (uint8_t)(jd.anchor_delta_pos ? table_of(jd.delta_pos - jd.anchor_delta_pos[a]) : 0);
        }
        if (overflow) return KVCOMM_EUNSUPPORTED;
        jb.n_sel = (int16_t)n_sel;
        jb.n_tab = (int16_t)n_tab;
        n_sel_total += n_sel;
        n_tab_total += n_tab;
        max_tab = n_tab > max_tab ? n_tab : max_tab;
        max_sel = n_sel > max_sel ? n_sel : max_sel;
        jb.n_token_tiles = (jd.seg_len + rpb - 1) / rpb;
        tiles_total += jb.n_token_tiles;
    }

    // Many small blocks: the memory system delivers more with more wavefronts in flight, and the
    // per-block set-up (weights, cos/sin) is a few dozen instructions.
    const int64_t target_blocks = (int64_t)KVC_ALIGN_BLOCKS * n_jobs;
    int64_t n_chunks = (target_blocks + tiles_total - 1) / tiles_total;
    if (n_chunks > p.LH) n_chunks = p.LH;
    if (n_chunks < 1) n_chunks = 1;
    p.lh_per_block = (int32_t)((p.LH + n_chunks - 1) / n_chunks);
    n_chunks = (p.LH + p.lh_per_block - 1) / p.lh_per_block;
    int32_t tile0 = 0;
    for (int j = 0; j < n_jobs; ++j) {
        p.job[j].tile0 = tile0;
        tile0 += p.job[j].n_token_tiles;
    }
    p.tiles_total = (int32_t)tiles_total;
    const int64_t n_blocks = n_chunks * tiles_total;
    if (n_blocks > 0x7fffffff) return KVCOMM_EUNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(stream);

    if (dt == KVCOMM_BF16) {
        switch (lpr) {
            case 4: return launch_align<bf16_t, 4>(p, (int)n_blocks, max_tab, max_sel, s);
            case 8: return launch_align<bf16_t, 8>(p, (int)n_blocks, max_tab, max_sel, s);
            case 16: return launch_align<bf16_t, 16>(p, (int)n_blocks, max_tab, max_sel, s);
        }
    } else {
        switch (lpr) {
            case 8: return launch_align<float, 8>(p, (int)n_blocks, max_tab, max_sel, s);
            case 16: return launch_align<float, 16>(p, (int)n_blocks, max_tab, max_sel, s);
            case 32: return launch_align<float, 32>(p, (int)n_blocks, max_tab, max_sel, s);
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
    return kvcomm_align_kv_batch(model, gran, anchor_layout, &job, 1, stream);
}
