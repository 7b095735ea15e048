// Host-side planning shared by the offset-approximation kernels (uncompressed and E4M3 deviations): the
// per-segment descriptors of a batched launch, the selection of anchors, the rotation tables, the cut into
// blocks and the aliasing rules of the boundary.  Device code only reads the structures filled here.
#pragma once

#include <math.h>

#include "kvcomm_device.h"

namespace kvc {

constexpr int kAlignBlock = 256;
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

// Which job a launch-wide tile index belongs to.
template <class P>
__device__ __forceinline__ int job_of_tile(const P &p, int r)
{
    int ji = 0;
#pragma unroll
    for (int i = 1; i < KVCOMM_MAX_BATCH; ++i)
        if (i < p.n_jobs && r >= p.job[i].tile0) ji = i;
    return ji;
}

struct AlignLaunch {
    int max_tab, max_sel, lpr;
    int64_t n_blocks;
};

// What a launch writes must not be something it also reads or writes elsewhere: an output may be exactly its
// own base tensor (in place: a lane owns both members of every rotation pair it touches), anything else that
// shares bytes with an output is an argument error.  Also checks that every job's weight buffer has the rows
// its own segment length asks for.  `anchor_es` = bytes per stored deviation element.
template <class JobT>
int check_align_aliasing(const kvcomm_model *model, int gran, const kvcomm_tensor &anchor_layout, int anchor_es,
                         const JobT *jobs, int n_jobs)
{
    const int L = model->n_layers, H = model->n_kv_heads, D = model->head_dim, es = elem_size(model->dtype);
    Extent out[KVCOMM_MAX_BATCH][2], base[KVCOMM_MAX_BATCH][2];
    for (int j = 0; j < n_jobs; ++j) {
        const JobT &jd = jobs[j];
        out[j][0] = extent_of(jd.out_k, L, H, jd.seg_len, D, es);
        out[j][1] = extent_of(jd.out_v, L, H, jd.seg_len, D, es);
        base[j][0] = extent_of(jd.base_k, L, H, jd.seg_len, D, es);
        base[j][1] = extent_of(jd.base_v, L, H, jd.seg_len, D, es);
        if (jd.n_anchors > 0 && jd.weights_slots != (int64_t)kvcomm_weight_slots(model, jd.seg_len, gran)) return KVCOMM_EINVAL;
    }
    for (int j = 0; j < n_jobs; ++j) {
        if (extents_overlap(out[j][0], out[j][1])) return KVCOMM_EINVAL;
        for (int w = 0; w < 2; ++w) {
            const Extent &o = out[j][w];
            for (int i = 0; i < n_jobs; ++i) {
                const JobT &ji = jobs[i];
                for (int v = 0; v < 2; ++v) {
                    const bool own_base = i == j && v == w;
                    if (!(own_base && same_extent(o, base[i][v])) && extents_overlap(o, base[i][v])) return KVCOMM_EINVAL;
                    if (i > j && extents_overlap(o, out[i][v])) return KVCOMM_EINVAL;
                }
                for (int a = 0; a < ji.n_anchors; ++a) {
                    if (ji.anchor_len[a] < ji.seg_len) continue;   // never read
                    if (extents_overlap(o, extent_of(ji.anchor_dk[a], anchor_layout, L, H, ji.seg_len, D, anchor_es)) ||
                        extents_overlap(o, extent_of(ji.anchor_dv[a], anchor_layout, L, H, ji.seg_len, D, anchor_es)))
                        return KVCOMM_EINVAL;
                }
                if (ji.n_anchors > 0 &&
                    extents_overlap(o, extent_flat(ji.weights, sizeof(float) * (size_t)ji.weights_slots * ji.n_anchors)))
                    return KVCOMM_EINVAL;
            }
        }
    }
    return KVCOMM_OK;
}

// Validates the jobs of a batched update and fills the launch parameters P (fields job, s_anc, H, LH, gran,
// n_jobs, lh_per_block, tiles_total, tab_delta, anc, col, tab, inv_freq).  `on_anchor(slot, job, a)` is called
// for every selected anchor with its launch-wide slot and may return an error status.
template <class P, class JobT, class OnAnchor>
int plan_align(const kvcomm_model *model, int gran, const kvcomm_tensor &anchor_layout, int anchor_es, const JobT *jobs,
               int n_jobs, int target_blocks_per_job, P &p, AlignLaunch &plan, OnAnchor &&on_anchor)
{
    int st = check_model(model);
    if (st) return st;
    if ((st = check_gran(gran))) return st;
    if (!jobs || n_jobs <= 0) return KVCOMM_EINVAL;
    if (n_jobs > KVCOMM_MAX_BATCH) return KVCOMM_EUNSUPPORTED;
    const int dt = model->dtype;
    bool any_anchor = false;
    for (int j = 0; j < n_jobs; ++j) {
        const JobT &jd = jobs[j];
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
    if (any_anchor) {
        // rows of the stored deviations move in 16-byte pieces whatever their element size
        if (anchor_layout.stride_layer < 0 || anchor_layout.stride_head < 0 || anchor_layout.stride_token < 0) return KVCOMM_EINVAL;
        const int64_t epv = 16 / anchor_es;
        if (anchor_layout.stride_layer % epv || anchor_layout.stride_head % epv || anchor_layout.stride_token % epv)
            return KVCOMM_EINVAL;
    }
    if ((st = check_align_aliasing(model, gran, anchor_layout, anchor_es, jobs, n_jobs))) return st;

    p.s_anc = strides_of(anchor_layout);
    p.H = model->n_kv_heads;
    p.LH = model->n_layers * model->n_kv_heads;
    p.gran = gran;
    p.n_jobs = n_jobs;
    for (int i = 0; i < model->head_dim / 2; ++i)
        p.inv_freq[i] = pow(model->rope_theta, -2.0 * (double)i / (double)model->head_dim);

    const int es = elem_size(dt);
    const int lpr = model->head_dim / (2 * (16 / es));
    const int rpb = kAlignBlock / lpr;
    int n_tab_total = 0, n_sel_total = 0, max_tab = 0, max_sel = 0;
    int64_t tiles_total = 0;
    for (int j = 0; j < n_jobs; ++j) {
        const JobT &jd = jobs[j];
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
            if ((st = on_anchor(s, jd, a))) return st;
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
    const int64_t target_blocks = (int64_t)target_blocks_per_job * n_jobs;
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
    plan.n_blocks = n_chunks * tiles_total;
    plan.max_tab = max_tab;
    plan.max_sel = max_sel;
    plan.lpr = lpr;
    if (plan.n_blocks > 0x7fffffff) return KVCOMM_EUNSUPPORTED;
    return KVCOMM_OK;
}

}  // namespace kvc
