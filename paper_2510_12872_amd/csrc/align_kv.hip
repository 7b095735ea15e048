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
// 256 threads owns a tile of 256/LPR consecutive tokens and walks over a chunk of
// (layer, head) pairs; its per-token anchor weights and the cos/sin tables therefore
// load once per block (LDS) and every access to a tensor is a run of whole 128-byte lines.
#include <math.h>

#include "kvcomm_device.h"

namespace {

using namespace kvc;

constexpr int kBlock = 256;
constexpr int kMaxTab = KVCOMM_MAX_ANCHORS + 1;

struct AlignParams {
    const void *base_k, *base_v;
    void *out_k, *out_v;
    Strides s_bk, s_bv, s_ok, s_ov, s_anc;
    const float *weights;
    int32_t H, S, LH;          // kv heads, tokens, layers*heads
    int32_t w_pitch;           // anchors per weight row (n_anchors of the call)
    int32_t n_sel;             // selected anchors (compacted below)
    int32_t gran;
    int32_t lh_per_block, n_token_tiles;
    int32_t n_tab;             // rotation tables built per block
    int32_t base_tab;          // table of the base keys' rotation + 1, 0 = identity
    double log2_theta;
    int32_t tab_delta[kMaxTab];                 // position delta of each table
    const void *dk[KVCOMM_MAX_ANCHORS];         // selected anchors, original order
    const void *dv[KVCOMM_MAX_ANCHORS];
    uint8_t col[KVCOMM_MAX_ANCHORS];            // weight column of selected anchor
    uint8_t tab[KVCOMM_MAX_ANCHORS];            // its rotation table + 1, 0 = identity
};

template <typename T, int LPR>
__global__ __launch_bounds__(kBlock) void align_kernel(const AlignParams p)
{
    constexpr int EPV = Elem<T>::EPV;
    constexpr int HALF = LPR * EPV;  // D / 2
    constexpr int RPB = kBlock / LPR;

    extern __shared__ __align__(16) unsigned char smem_raw[];
    float2 *cs = reinterpret_cast<float2 *>(smem_raw);                          // [n_tab][HALF] (cos, sin)
    float *w_lds = reinterpret_cast<float *>(smem_raw) + 2 * p.n_tab * HALF;    // [RPB][n_sel]

    const int tid = threadIdx.x;
    const int row = tid / LPR;
    const int lir = tid % LPR;
    const int tile = blockIdx.x % p.n_token_tiles;
    const int chunk = blockIdx.x / p.n_token_tiles;
    const int t = tile * RPB + row;
    const bool valid = t < p.S;
    const int lh0 = chunk * p.lh_per_block;
    const int lh1 = min(lh0 + p.lh_per_block, p.LH);

    // cos/sin of delta * theta^(-2i/D): angle and reduction in double, stored as fp32.
    for (int idx = tid; idx < p.n_tab * HALF; idx += kBlock) {
        const int r = idx / HALF, i = idx % HALF;
        const double freq = exp2(-((double)i / (double)HALF) * p.log2_theta);
        double s, c;
        sincos((double)p.tab_delta[r] * freq, &s, &c);
        cs[idx] = make_float2((float)c, (float)s);
    }
    if (p.gran != KVCOMM_W_LAYER_HEAD_TOKEN) {
        for (int idx = tid; idx < RPB * p.n_sel; idx += kBlock) {
            const int r = idx / p.n_sel, a = idx % p.n_sel;
            const int tt = tile * RPB + r;
            const int64_t slot = p.gran == KVCOMM_W_TOKEN ? tt : 0;
            w_lds[idx] = tt < p.S ? p.weights[slot * p.w_pitch + p.col[a]] : 0.f;
        }
    }
    __syncthreads();
    if (!valid) return;

    float bc[EPV], bs[EPV];
    if (p.base_tab) {
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
            const float2 v = cs[(p.base_tab - 1) * HALF + lir * EPV + e];
            bc[e] = v.x;
            bs[e] = v.y;
        }
    }

    const T *bk = static_cast<const T *>(p.base_k);
    const T *bv = static_cast<const T *>(p.base_v);
    T *ok = static_cast<T *>(p.out_k);
    T *ov = static_cast<T *>(p.out_v);
    const int64_t col0 = (int64_t)lir * EPV;

    for (int lh = lh0; lh < lh1; ++lh) {
        const int l = lh / p.H, h = lh % p.H;
        const T *kp = bk + l * p.s_bk.layer + h * p.s_bk.head + t * p.s_bk.token + col0;
        const T *vp = bv + l * p.s_bv.layer + h * p.s_bv.head + t * p.s_bv.token + col0;
        const u32x4 rklo = load16_stream(kp), rkhi = load16_stream(kp + HALF);
        const u32x4 rvlo = load16_stream(vp), rvhi = load16_stream(vp + HALF);
        const int64_t aoff = l * p.s_anc.layer + h * p.s_anc.head + t * p.s_anc.token + col0;
        const float *wrow = p.gran == KVCOMM_W_LAYER_HEAD_TOKEN
                                ? p.weights + ((int64_t)lh * p.S + t) * p.w_pitch
                                : nullptr;

        float klo[EPV], khi[EPV], vlo[EPV], vhi[EPV];
        unpack<T>(rklo, klo);
        unpack<T>(rkhi, khi);
        unpack<T>(rvlo, vlo);
        unpack<T>(rvhi, vhi);
        if (p.base_tab) {
#pragma unroll
            for (int e = 0; e < EPV; ++e) {
                const float a = klo[e], b = khi[e];
                klo[e] = a * bc[e] - b * bs[e];
                khi[e] = b * bc[e] + a * bs[e];
            }
        }

        // One anchor: 4 independent 16-byte loads; two anchors are kept in flight.
        auto accumulate = [&](int a, const u32x4 &rdklo, const u32x4 &rdkhi, const u32x4 &rdvlo, const u32x4 &rdvhi) {
            const float w = wrow ? wrow[p.col[a]] : w_lds[row * p.n_sel + a];
            float dklo[EPV], dkhi[EPV], dvlo[EPV], dvhi[EPV];
            unpack<T>(rdklo, dklo);
            unpack<T>(rdkhi, dkhi);
            unpack<T>(rdvlo, dvlo);
            unpack<T>(rdvhi, dvhi);
            const int tb = p.tab[a];
            if (tb) {
                const float2 *tcs = cs + (tb - 1) * HALF + lir * EPV;
#pragma unroll
                for (int e = 0; e < EPV; ++e) {
                    const float2 v = tcs[e];
                    const float x = dklo[e], y = dkhi[e];
                    dklo[e] = x * v.x - y * v.y;
                    dkhi[e] = y * v.x + x * v.y;
                }
            }
#pragma unroll
            for (int e = 0; e < EPV; ++e) {
                klo[e] += w * dklo[e];
                khi[e] += w * dkhi[e];
                vlo[e] += w * dvlo[e];
                vhi[e] += w * dvhi[e];
            }
        };

        int a = 0;
        for (; a + 2 <= p.n_sel; a += 2) {
            const T *dk0 = static_cast<const T *>(p.dk[a]) + aoff, *dv0 = static_cast<const T *>(p.dv[a]) + aoff;
            const T *dk1 = static_cast<const T *>(p.dk[a + 1]) + aoff, *dv1 = static_cast<const T *>(p.dv[a + 1]) + aoff;
            const u32x4 x0 = load16_stream(dk0), x1 = load16_stream(dk0 + HALF);
            const u32x4 x2 = load16_stream(dv0), x3 = load16_stream(dv0 + HALF);
            const u32x4 y0 = load16_stream(dk1), y1 = load16_stream(dk1 + HALF);
            const u32x4 y2 = load16_stream(dv1), y3 = load16_stream(dv1 + HALF);
            accumulate(a, x0, x1, x2, x3);
            accumulate(a + 1, y0, y1, y2, y3);
        }
        if (a < p.n_sel) {
            const T *dk0 = static_cast<const T *>(p.dk[a]) + aoff, *dv0 = static_cast<const T *>(p.dv[a]) + aoff;
            const u32x4 x0 = load16_stream(dk0), x1 = load16_stream(dk0 + HALF);
            const u32x4 x2 = load16_stream(dv0), x3 = load16_stream(dv0 + HALF);
            accumulate(a, x0, x1, x2, x3);
        }

        T *okp = ok + l * p.s_ok.layer + h * p.s_ok.head + t * p.s_ok.token + col0;
        T *ovp = ov + l * p.s_ov.layer + h * p.s_ov.head + t * p.s_ov.token + col0;
        store16_stream(okp, pack<T>(klo));
        store16_stream(okp + HALF, pack<T>(khi));
        store16_stream(ovp, pack<T>(vlo));
        store16_stream(ovp + HALF, pack<T>(vhi));
    }
}

template <typename T, int LPR>
int launch_align(const AlignParams &p, int n_blocks, hipStream_t stream)
{
    constexpr int HALF = LPR * Elem<T>::EPV;
    constexpr int RPB = kBlock / LPR;
    const size_t lds = sizeof(float2) * (size_t)p.n_tab * HALF + sizeof(float) * (size_t)RPB * p.n_sel;
    hipLaunchKernelGGL((align_kernel<T, LPR>), dim3(n_blocks), dim3(kBlock), lds, stream, p);
    return launch_status();
}

}  // namespace

extern "C" int kvcomm_align_kv(const kvcomm_model *model, int32_t gran, kvcomm_tensor base_k, kvcomm_tensor base_v,
                               int32_t seg_len, const void *const *anchor_dk, const void *const *anchor_dv,
                               kvcomm_tensor anchor_layout, const int32_t *anchor_len, int32_t n_anchors,
                               const float *weights, int32_t delta_pos, const int32_t *anchor_delta_pos,
                               kvcomm_tensor out_k, kvcomm_tensor out_v, void *stream)
{
    int st = check_model(model);
    if (st) return st;
    if ((st = check_gran(gran))) return st;
    if (seg_len <= 0 || n_anchors < 0) return KVCOMM_EINVAL;
    if (n_anchors > KVCOMM_MAX_ANCHORS) return KVCOMM_EUNSUPPORTED;
    const int dt = model->dtype;
    if ((st = check_tensor(base_k, dt, true)) || (st = check_tensor(base_v, dt, true)) ||
        (st = check_tensor(out_k, dt, true)) || (st = check_tensor(out_v, dt, true)))
        return st;
    if (n_anchors > 0) {
        if (!anchor_dk || !anchor_dv || !anchor_len || !weights) return KVCOMM_EINVAL;
        if ((st = check_tensor(anchor_layout, dt, false))) return st;
    }

    AlignParams p{};
    p.base_k = base_k.ptr;
    p.base_v = base_v.ptr;
    p.out_k = out_k.ptr;
    p.out_v = out_v.ptr;
    p.s_bk = strides_of(base_k);
    p.s_bv = strides_of(base_v);
    p.s_ok = strides_of(out_k);
    p.s_ov = strides_of(out_v);
    p.s_anc = strides_of(anchor_layout);
    p.weights = weights;
    p.H = model->n_kv_heads;
    p.S = seg_len;
    p.LH = model->n_layers * model->n_kv_heads;
    p.w_pitch = n_anchors;
    p.gran = gran;
    p.log2_theta = log2(model->rope_theta);

    // Rotation tables: one per distinct non-zero position delta (base keys: delta_pos;
    // anchor a's deviation: delta_pos - anchor_delta_pos[a]).
    auto table_of = [&](int32_t d) -> int {
        if (d == 0) return 0;
        for (int r = 0; r < p.n_tab; ++r)
            if (p.tab_delta[r] == d) return r + 1;
        p.tab_delta[p.n_tab] = d;
        return ++p.n_tab;
    };
    p.base_tab = table_of(delta_pos);
    for (int a = 0; a < n_anchors; ++a) {
        if (anchor_len[a] < 0) return KVCOMM_EINVAL;
        if (anchor_len[a] < seg_len) continue;  // not selected: never read
        if (!anchor_dk[a] || !anchor_dv[a] || !aligned16(anchor_dk[a]) || !aligned16(anchor_dv[a])) return KVCOMM_EINVAL;
        const int s = p.n_sel++;
        p.dk[s] = anchor_dk[a];
        p.dv[s] = anchor_dv[a];
        p.col[s] = (uint8_t)a;
        p.tab[s] = (uint8_t)(anchor_delta_pos ? table_of(delta_pos - anchor_delta_pos[a]) : 0);
    }

    const int es = elem_size(dt);
    const int lpr = model->head_dim / (2 * (16 / es));
    const int rpb = kBlock / lpr;
    p.n_token_tiles = (seg_len + rpb - 1) / rpb;
    // Enough blocks to fill 256 CUs several times over, while each block still walks a few
    // (layer, head) pairs so that its table / weight set-up is amortised.
    const int target_blocks = 4096;
    int n_chunks = (target_blocks + p.n_token_tiles - 1) / p.n_token_tiles;
    if (n_chunks > p.LH) n_chunks = p.LH;
    if (n_chunks < 1) n_chunks = 1;
    p.lh_per_block = (p.LH + n_chunks - 1) / n_chunks;
    n_chunks = (p.LH + p.lh_per_block - 1) / p.lh_per_block;
    const int n_blocks = n_chunks * p.n_token_tiles;
    hipStream_t s = static_cast<hipStream_t>(stream);

    if (dt == KVCOMM_BF16) {
        switch (lpr) {
            case 4: return launch_align<bf16_t, 4>(p, n_blocks, s);
            case 8: return launch_align<bf16_t, 8>(p, n_blocks, s);
            case 16: return launch_align<bf16_t, 16>(p, n_blocks, s);
        }
    } else {
        switch (lpr) {
            case 8: return launch_align<float, 8>(p, n_blocks, s);
            case 16: return launch_align<float, 16>(p, n_blocks, s);
            case 32: return launch_align<float, 32>(p, n_blocks, s);
        }
    }
    return KVCOMM_EUNSUPPORTED;
}
