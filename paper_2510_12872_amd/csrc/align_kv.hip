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

constexpr int kBlock = 256;
constexpr int kMaxTab = KVCOMM_MAX_ANCHORS + 1;
constexpr int kMaxHalf = 128;  // head_dim / 2 for the largest supported head_dim

struct AlignParams {
    const void *base[2];   // [0] keys, [1] values
    void *out[2];
    Strides s_base[2], s_out[2], s_anc;
    const float *weights;
    int32_t H, S, LH;          // kv heads, tokens, layers*heads
    int32_t w_pitch;           // anchors per weight row (n_anchors of the call)
    int32_t n_sel;             // selected anchors (compacted below)
    int32_t gran;
    int32_t lh_per_block, n_token_tiles;
    int32_t n_tab;             // rotation tables built per block
    int32_t base_tab;          // table of the base keys' rotation + 1, 0 = identity
    int32_t tab_delta[kMaxTab];                 // position delta of each table
    const void *anc[2][KVCOMM_MAX_ANCHORS];     // [0] dK, [1] dV of the selected anchors, original order
    uint8_t col[KVCOMM_MAX_ANCHORS];            // weight column of selected anchor
    uint8_t tab[KVCOMM_MAX_ANCHORS];            // its rotation table + 1, 0 = identity
    double inv_freq[kMaxHalf];                  // theta^(-2i/D), i < D/2
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
    const int which = blockIdx.y;          // 0 = keys (rotated), 1 = values
    const bool is_k = which == 0;
    const int t = tile * RPB + row;
    const bool valid = t < p.S;
    const int lh0 = chunk * p.lh_per_block;
    const int lh1 = min(lh0 + p.lh_per_block, p.LH);

    if (is_k) {
        // cos/sin of delta * theta^(-2i/D): product and reduction modulo 2*pi in double.
        for (int idx = tid; idx < p.n_tab * HALF; idx += kBlock) {
            const int r = idx / HALF, i = idx % HALF;
            cs[idx] = rope_cos_sin(p.tab_delta[r], p.inv_freq[i]);
        }
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

    const bool rot_base = is_k && p.base_tab != 0;
    float bc[EPV], bs[EPV];
    if (rot_base) {
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
            const float2 v = cs[(p.base_tab - 1) * HALF + lir * EPV + e];
            bc[e] = v.x;
            bs[e] = v.y;
        }
    }

    const T *bp = static_cast<const T *>(p.base[which]);
    T *op = static_cast<T *>(p.out[which]);
    const Strides sb = p.s_base[which], so = p.s_out[which];
    const int64_t col0 = (int64_t)lir * EPV;

    for (int lh = lh0; lh < lh1; ++lh) {
        const int l = lh / p.H, h = lh % p.H;
        const T *xp = bp + l * sb.layer + h * sb.head + t * sb.token + col0;
        const u32x4 rlo = load16_stream(xp), rhi = load16_stream(xp + HALF);
        const int64_t aoff = l * p.s_anc.layer + h * p.s_anc.head + t * p.s_anc.token + col0;
        const float *wrow = p.gran == KVCOMM_W_LAYER_HEAD_TOKEN
                                ? p.weights + ((int64_t)lh * p.S + t) * p.w_pitch
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
            const float w = wrow ? wrow[p.col[a]] : w_lds[row * p.n_sel + a];
            float dlo[EPV], dhi[EPV];
            unpack<T>(rdlo, dlo);
            unpack<T>(rdhi, dhi);
            const int tb = is_k ? p.tab[a] : 0;
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

        // Four anchors (eight independent 16-byte loads) are kept in flight.
        int a = 0;
        for (; a + 4 <= p.n_sel; a += 4) {
            u32x4 x[4][2];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const T *d = static_cast<const T *>(p.anc[which][a + u]) + aoff;
                x[u][0] = load16_stream(d);
                x[u][1] = load16_stream(d + HALF);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) accumulate(a + u, x[u][0], x[u][1]);
        }
        for (; a < p.n_sel; ++a) {
            const T *d = static_cast<const T *>(p.anc[which][a]) + aoff;
            const u32x4 x0 = load16_stream(d), x1 = load16_stream(d + HALF);
            accumulate(a, x0, x1);
        }

        T *yp = op + l * so.layer + h * so.head + t * so.token + col0;
        store16_stream(yp, pack<T>(lo));
        store16_stream(yp + HALF, pack<T>(hi));
    }
}

template <typename T, int LPR>
int launch_align(const AlignParams &p, int n_blocks, hipStream_t stream)
{
    constexpr int HALF = LPR * Elem<T>::EPV;
    constexpr int RPB = kBlock / LPR;
    const size_t lds = sizeof(float2) * (size_t)p.n_tab * HALF + sizeof(float) * (size_t)RPB * p.n_sel;
    hipLaunchKernelGGL((align_kernel<T, LPR>), dim3(n_blocks, 2), dim3(kBlock), lds, stream, p);
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
    p.base[0] = base_k.ptr;
    p.base[1] = base_v.ptr;
    p.out[0] = out_k.ptr;
    p.out[1] = out_v.ptr;
    p.s_base[0] = strides_of(base_k);
    p.s_base[1] = strides_of(base_v);
    p.s_out[0] = strides_of(out_k);
    p.s_out[1] = strides_of(out_v);
    p.s_anc = strides_of(anchor_layout);
    p.weights = weights;
    p.H = model->n_kv_heads;
    p.S = seg_len;
    p.LH = model->n_layers * model->n_kv_heads;
    p.w_pitch = n_anchors;
    p.gran = gran;
    for (int i = 0; i < model->head_dim / 2; ++i)
        p.inv_freq[i] = pow(model->rope_theta, -2.0 * (double)i / (double)model->head_dim);

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
        p.anc[0][s] = anchor_dk[a];
        p.anc[1][s] = anchor_dv[a];
        p.col[s] = (uint8_t)a;
        p.tab[s] = (uint8_t)(anchor_delta_pos ? table_of(delta_pos - anchor_delta_pos[a]) : 0);
    }

    const int es = elem_size(dt);
    const int lpr = model->head_dim / (2 * (16 / es));
    const int rpb = kBlock / lpr;
    p.n_token_tiles = (seg_len + rpb - 1) / rpb;
    // Many small blocks: the memory system delivers more with more wavefronts in flight, and the
    // per-block set-up (weights, cos/sin) is a few dozen instructions.
    const int target_blocks = 32768;
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
