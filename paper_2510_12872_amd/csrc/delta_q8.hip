// Compressed anchor deviations: one byte per element in the OCP 8-bit floating-point format E4M3 times a
// power-of-two scale per tensor (the appendix on memory cost notes that the deviation tensors are small
// in magnitude and names their compression as future work).  The stored deviations are 2 * A of the
// 2 * (A + 2) rows the offset approximation moves per (layer, head, token), so halving them cuts the
// HBM traffic of that step from 2*D*es*(A+2) to D*(4*es + 2*A) bytes per row (40 % less for bf16, A = 8).
//   kvcomm_quantize_deltas   stored deviation (model dtype) -> E4M3 bytes: x / scale rounded to nearest even,
//                            saturating at +-448 (lossy: relative error <= 2^-4 above scale * 2^-6);
//   kvcomm_align_kv_q8       kvcomm_align_kv reading E4M3 deviations; the scale is folded into the anchor
//                            weight, so the inner loop is that of the uncompressed kernel plus the unpacking.
// gfx950's v_cvt_pk_f32_fp8 / v_cvt_pk_fp8_f32 implement exactly this format; the encoder clamps first, so
// the hardware's own overflow behaviour never matters.
#include "align_common.h"

namespace {

using namespace kvc;

#ifndef KVC_ALIGNQ8_BLOCKS
#define KVC_ALIGNQ8_BLOCKS 2048   // blocks per tensor and segment the grid of the compressed update aims at
#endif

#ifndef KVC_ALIGNQ8_WPE
#define KVC_ALIGNQ8_WPE 4   // wavefronts per SIMD the register budget is sized for
#endif
#ifndef KVC_ALIGNQ8_INFLIGHT
#define KVC_ALIGNQ8_INFLIGHT 2   // anchors loaded together (twice that in flight: two stages); 4 spills at this budget
#endif

constexpr int kBlock = kAlignBlock;
constexpr int kQ8InFlight = KVC_ALIGNQ8_INFLIGHT;

// EPV consecutive E4M3 bytes -> floats.
template <int EPV>
__device__ __forceinline__ void unpack_q8(const uint32_t (&raw)[EPV / 4], float (&out)[EPV])
{
#pragma unroll
    for (int w = 0; w < EPV / 4; ++w) {
        const f32x2 a = __builtin_amdgcn_cvt_pk_f32_fp8(raw[w], false);
        const f32x2 b = __builtin_amdgcn_cvt_pk_f32_fp8(raw[w], true);
        out[4 * w] = a[0];
        out[4 * w + 1] = a[1];
        out[4 * w + 2] = b[0];
        out[4 * w + 3] = b[1];
    }
}

// Deviation bytes of one anchor for this lane's channels of both halves.
// 16-bit rows (8 channels per lane and half = 8 bytes each): instead of two 8-byte loads per lane, the two
// lanes of a pair load 16 bytes each -- the even lane the pair's 16 channels of the first half, the odd lane
// those of the second half -- and swap the halves they do not own with one DPP move per register (quad
// permutation 1,0,3,2): half as many load instructions for the same bytes.
// fp32 rows (4 channels per lane and half): two 4-byte loads.
// `row` points at the anchor's bytes of this token, `lir` is the lane's index in the row.
template <int EPV>
struct Q8Raw;
template <>
struct Q8Raw<8> {
    u32x4 raw;
    __device__ __forceinline__ void load(const uint8_t *row, int lir, int half_bytes)
    {
        raw = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(row + 8 * (lir & ~1) + ((lir & 1) ? half_bytes : 0)));
    }
    __device__ __forceinline__ void split(int lir, uint32_t (&lo)[2], uint32_t (&hi)[2]) const
    {
        // even lane holds [lo_even, lo_odd], odd lane holds [hi_even, hi_odd] (8 bytes each)
        const bool odd = lir & 1;
        const uint32_t s0 = odd ? raw[0] : raw[2];   // what the partner needs: even sends lo_odd, odd sends hi_even
        const uint32_t s1 = odd ? raw[1] : raw[3];
        const uint32_t g0 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)s0, 0xB1, 0xf, 0xf, true);
        const uint32_t g1 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)s1, 0xB1, 0xf, 0xf, true);
        lo[0] = odd ? g0 : raw[0];
        lo[1] = odd ? g1 : raw[1];
        hi[0] = odd ? raw[2] : g0;
        hi[1] = odd ? raw[3] : g1;
    }
};
template <>
struct Q8Raw<4> {
    uint32_t raw[2];
    __device__ __forceinline__ void load(const uint8_t *row, int lir, int half_bytes)
    {
        raw[0] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(row + 4 * lir));
        raw[1] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(row + 4 * lir + half_bytes));
    }
    __device__ __forceinline__ void split(int, uint32_t (&lo)[1], uint32_t (&hi)[1]) const
    {
        lo[0] = raw[0];
        hi[0] = raw[1];
    }
};

// ------------------------------------------------------------------------------ quantise
struct QuantParams {
    const void *in;
    uint8_t *out;
    Strides s_in, s_out;
    int32_t H, S, LH, n_token_tiles;
    float inv_scale;
};

#ifndef KVC_QUANT_ROWS
#define KVC_QUANT_ROWS 4   // rows per thread: that many independent 16-byte loads in flight
#endif

template <typename T, int LPR>  // LPR lanes per row, each EPV elements
__global__ __launch_bounds__(kBlock) void quantize_kernel(const QuantParams p)
{
    constexpr int EPV = Elem<T>::EPV;
    constexpr int RPB = kBlock / LPR;
    constexpr int U = KVC_QUANT_ROWS;
    const int row = threadIdx.x / LPR, lir = threadIdx.x % LPR;
    const int tile = blockIdx.x % p.n_token_tiles;   // a tile is U * RPB consecutive tokens
    const int lh = blockIdx.x / p.n_token_tiles;
    const int l = lh / p.H, h = lh % p.H;
    const T *xb = static_cast<const T *>(p.in) + l * p.s_in.layer + h * p.s_in.head + lir * EPV;
    uint8_t *yb = p.out + l * p.s_out.layer + h * p.s_out.head + lir * EPV;
    u32x4 raw[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int t = (tile * U + u) * RPB + row;
        if (t < p.S) raw[u] = load16_stream(xb + t * p.s_in.token);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int t = (tile * U + u) * RPB + row;
        if (t >= p.S) continue;
        float x[EPV];
        unpack<T>(raw[u], x);
        uint32_t w[EPV / 4];
#pragma unroll
        for (int i = 0; i < EPV / 4; ++i) {
            // The clamp (maximum / minimum by number) turns a NaN into a bound, so NaN inputs are patched
            // afterwards: their code is 0x7f, the format's NaN, whatever the sign.
            float c[4];
            uint32_t nan_bytes = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float v = x[4 * i + e] * p.inv_scale;
                c[e] = fminf(fmaxf(v, -448.f), 448.f);
                nan_bytes |= v != v ? 0xffu << (8 * e) : 0u;
            }
            int packed = 0;
            packed = __builtin_amdgcn_cvt_pk_fp8_f32(c[0], c[1], packed, false);
            packed = __builtin_amdgcn_cvt_pk_fp8_f32(c[2], c[3], packed, true);
            w[i] = ((uint32_t)packed & ~nan_bytes) | (0x7f7f7f7fu & nan_bytes);
        }
        uint8_t *yp = yb + t * p.s_out.token;
        if constexpr (EPV == 8) {
            const u32x2 v = {w[0], w[1]};
            __builtin_nontemporal_store(v, reinterpret_cast<u32x2 *>(yp));
        } else {
            __builtin_nontemporal_store(w[0], reinterpret_cast<uint32_t *>(yp));
        }
    }
}

// --------------------------------------------------------------------------------- align
// Same launch-wide layout as the uncompressed update (per-segment descriptors, selected anchors and rotation
// tables of all segments in the kernel arguments); a deviation's power-of-two scale travels as its exponent.
struct AlignQ8Params {
    AlignJob job[KVCOMM_MAX_BATCH];
    Strides s_anc;             // in bytes (= elements of the E4M3 tensors)
    int32_t H, LH;
    int32_t gran, n_jobs;
    int32_t lh_per_block;
    int32_t tiles_total;
    int32_t tab_delta[kMaxTab];
    const void *anc[2][KVCOMM_MAX_ANCHORS];
    int8_t scale_exp[2][KVCOMM_MAX_ANCHORS];   // [0] key, [1] value deviation scale = 2^scale_exp of a selected anchor
    uint8_t col[KVCOMM_MAX_ANCHORS];
    uint8_t tab[KVCOMM_MAX_ANCHORS];
    double inv_freq[kMaxHalf];
};
static_assert(sizeof(AlignQ8Params) <= 4096, "kernel arguments are limited to 4 KB");

__device__ __forceinline__ float pow2f(int e) { return __uint_as_float((uint32_t)(e + 127) << 23); }  // -126 <= e <= 127

// Work split as in align_kernel: LPR = D / (2 * EPV) lanes per row, lane r owns channels [r*EPV, r*EPV+EPV)
// of both halves; a block is 256 / LPR tokens of a run of (layer, head) pairs of ONE tensor of one segment.
template <typename T, int LPR>
__global__ __launch_bounds__(kBlock, KVC_ALIGNQ8_WPE) void align_q8_kernel(const AlignQ8Params p)
{
    constexpr int EPV = Elem<T>::EPV;
    constexpr int HALF = LPR * EPV;
    constexpr int RPB = kBlock / LPR;

    const int chunk = blockIdx.x / p.tiles_total;
    const int r = blockIdx.x % p.tiles_total;
    const AlignJob &jb = p.job[job_of_tile(p, r)];
    const int n_sel = jb.n_sel, a0 = jb.a0;

    extern __shared__ __align__(16) unsigned char smem_raw[];
    float2 *cs = reinterpret_cast<float2 *>(smem_raw);                         // [n_tab][HALF]
    float *w_lds = reinterpret_cast<float *>(smem_raw) + 2 * jb.n_tab * HALF;  // [RPB][n_sel], scale folded in

    const int tid = threadIdx.x;
    const int row = tid / LPR, lir = tid % LPR;
    const int tile = r - jb.tile0;
    const int which = blockIdx.y;
    const bool is_k = which == 0;
    const int t = tile * RPB + row;
    const bool valid = t < jb.S;
    const int lh0 = chunk * p.lh_per_block;
    const int lh1 = min(lh0 + p.lh_per_block, p.LH);

    if (is_k)
        for (int idx = tid; idx < jb.n_tab * HALF; idx += kBlock)
            cs[idx] = rope_cos_sin(p.tab_delta[jb.t0 + idx / HALF], p.inv_freq[idx % HALF]);
    if (p.gran != KVCOMM_W_LAYER_HEAD_TOKEN) {
        for (int idx = tid; idx < RPB * n_sel; idx += kBlock) {
            const int rr = idx / n_sel, a = idx % n_sel;
            const int tt = tile * RPB + rr;
            const int64_t slot = p.gran == KVCOMM_W_TOKEN ? tt : 0;
            w_lds[idx] = tt < jb.S ? jb.weights[slot * jb.w_pitch + p.col[a0 + a]] * pow2f(p.scale_exp[which][a0 + a]) : 0.f;
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
    auto anchor_row = [&](int a) { return static_cast<const uint8_t *>(p.anc[which][a0 + a]); };

    // What one (layer, head) pair needs first: the base row and the first kQ8InFlight anchors.  The loads of
    // the next pair are issued before the arithmetic of the current one (registers double-buffered).
    struct Stage {
        u32x4 rlo, rhi;
        Q8Raw<EPV> x[kQ8InFlight];
    };
    auto anchor_off = [&](int lh) {
        const int l = lh / p.H, h = lh % p.H;
        return l * p.s_anc.layer + h * p.s_anc.head + t * p.s_anc.token;
    };
    auto issue = [&](int lh, Stage &st) {
        const int l = lh / p.H, h = lh % p.H;
        const T *xp = bp + l * sb.layer + h * sb.head + t * sb.token + col0;
        st.rlo = load16_stream(xp);
        st.rhi = load16_stream(xp + HALF);
        const int64_t roff = anchor_off(lh);
#pragma unroll
        for (int u = 0; u < kQ8InFlight; ++u)
            if (u < n_sel) st.x[u].load(anchor_row(u) + roff, lir, HALF);
    };

    Stage cur;
    issue(lh0, cur);
    for (int lh = lh0; lh < lh1; ++lh) {
        const int l = lh / p.H, h = lh % p.H;
        Stage nxt;
        if (lh + 1 < lh1) issue(lh + 1, nxt);
        const float *wrow = p.gran == KVCOMM_W_LAYER_HEAD_TOKEN ? jb.weights + ((int64_t)lh * jb.S + t) * jb.w_pitch : nullptr;

        float lo[EPV], hi[EPV];
        unpack<T>(cur.rlo, lo);
        unpack<T>(cur.rhi, hi);
        if (rot_base) {
#pragma unroll
            for (int e = 0; e < EPV; ++e) {
                const float a = lo[e], b = hi[e];
                lo[e] = a * bc[e] - b * bs[e];
                hi[e] = b * bc[e] + a * bs[e];
            }
        }
        auto accumulate = [&](int a, const Q8Raw<EPV> &raw) {
            uint32_t rdlo[EPV / 4], rdhi[EPV / 4];
            raw.split(lir, rdlo, rdhi);
            const float w = wrow ? wrow[p.col[a0 + a]] * pow2f(p.scale_exp[which][a0 + a]) : w_lds[row * n_sel + a];
            float dlo[EPV], dhi[EPV];
            unpack_q8<EPV>(rdlo, dlo);
            unpack_q8<EPV>(rdhi, dhi);
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
#pragma unroll
        for (int u = 0; u < kQ8InFlight; ++u)
            if (u < n_sel) accumulate(u, cur.x[u]);
        // further anchors: kQ8InFlight at a time
        const int64_t roff = anchor_off(lh);
        int a = kQ8InFlight;
        for (; a + kQ8InFlight <= n_sel; a += kQ8InFlight) {
            Q8Raw<EPV> x[kQ8InFlight];
#pragma unroll
            for (int u = 0; u < kQ8InFlight; ++u) x[u].load(anchor_row(a + u) + roff, lir, HALF);
#pragma unroll
            for (int u = 0; u < kQ8InFlight; ++u) accumulate(a + u, x[u]);
        }
        for (; a < n_sel; ++a) {
            Q8Raw<EPV> x;
            x.load(anchor_row(a) + roff, lir, HALF);
            accumulate(a, x);
        }
        T *yp = op + l * so.layer + h * so.head + t * so.token + col0;
        store16_stream(yp, pack<T>(lo));
        store16_stream(yp + HALF, pack<T>(hi));
        cur = nxt;   // (indeterminate after the last pair, and unused)
    }
}

template <typename T, int LPR>
int launch_align_q8(const AlignQ8Params &p, int n_blocks, int max_tab, int max_sel, hipStream_t stream)
{
    constexpr int HALF = LPR * Elem<T>::EPV;
    constexpr int RPB = kBlock / LPR;
    const size_t lds = sizeof(float2) * (size_t)max_tab * HALF + sizeof(float) * (size_t)RPB * max_sel;
    return launch(align_q8_kernel<T, LPR>, dim3(n_blocks, 2), dim3(kBlock), lds, stream, p);
}

// Byte tensors: pointer 16-byte aligned, strides multiples of 16 bytes.
int check_tensor_q8(const kvcomm_tensor &t, bool need_ptr)
{
    if (need_ptr && (!t.ptr || !aligned16(t.ptr))) return KVCOMM_EINVAL;
    if (t.stride_layer < 0 || t.stride_head < 0 || t.stride_token < 0) return KVCOMM_EINVAL;
    if (t.stride_layer % 16 || t.stride_head % 16 || t.stride_token % 16) return KVCOMM_EINVAL;
    return KVCOMM_OK;
}

// s = 2^e with -126 <= e <= 127 (a normal power of two)?  Writes e.
bool power_of_two(float s, int *exp_out = nullptr)
{
    if (!(s > 0.f) || !isfinite(s)) return false;
    int e;
    if (frexpf(s, &e) != 0.5f || e - 1 < -126) return false;
    if (exp_out) *exp_out = e - 1;
    return true;
}

}  // namespace

extern "C" int kvcomm_quantize_deltas(const kvcomm_model *model, kvcomm_tensor in, int32_t n_tokens, float scale,
                                      kvcomm_tensor out, void *stream)
{
    int st = check_model(model);
    if (st) return st;
    if (n_tokens <= 0 || !power_of_two(scale)) return KVCOMM_EINVAL;
    const int dt = model->dtype;
    if ((st = check_tensor(in, dt, true)) || (st = check_tensor_q8(out, true))) return st;
    QuantParams p{};
    p.in = in.ptr;
    p.out = static_cast<uint8_t *>(out.ptr);
    p.s_in = strides_of(in);
    p.s_out = strides_of(out);
    p.H = model->n_kv_heads;
    p.S = n_tokens;
    p.LH = model->n_layers * model->n_kv_heads;
    p.inv_scale = 1.f / scale;
    const int lpr = model->head_dim / (16 / elem_size(dt));
    const int rpb = (kBlock / lpr) * KVC_QUANT_ROWS;   // tokens per block
    p.n_token_tiles = (n_tokens + rpb - 1) / rpb;
    const int64_t n_blocks = (int64_t)p.n_token_tiles * p.LH;
    if (n_blocks > 0x7fffffff) return KVCOMM_EUNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(stream);
    st = KVCOMM_EUNSUPPORTED;
    if (dt == KVCOMM_BF16) {
        switch (lpr) {
            case 8: return launch(quantize_kernel<bf16_t, 8>, dim3((unsigned)n_blocks), dim3(kBlock), 0, s, p);
            case 16: return launch(quantize_kernel<bf16_t, 16>, dim3((unsigned)n_blocks), dim3(kBlock), 0, s, p);
            case 32: return launch(quantize_kernel<bf16_t, 32>, dim3((unsigned)n_blocks), dim3(kBlock), 0, s, p);
        }
    } else {
        switch (lpr) {
            case 16: return launch(quantize_kernel<float, 16>, dim3((unsigned)n_blocks), dim3(kBlock), 0, s, p);
            case 32: return launch(quantize_kernel<float, 32>, dim3((unsigned)n_blocks), dim3(kBlock), 0, s, p);
            case 64: return launch(quantize_kernel<float, 64>, dim3((unsigned)n_blocks), dim3(kBlock), 0, s, p);
        }
    }
    return st;
}

extern "C" int kvcomm_align_kv_q8_batch(const kvcomm_model *model, int32_t gran, kvcomm_tensor anchor_layout,
                                        const kvcomm_align_q8_job *jobs, int32_t n_jobs, void *stream)
{
    AlignQ8Params p{};
    AlignLaunch pl{};
    for (int j = 0; jobs && j < n_jobs && j < KVCOMM_MAX_BATCH; ++j)
        if (jobs[j].n_anchors > 0 && (!jobs[j].anchor_scale_k || !jobs[j].anchor_scale_v)) return KVCOMM_EINVAL;
    int st = plan_align(model, gran, anchor_layout, 1, jobs, n_jobs, KVC_ALIGNQ8_BLOCKS, p, pl,
                        [&p](int slot, const kvcomm_align_q8_job &jd, int a) {
                            int ek, ev;
                            if (!power_of_two(jd.anchor_scale_k[a], &ek) || !power_of_two(jd.anchor_scale_v[a], &ev))
                                return (int)KVCOMM_EINVAL;
                            p.scale_exp[0][slot] = (int8_t)ek;
                            p.scale_exp[1][slot] = (int8_t)ev;
                            return (int)KVCOMM_OK;
                        });
    if (st) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int nb = (int)pl.n_blocks;
    if (model->dtype == KVCOMM_BF16) {
        switch (pl.lpr) {
            case 4: return launch_align_q8<bf16_t, 4>(p, nb, pl.max_tab, pl.max_sel, s);
            case 8: return launch_align_q8<bf16_t, 8>(p, nb, pl.max_tab, pl.max_sel, s);
            case 16: return launch_align_q8<bf16_t, 16>(p, nb, pl.max_tab, pl.max_sel, s);
        }
    } else {
        switch (pl.lpr) {
            case 8: return launch_align_q8<float, 8>(p, nb, pl.max_tab, pl.max_sel, s);
            case 16: return launch_align_q8<float, 16>(p, nb, pl.max_tab, pl.max_sel, s);
            case 32: return launch_align_q8<float, 32>(p, nb, pl.max_tab, pl.max_sel, s);
        }
    }
    return KVCOMM_EUNSUPPORTED;
}

extern "C" int kvcomm_align_kv_q8(const kvcomm_model *model, int32_t gran, kvcomm_tensor base_k, kvcomm_tensor base_v,
                                  int32_t seg_len, const void *const *anchor_dk, const void *const *anchor_dv,
                                  kvcomm_tensor anchor_layout, const int32_t *anchor_len, const float *anchor_scale_k,
                                  const float *anchor_scale_v, int32_t n_anchors, const float *weights,
                                  int32_t delta_pos, const int32_t *anchor_delta_pos, kvcomm_tensor out_k,
                                  kvcomm_tensor out_v, void *stream)
{
    kvcomm_align_q8_job job{};
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
    job.anchor_scale_k = anchor_scale_k;
    job.anchor_scale_v = anchor_scale_v;
    job.n_anchors = n_anchors;
    job.weights = weights;
    job.weights_slots = check_model(model) || check_gran(gran) ? 0 : (int64_t)kvcomm_weight_slots(model, seg_len, gran);
    return kvcomm_align_kv_q8_batch(model, gran, anchor_layout, &job, 1, stream);
}
