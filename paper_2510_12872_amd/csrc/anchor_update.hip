// The add-anchor side of Algorithm 1, as far as it is arithmetic on cache tensors:
//   kvcomm_anchor_predict   Eq. "pred": entropy of the anchor weights against gamma * log |A_phi|,
//                           plus the length test;
//   kvcomm_capture_offsets  fallback branch: the offset between the real KV-cache of a dense
//                           generation and the re-positioned base cache fills a new anchor.
// capture_kernel is the mirror image of the align kernel (one streaming pass, HBM bound:
// four rows read and two written per (layer, head, token)); the prediction is two tiny kernels
// with fixed-order double sums.
#include <math.h>

#include "kvcomm_device.h"

namespace {

using namespace kvc;

constexpr int kBlock = 256;
constexpr int kMaxHalf = 128;
constexpr int kMaxPredictBlocks = 1024;

// ------------------------------------------------------------------------------ prediction
struct PredictParams {
    const float *weights;   // [n_slots, n_anchors]
    float *entropy_out;     // [n_slots] or null
    float *result_out;      // [2]
    double *partial;        // [n_blocks]
    int64_t n_slots, slots_per_block;
    int32_t n_anchors, n_sel, n_blocks, longer;
    double gamma;
    uint8_t is_sel[KVCOMM_MAX_ANCHORS];
};

// Fixed LDS tree over the 256 threads of a block; the total is returned to every thread.
__device__ __forceinline__ double block_sum(double v, double *red)
{
    const int tid = threadIdx.x;
    red[tid] = v;
    __syncthreads();
    for (int off = kBlock / 2; off >= 1; off >>= 1) {
        if (tid < off) red[tid] += red[tid + off];
        __syncthreads();
    }
    const double tot = red[0];
    __syncthreads();
    return tot;
}

// Block b owns the contiguous slot range [b * spb, (b+1) * spb); thread i adds the entropies of
// slots i, i + 256, ... of that range in increasing order.
__global__ __launch_bounds__(kBlock) void entropy_partial_kernel(const PredictParams p)
{
    __shared__ double red[kBlock];
    const int64_t lo = (int64_t)blockIdx.x * p.slots_per_block;
    const int64_t hi = min(lo + p.slots_per_block, p.n_slots);
    double s = 0.0;
    for (int64_t j = lo + threadIdx.x; j < hi; j += kBlock) {
        const float *w = p.weights + j * p.n_anchors;
        double h = 0.0;
        for (int a = 0; a < p.n_anchors; ++a) {
            const double x = (double)w[a];
            if (p.is_sel[a] && x > 0.0) h -= x * log(x);
        }
        if (p.entropy_out) p.entropy_out[j] = (float)h;
        s += h;
    }
    const double tot = block_sum(s, red);
    if (threadIdx.x == 0) p.partial[blockIdx.x] = tot;
}

__global__ __launch_bounds__(kBlock) void predict_final_kernel(const PredictParams p)
{
    __shared__ double red[kBlock];
    double s = 0.0;
    for (int b = threadIdx.x; b < p.n_blocks; b += kBlock) s += p.partial[b];
    const double mean = block_sum(s, red) / (double)p.n_slots;
    if (threadIdx.x == 0) {
        bool fresh = p.longer || p.n_sel == 0;
        if (!fresh) fresh = mean > p.gamma * log((double)p.n_sel);
        p.result_out[0] = fresh ? 1.f : 0.f;
        p.result_out[1] = (float)mean;
    }
}

// --------------------------------------------------------------------------------- capture
struct CaptureParams {
    const void *base[2], *real[2];  // [0] keys, [1] values
    void *out[2];
    Strides s_base[2], s_real[2], s_out[2];
    int32_t H, S, LH, lh_per_block, n_token_tiles, delta;
    double inv_freq[kMaxHalf];
};

// Same work split as the align kernel: LPR = D / (2 * EPV) lanes per row, lane r owning both
// members of each rotation pair; a block is 256 / LPR consecutive tokens of a run of (layer, head)
// pairs of ONE tensor (blockIdx.y: 0 = keys, 1 = values).
template <typename T, int LPR>
__global__ __launch_bounds__(kBlock) void capture_kernel(const CaptureParams p)
{
    constexpr int EPV = Elem<T>::EPV;
    constexpr int HALF = LPR * EPV;
    constexpr int RPB = kBlock / LPR;
    __shared__ __align__(8) float cs_raw[2 * HALF];
    float2 *cs = reinterpret_cast<float2 *>(cs_raw);

    const int tid = threadIdx.x;
    const int row = tid / LPR, lir = tid % LPR;
    const int tile = blockIdx.x % p.n_token_tiles;
    const int chunk = blockIdx.x / p.n_token_tiles;
    const int which = blockIdx.y;
    const bool rot = which == 0 && p.delta != 0;
    const int t = tile * RPB + row;
    if (rot)
        for (int i = tid; i < HALF; i += kBlock) cs[i] = rope_cos_sin(p.delta, p.inv_freq[i]);
    __syncthreads();
    if (t >= p.S) return;

    float bc[EPV], bs[EPV];
    if (rot) {
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
            const float2 v = cs[lir * EPV + e];
            bc[e] = v.x;
            bs[e] = v.y;
        }
    }
    const T *bp = static_cast<const T *>(p.base[which]);
    const T *rp = static_cast<const T *>(p.real[which]);
    T *op = static_cast<T *>(p.out[which]);
    const Strides sb = p.s_base[which], sr = p.s_real[which], so = p.s_out[which];
    const int64_t col0 = (int64_t)lir * EPV;
    const int lh1 = min((chunk + 1) * p.lh_per_block, p.LH);
    for (int lh = chunk * p.lh_per_block; lh < lh1; ++lh) {
        const int l = lh / p.H, h = lh % p.H;
        const T *xp = bp + l * sb.layer + h * sb.head + t * sb.token + col0;
        const T *yp = rp + l * sr.layer + h * sr.head + t * sr.token + col0;
        const u32x4 xlo = load16_stream(xp), xhi = load16_stream(xp + HALF);
        const u32x4 ylo = load16_stream(yp), yhi = load16_stream(yp + HALF);
        float blo[EPV], bhi[EPV], rlo[EPV], rhi[EPV];
        unpack<T>(xlo, blo);
        unpack<T>(xhi, bhi);
        unpack<T>(ylo, rlo);
        unpack<T>(yhi, rhi);
        if (rot) {
#pragma unroll
            for (int e = 0; e < EPV; ++e) {
                const float a = blo[e], b = bhi[e];
                blo[e] = a * bc[e] - b * bs[e];
                bhi[e] = b * bc[e] + a * bs[e];
            }
        }
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
            rlo[e] -= blo[e];
            rhi[e] -= bhi[e];
        }
        T *zp = op + l * so.layer + h * so.head + t * so.token + col0;
        store16_stream(zp, pack<T>(rlo));
        store16_stream(zp + HALF, pack<T>(rhi));
    }
}

template <typename T, int LPR>
int launch_capture(const CaptureParams &p, int n_blocks, hipStream_t stream)
{
    return launch(capture_kernel<T, LPR>, dim3(n_blocks, 2), dim3(kBlock), 0, stream, p);
}

}  // namespace

extern "C" size_t kvcomm_anchor_predict_workspace(int64_t n_slots)
{
    if (n_slots <= 0) return 0;
    const int64_t nb = (n_slots + kBlock - 1) / kBlock;
    return sizeof(double) * (size_t)(nb < kMaxPredictBlocks ? nb : kMaxPredictBlocks);
}

extern "C" int kvcomm_anchor_predict(const float *weights, int64_t n_slots, const int32_t *anchor_len,
                                     int32_t n_anchors, int32_t seg_len, float gamma, float *entropy_out,
                                     float *result_out, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!weights || !anchor_len || !result_out || n_slots <= 0 || n_anchors <= 0 || seg_len <= 0) return KVCOMM_EINVAL;
    if (n_anchors > KVCOMM_MAX_ANCHORS) return KVCOMM_EUNSUPPORTED;
    if (!(gamma >= 0.f)) return KVCOMM_EINVAL;  // also rejects NaN
    PredictParams p{};
    int max_len = 0;
    for (int a = 0; a < n_anchors; ++a) {
        if (anchor_len[a] < 0) return KVCOMM_EINVAL;
        if (anchor_len[a] > max_len) max_len = anchor_len[a];
        if (anchor_len[a] >= seg_len) {
            p.is_sel[a] = 1;
            ++p.n_sel;
        }
    }
    const size_t need = kvcomm_anchor_predict_workspace(n_slots);
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 7u)) return KVCOMM_EWORKSPACE;
    p.weights = weights;
    p.entropy_out = entropy_out;
    p.result_out = result_out;
    p.partial = static_cast<double *>(workspace);
    p.n_slots = n_slots;
    p.n_blocks = (int32_t)(need / sizeof(double));
    p.slots_per_block = (n_slots + p.n_blocks - 1) / p.n_blocks;
    p.n_anchors = n_anchors;
    p.longer = seg_len > max_len;
    p.gamma = (double)gamma;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (int st = launch(entropy_partial_kernel, dim3(p.n_blocks), dim3(kBlock), 0, s, p)) return st;
    return launch(predict_final_kernel, dim3(1), dim3(kBlock), 0, s, p);
}

extern "C" int kvcomm_capture_offsets(const kvcomm_model *model, kvcomm_tensor base_k, kvcomm_tensor base_v,
                                      kvcomm_tensor real_k, kvcomm_tensor real_v, int32_t seg_len, int32_t delta_pos,
                                      kvcomm_tensor out_dk, kvcomm_tensor out_dv, void *stream)
{
    int st = check_model(model);
    if (st) return st;
    if (seg_len <= 0) return KVCOMM_EINVAL;
    const int dt = model->dtype;
    if ((st = check_tensor(base_k, dt, true)) || (st = check_tensor(base_v, dt, true)) ||
        (st = check_tensor(real_k, dt, true)) || (st = check_tensor(real_v, dt, true)) ||
        (st = check_tensor(out_dk, dt, true)) || (st = check_tensor(out_dv, dt, true)))
        return st;

    CaptureParams p{};
    p.base[0] = base_k.ptr;
    p.base[1] = base_v.ptr;
    p.real[0] = real_k.ptr;
    p.real[1] = real_v.ptr;
    p.out[0] = out_dk.ptr;
    p.out[1] = out_dv.ptr;
    p.s_base[0] = strides_of(base_k);
    p.s_base[1] = strides_of(base_v);
    p.s_real[0] = strides_of(real_k);
    p.s_real[1] = strides_of(real_v);
    p.s_out[0] = strides_of(out_dk);
    p.s_out[1] = strides_of(out_dv);
    p.H = model->n_kv_heads;
    p.S = seg_len;
    p.LH = model->n_layers * model->n_kv_heads;
    p.delta = delta_pos;
    for (int i = 0; i < model->head_dim / 2; ++i)
        p.inv_freq[i] = pow(model->rope_theta, -2.0 * (double)i / (double)model->head_dim);

    const int es = elem_size(dt);
    const int lpr = model->head_dim / (2 * (16 / es));
    const int rpb = kBlock / lpr;
    p.n_token_tiles = (seg_len + rpb - 1) / rpb;
    const int target_blocks = 16384;
    int n_chunks = (target_blocks + p.n_token_tiles - 1) / p.n_token_tiles;
    if (n_chunks > p.LH) n_chunks = p.LH;
    if (n_chunks < 1) n_chunks = 1;
    p.lh_per_block = (p.LH + n_chunks - 1) / n_chunks;
    n_chunks = (p.LH + p.lh_per_block - 1) / p.lh_per_block;
    const int n_blocks = n_chunks * p.n_token_tiles;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dt == KVCOMM_BF16) {
        switch (lpr) {
            case 4: return launch_capture<bf16_t, 4>(p, n_blocks, s);
            case 8: return launch_capture<bf16_t, 8>(p, n_blocks, s);
            case 16: return launch_capture<bf16_t, 16>(p, n_blocks, s);
        }
    } else {
        switch (lpr) {
            case 8: return launch_capture<float, 8>(p, n_blocks, s);
            case 16: return launch_capture<float, 16>(p, n_blocks, s);
            case 32: return launch_capture<float, 32>(p, n_blocks, s);
        }
    }
    return KVCOMM_EUNSUPPORTED;
}
