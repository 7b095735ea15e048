// kvcomm_suffix_attn: causal attention of the non-shared suffix queries over the assembled,
// aligned cache (workflow step 4 of the paper; q, k, v as in Sec. 3.1).  Suffix query i sits
// at cache position n_ctx + i and sees keys 0 .. n_ctx + i.
//
// bf16 path (attn_mfma_kernel): flash-style single pass on bf16 MFMA (32x32x16) with fp32
// accumulation and an fp32 online softmax.
//   * GQA packing: the G query heads that share a kv head are folded into the row axis of one
//     tile (row r = i * G + g), so each K/V tile staged in LDS serves G heads at once.
//   * Both products are computed transposed, S^T = K Q^T and O^T = V^T P^T.  In the 32x32
//     accumulator layout a lane then owns ONE query column: the row max and row sum of the
//     softmax are in-register reductions plus a single exchange with lane+32, the rescale of
//     O is a per-lane scalar, and the exponentiated scores are already laid out as the B
//     operand of the second product (the key order inside a 16-key step is a fixed
//     permutation, applied identically to V^T when it is written to LDS).
//   * K tile [64 keys][D] and V^T tile [D][64 keys] live in LDS with an XOR swizzle of the
//     16-byte chunk index so that the 16-byte operand reads are bank-conflict free; V is
//     transposed in registers (4 keys x 8 channels per thread) on its way into LDS.
//   * Global loads of tile j+1 are issued before the MFMA work of tile j.
//   * Row tiles are ordered longest-first and the block index is remapped so that the row
//     tiles of one (layer, kv head) run on the same XCD and share its L2.
// fp32 path (attn_f32_kernel): one wavefront per query row, plain fp32 FMA and expf with an
// online softmax over 64-key chunks; it exists for exactness, not speed.
#include <math.h>

#include "kvcomm_device.h"

namespace {

using namespace kvc;

struct AttnParams {
    const void *q, *k, *v;
    void *out;
    float *lse;
    Strides s_q, s_k, s_v, s_o;
    int32_t L, Hkv, G, n_ctx, tq, N;
    int32_t n_row_tiles;
    float scale;       // softmax scale
    float scale_log2;  // scale * log2(e)
};

// ------------------------------------------------------------------------------- bf16 MFMA
constexpr int kKT = 64;  // keys per LDS tile

__device__ __forceinline__ bf16x8 as_bf16x8(const u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

typedef __attribute__((address_space(3))) unsigned char lds_byte;
typedef short s16x4 __attribute__((ext_vector_type(4)));

// Two 8-byte transposing LDS reads (ds_read_b64_tr_b16) -> one 8 x bf16 MFMA operand.
// Within each group of 16 lanes the instruction returns to lane i, element e, the 16-bit
// element (i % 4) found at the address supplied by lane 4*e + i/4 of the group.
__device__ __forceinline__ bf16x8 lds_read_tr_pair(const lds_byte *a0, const lds_byte *a1)
{
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)a0);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)a1);
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

template <int D, int QB, int WPE>
__global__ __launch_bounds__(256, WPE) void attn_mfma_kernel(const AttnParams p)
{
    constexpr int NKS = D / 16;      // k-steps of S^T = K Q^T
    constexpr int NDB = D / 32;      // 32-row blocks of O^T
    constexpr int MW = 32 * QB;      // query rows per wavefront
    constexpr int BM = 4 * MW;       // query rows per block
    constexpr int KCH = D / 8;       // 16-byte chunks per K / V row
    constexpr int ROWB = D * 2;      // bytes per K / V row
    constexpr int TILEB = kKT * ROWB;               // bytes per K (or V) tile
    constexpr int LPT = (kKT * KCH) / 256;          // direct loads per thread and tensor
    constexpr int KSWZ = (KCH < 16 ? KCH : 16) - 1; // K chunk swizzle: c ^ (key & KSWZ)
    constexpr int VSWZ = KCH - 1;                   // V chunk swizzle: c ^ ((4 * (key & 3)) & VSWZ)

    // [buffer][K tile | V tile]; both tiles are [64 keys][D] with XOR-swizzled 16-byte chunks.
    __shared__ __align__(16) unsigned char smem[2 * 2 * TILEB];
    lds_byte *lds = (lds_byte *)smem;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, n = lane & 31, hg = lane >> 5;

    // XCD-aware block order: hardware deals consecutive block ids round-robin to the 8 XCDs;
    // give each XCD one contiguous range of logical tiles.
    int logical;
    {
        const int nb = gridDim.x, b = blockIdx.x;
        const int base = nb >> 3, rem = nb & 7, x = b & 7;
        logical = x * base + min(x, rem) + (b >> 3);
    }
    const int lh = logical / p.n_row_tiles;
    const int rt = p.n_row_tiles - 1 - logical % p.n_row_tiles;  // longest rows first
    const int l = lh / p.Hkv, hkv = lh % p.Hkv;

    const bf16_t *qb_ = static_cast<const bf16_t *>(p.q);
    const bf16_t *kb_ = static_cast<const bf16_t *>(p.k) + l * p.s_k.layer + hkv * p.s_k.head;
    const bf16_t *vb_ = static_cast<const bf16_t *>(p.v) + l * p.s_v.layer + hkv * p.s_v.head;

    // This lane's query column in each 32-row block of the wavefront.
    int qi[QB], qg[QB];
    bool qvalid[QB];
    bf16x8 qf[QB][NKS];
#pragma unroll
    for (int b = 0; b < QB; ++b) {
        const int r = rt * BM + wave * MW + b * 32 + n;
        const int i = r / p.G;
        qg[b] = r % p.G;
        qvalid[b] = i < p.tq;
        qi[b] = min(i, p.tq - 1);
        const bf16_t *qrow = qb_ + l * p.s_q.layer + (int64_t)(hkv * p.G + qg[b]) * p.s_q.head + qi[b] * p.s_q.token;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) qf[b][ks] = as_bf16x8(load16(qrow + ks * 16 + hg * 8));
    }

    const int wg_imax = min(p.tq - 1, (rt * BM + BM - 1) / p.G);
    const int n_tiles = (p.n_ctx + wg_imax + 1 + kKT - 1) / kKT;
    const int wave_last_key = p.n_ctx + min(p.tq - 1, (rt * BM + wave * MW + MW - 1) / p.G);
    const int wave_nomask_key = p.n_ctx + min(p.tq - 1, (rt * BM + wave * MW) / p.G);

    f32x16 o[NDB][QB];
    float m[QB], lsum[QB];
#pragma unroll
    for (int b = 0; b < QB; ++b) {
        m[b] = -INFINITY;
        lsum[b] = 0.f;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int j = 0; j < 16; ++j) o[db][b][j] = 0.f;
    }

    // ---- global -> LDS direct loads (global_load_lds_dwordx4): lane i of a wavefront fills the
    // 16-byte LDS chunk (base + i); the swizzle is applied by choosing which global chunk it fetches.
    // Wavefront w fills chunks [(4w + it) * 64, +64) of each tile, i.e. 64 / KCH consecutive keys.
    int ld_key[LPT], ld_kc[LPT], ld_vc[LPT];
#pragma unroll
    for (int it = 0; it < LPT; ++it) {
        const int P = (wave * LPT + it) * 64 + lane;
        const int key = P / KCH, pc = P % KCH;
        ld_key[it] = key;
        ld_kc[it] = (pc ^ (key & KSWZ)) * 8;                    // element offset inside the row
        ld_vc[it] = (pc ^ ((4 * (key & 3)) & VSWZ)) * 8;
    }
    auto issue_loads = [&](int tile, int buf) {
        const int key0 = tile * kKT;
#pragma unroll
        for (int it = 0; it < LPT; ++it) {
            const int key = min(key0 + ld_key[it], p.N - 1);  // rows past the cache end are never unmasked
            lds_byte *dk = lds + buf * 2 * TILEB + (wave * LPT + it) * 1024;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(kb_ + (int64_t)key * p.s_k.token + ld_kc[it]),
                                             (__attribute__((address_space(3))) void *)dk, 16, 0, 0);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(vb_ + (int64_t)key * p.s_v.token + ld_vc[it]),
                                             (__attribute__((address_space(3))) void *)(dk + TILEB), 16, 0, 0);
        }
    };

    // ---- per-lane LDS read offsets
    // K operand (rows = keys): lane (n, hg) reads chunk 2*ks + hg of key 32*kb + n.
    int k_off[NKS];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) k_off[ks] = n * ROWB + (((2 * ks + hg) ^ (n & KSWZ)) * 16);
    // V^T operand through transposing reads: lane i of a 16-lane group supplies the address of
    // 4 channels [32*db + 16*gi + 4*(i%4), +4) of key 16*ks + 4*hg + i/4 (second read: + 8 keys).
    int v_off[NDB];
    {
        const int i16 = lane & 15, gi = (lane >> 4) & 1;
        const int row = 4 * hg + (i16 >> 2);
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
            const int col = 32 * db + 16 * gi + 4 * (i16 & 3);
            const int pc = (col >> 3) ^ ((4 * (row & 3)) & VSWZ);
            v_off[db] = row * ROWB + pc * 16 + (col & 7) * 2;
        }
    }

    issue_loads(0, 0);
    __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): tile 0 has landed in LDS
    __syncthreads();

    for (int tile = 0; tile < n_tiles; ++tile) {
        const int buf = tile & 1;
        const int key0 = tile * kKT;
        // Tile j+1 streams into the other buffer while tile j is consumed.
        if (tile + 1 < n_tiles) issue_loads(tile + 1, buf ^ 1);

        if (key0 <= wave_last_key) {  // wavefront-uniform: else the tile lies after all of its queries
            const lds_byte *kl = lds + buf * 2 * TILEB;
            const lds_byte *vl = kl + TILEB;

            // ---- S^T = K Q^T : [64 keys] x [MW queries]
            f32x16 s[2][QB];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int b = 0; b < QB; ++b)
#pragma unroll
                    for (int j = 0; j < 16; ++j) s[kb][b][j] = 0.f;
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    const bf16x8 a = as_bf16x8(*(const __attribute__((address_space(3))) u32x4 *)(kl + kb * 32 * ROWB + k_off[ks]));
#pragma unroll
                    for (int b = 0; b < QB; ++b)
                        s[kb][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[b][ks], s[kb][b], 0, 0, 0);
                }
            }

            // ---- online softmax; lane (n, hg) holds key rows 8*(j/4) + 4*hg + j%4 of each block
            const bool need_mask = key0 + kKT - 1 > wave_nomask_key;
            bf16x8 pf[QB][4];
#pragma unroll
            for (int b = 0; b < QB; ++b) {
                if (need_mask) {
                    const int limit = p.n_ctx + qi[b] - key0;  // last visible key, relative to the tile
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                        for (int j = 0; j < 16; ++j) {
                            const int key = kb * 32 + 8 * (j >> 2) + 4 * hg + (j & 3);
                            if (key > limit) s[kb][b][j] = -INFINITY;
                        }
                }
                float mx = s[0][b][0];
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int j = 0; j < 16; ++j) mx = fmaxf(mx, s[kb][b][j]);
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float m_new = fmaxf(m[b], mx);  // finite: key 0 is visible to every query
                const float mc = m_new * p.scale_log2;
                float rs = 0.f;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int j = 0; j < 16; ++j) {
                        const float e = __builtin_amdgcn_exp2f(s[kb][b][j] * p.scale_log2 - mc);
                        s[kb][b][j] = e;
                        rs += e;
                    }
                // Rescale the running sum and O only when some query of the wavefront saw a new max.
                if (__builtin_amdgcn_ballot_w64(m_new > m[b]) != 0) {
                    const float corr = __builtin_amdgcn_exp2f((m[b] - m_new) * p.scale_log2);
                    lsum[b] *= corr;
#pragma unroll
                    for (int db = 0; db < NDB; ++db)
#pragma unroll
                        for (int j = 0; j < 16; ++j) o[db][b][j] *= corr;
                }
                lsum[b] += rs;
                m[b] = m_new;
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    u32x4 pk;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        pk[e] = pack_bf16x2(s[ks >> 1][b][8 * (ks & 1) + 2 * e], s[ks >> 1][b][8 * (ks & 1) + 2 * e + 1]);
                    pf[b][ks] = as_bf16x8(pk);
                }
            }

            // ---- O^T += V^T P^T : [D channels] x [MW queries]
#pragma unroll
            for (int db = 0; db < NDB; ++db) {
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    const lds_byte *va = vl + ks * 16 * ROWB + v_off[db];
                    const bf16x8 a = lds_read_tr_pair(va, va + 8 * ROWB);
#pragma unroll
                    for (int b = 0; b < QB; ++b)
                        o[db][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[b][ks], o[db][b], 0, 0, 0);
                }
            }
        }
        __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): this wavefront's share of tile j+1 is in LDS
        __syncthreads();                     // ... and so is everybody else's; tile j is no longer read
    }

    // ---- epilogue: normalise and store; lane (n, hg) holds channels 32*db + 8*(j/4) + 4*hg + j%4
    bf16_t *ob = static_cast<bf16_t *>(p.out);
#pragma unroll
    for (int b = 0; b < QB; ++b) {
        const float ltot = lsum[b] + __shfl_xor(lsum[b], 32);
        if (!qvalid[b]) continue;
        const float inv = 1.f / ltot;
        const int hq = hkv * p.G + qg[b];
        bf16_t *orow = ob + l * p.s_o.layer + (int64_t)hq * p.s_o.head + qi[b] * p.s_o.token;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int j4 = 0; j4 < 4; ++j4) {
                u32x2 w;
                w[0] = pack_bf16x2(o[db][b][4 * j4] * inv, o[db][b][4 * j4 + 1] * inv);
                w[1] = pack_bf16x2(o[db][b][4 * j4 + 2] * inv, o[db][b][4 * j4 + 3] * inv);
                *reinterpret_cast<u32x2 *>(orow + db * 32 + 8 * j4 + 4 * hg) = w;
            }
        if (p.lse && hg == 0)
            p.lse[((int64_t)l * p.Hkv * p.G + hq) * p.tq + qi[b]] = m[b] * p.scale + logf(ltot);
    }
}

// ------------------------------------------------------------------------------- fp32 path
template <int D>
__global__ __launch_bounds__(256) void attn_f32_kernel(const AttnParams p)
{
    constexpr int CPL = D / 64;  // output channels per lane
    __shared__ float q_lds[4][D];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + wave;  // over (l, hq, i)
    const int Hq = p.Hkv * p.G;
    if (row >= (int64_t)p.L * Hq * p.tq) return;
    const int i = (int)(row % p.tq);
    const int hq = (int)((row / p.tq) % Hq);
    const int l = (int)(row / ((int64_t)p.tq * Hq));
    const int hkv = hq / p.G;
    const float *q = static_cast<const float *>(p.q) + l * p.s_q.layer + (int64_t)hq * p.s_q.head + i * p.s_q.token;
    const float *k = static_cast<const float *>(p.k) + l * p.s_k.layer + (int64_t)hkv * p.s_k.head;
    const float *v = static_cast<const float *>(p.v) + l * p.s_v.layer + (int64_t)hkv * p.s_v.head;
    for (int c = lane; c < D; c += 64) q_lds[wave][c] = q[c];
    // only this wavefront reads q_lds[wave]; its writes are ordered before the reads below
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    const int last = p.n_ctx + i;
    float m = -INFINITY, lsum = 0.f;
    float acc[CPL];
#pragma unroll
    for (int c = 0; c < CPL; ++c) acc[c] = 0.f;

    for (int j0 = 0; j0 <= last; j0 += 64) {
        const int j = j0 + lane;
        float sc = -INFINITY;
        if (j <= last) {
            const float *kr = k + (int64_t)j * p.s_k.token;
            float dot = 0.f;
#pragma unroll 4
            for (int c = 0; c < D; c += 4) {
                const f32x4 kv = *reinterpret_cast<const f32x4 *>(kr + c);
                dot = fmaf(q_lds[wave][c], kv[0], dot);
                dot = fmaf(q_lds[wave][c + 1], kv[1], dot);
                dot = fmaf(q_lds[wave][c + 2], kv[2], dot);
                dot = fmaf(q_lds[wave][c + 3], kv[3], dot);
            }
            sc = dot * p.scale;
        }
        float cmax = sc;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) cmax = fmaxf(cmax, __shfl_xor(cmax, off));
        const float m_new = fmaxf(m, cmax);  // finite: lane 0 of every chunk is visible
        const float corr = expf(m - m_new);
        const float pj = j <= last ? expf(sc - m_new) : 0.f;
        float psum = pj;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) psum += __shfl_xor(psum, off);
        lsum = lsum * corr + psum;
        m = m_new;
#pragma unroll
        for (int c = 0; c < CPL; ++c) acc[c] *= corr;
        const int cnt = min(64, last - j0 + 1);
        for (int jj = 0; jj < cnt; ++jj) {
            const float pv = __shfl(pj, jj);
            const float *vr = v + (int64_t)(j0 + jj) * p.s_v.token;
#pragma unroll
            for (int c = 0; c < CPL; ++c) acc[c] = fmaf(pv, vr[lane + 64 * c], acc[c]);
        }
    }
    float *o = static_cast<float *>(p.out) + l * p.s_o.layer + (int64_t)hq * p.s_o.head + i * p.s_o.token;
    const float inv = 1.f / lsum;
#pragma unroll
    for (int c = 0; c < CPL; ++c) o[lane + 64 * c] = acc[c] * inv;
    if (p.lse && lane == 0) p.lse[row] = m + logf(lsum);
}

}  // namespace

extern "C" size_t kvcomm_suffix_attn_workspace(const kvcomm_model *, int32_t, int32_t) { return 0; }

extern "C" int kvcomm_suffix_attn(const kvcomm_model *model, kvcomm_tensor q, kvcomm_tensor cache_k,
                                  kvcomm_tensor cache_v, int32_t n_ctx, int32_t tq, float softmax_scale,
                                  kvcomm_tensor out, float *lse_out, void *, size_t, void *stream)
{
    int st = check_model(model);
    if (st) return st;
    if (tq <= 0 || n_ctx < 0) return KVCOMM_EINVAL;
    const int dt = model->dtype;
    if ((st = check_tensor(q, dt, true)) || (st = check_tensor(cache_k, dt, true)) ||
        (st = check_tensor(cache_v, dt, true)) || (st = check_tensor(out, dt, true)))
        return st;

    AttnParams p{};
    p.q = q.ptr;
    p.k = cache_k.ptr;
    p.v = cache_v.ptr;
    p.out = out.ptr;
    p.lse = lse_out;
    p.s_q = strides_of(q);
    p.s_k = strides_of(cache_k);
    p.s_v = strides_of(cache_v);
    p.s_o = strides_of(out);
    p.L = model->n_layers;
    p.Hkv = model->n_kv_heads;
    p.G = model->n_q_heads / model->n_kv_heads;
    p.n_ctx = n_ctx;
    p.tq = tq;
    p.N = n_ctx + tq;
    p.scale = softmax_scale > 0.f ? softmax_scale : (float)(1.0 / sqrt((double)model->head_dim));
    p.scale_log2 = (float)((double)p.scale * 1.4426950408889634);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int D = model->head_dim;

    if (dt == KVCOMM_F32) {
        const int64_t rows = (int64_t)p.L * model->n_q_heads * tq;
        const unsigned n_blocks = (unsigned)((rows + 3) / 4);
        switch (D) {
            case 64: hipLaunchKernelGGL(attn_f32_kernel<64>, dim3(n_blocks), dim3(256), 0, s, p); break;
            case 128: hipLaunchKernelGGL(attn_f32_kernel<128>, dim3(n_blocks), dim3(256), 0, s, p); break;
            case 256: hipLaunchKernelGGL(attn_f32_kernel<256>, dim3(n_blocks), dim3(256), 0, s, p); break;
            default: return KVCOMM_EUNSUPPORTED;
        }
        return launch_status();
    }

#ifndef KVC_ATTN_QB
#define KVC_ATTN_QB 1
#endif
#ifndef KVC_ATTN_WPE
#define KVC_ATTN_WPE 2
#endif
    constexpr int QB = KVC_ATTN_QB;
    constexpr int WPE = KVC_ATTN_WPE;
    constexpr int BM = 4 * 32 * QB;
    p.n_row_tiles = (p.G * tq + BM - 1) / BM;
    const unsigned n_blocks = (unsigned)(p.L * p.Hkv * p.n_row_tiles);
    switch (D) {
        case 64: hipLaunchKernelGGL((attn_mfma_kernel<64, QB, WPE>), dim3(n_blocks), dim3(256), 0, s, p); break;
        case 128: hipLaunchKernelGGL((attn_mfma_kernel<128, QB, WPE>), dim3(n_blocks), dim3(256), 0, s, p); break;
        case 256: hipLaunchKernelGGL((attn_mfma_kernel<256, 1, 1>), dim3(n_blocks), dim3(256), 0, s, p); break;
        default: return KVCOMM_EUNSUPPORTED;
    }
    return launch_status();
}
