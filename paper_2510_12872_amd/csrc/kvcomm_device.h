// Device-side helpers shared by the three gfx950 kernels of libkvcomm: 16-byte vector
// moves, bf16 <-> fp32 conversion and host-side argument checks.  Nothing here is used by
// (or shared with) the CPU oracle.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <utility>
#include <vector>

#include "kvcomm.h"

namespace kvc {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct bf16_t {
    uint16_t bits;
};

struct Strides {
    int64_t layer, head, token;
};

static inline Strides strides_of(const kvcomm_tensor &t) { return Strides{t.stride_layer, t.stride_head, t.stride_token}; }

template <typename T>
struct Elem;
template <>
struct Elem<float> {
    static constexpr int EPV = 4;  // elements per 16-byte vector
};
template <>
struct Elem<bf16_t> {
    static constexpr int EPV = 8;
};

// Streaming 16-byte accesses: every cache row of the align / distance kernels is touched
// exactly once, so mark the traffic non-temporal to keep it from displacing the small
// reused data (weights, rotation tables) in L2.
__device__ __forceinline__ u32x4 load16_stream(const void *p) { return __builtin_nontemporal_load((const u32x4 *)p); }
__device__ __forceinline__ void store16_stream(void *p, u32x4 v) { __builtin_nontemporal_store(v, (u32x4 *)p); }
__device__ __forceinline__ u32x4 load16(const void *p) { return *(const u32x4 *)p; }

// Two floats -> packed bf16 pair, round to nearest even (v_cvt_pk_bf16_f32).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    f32x2 f = {lo, hi};
    bf16x2 r = __builtin_convertvector(f, bf16x2);
    return __builtin_bit_cast(uint32_t, r);
}

template <typename T>
__device__ __forceinline__ void unpack(const u32x4 raw, float (&out)[Elem<T>::EPV]);

template <>
__device__ __forceinline__ void unpack<float>(const u32x4 raw, float (&out)[4])
{
#pragma unroll
    for (int i = 0; i < 4; ++i) out[i] = __uint_as_float(raw[i]);
}

template <>
__device__ __forceinline__ void unpack<bf16_t>(const u32x4 raw, float (&out)[8])
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        out[2 * i] = __uint_as_float(raw[i] << 16);
        out[2 * i + 1] = __uint_as_float(raw[i] & 0xffff0000u);
    }
}

template <typename T>
__device__ __forceinline__ u32x4 pack(const float (&in)[Elem<T>::EPV]);

template <>
__device__ __forceinline__ u32x4 pack<float>(const float (&in)[4])
{
    u32x4 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = __float_as_uint(in[i]);
    return r;
}

template <>
__device__ __forceinline__ u32x4 pack<bf16_t>(const float (&in)[8])
{
    u32x4 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = pack_bf16x2(in[2 * i], in[2 * i + 1]);
    return r;
}

// cos / sin of the RoPE angle delta * inv_freq: product and reduction modulo 2*pi in double
// (inv_freq = theta^(-2i/D) comes from the host in double), sine and cosine of the reduced angle in fp32.
__device__ __forceinline__ float2 rope_cos_sin(int32_t delta, double inv_freq)
{
    const double x = (double)delta * inv_freq;
    const double k = rint(x * 0.15915494309189535);  // 1 / (2 pi)
    double red = fma(-k, 6.283185307179586, x);      // 2 pi, high part
    red = fma(-k, 2.4492935982947064e-16, red);      // 2 pi, low part
    const float rf = (float)red;
    return make_float2(cosf(rf), sinf(rf));
}

// ------------------------------------------------------------------------- host-side checks
static inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static inline int elem_size(int dtype) { return dtype == KVCOMM_BF16 ? 2 : 4; }

// Model fields every entry point relies on.
static inline int check_model(const kvcomm_model *m)
{
    if (!m) return KVCOMM_EINVAL;
    if (m->n_layers <= 0 || m->n_kv_heads <= 0 || m->n_q_heads <= 0 || m->head_dim <= 0) return KVCOMM_EINVAL;
    if (m->dtype != KVCOMM_F32 && m->dtype != KVCOMM_BF16) return KVCOMM_EINVAL;
    if (!(m->rope_theta > 0.0)) return KVCOMM_EINVAL;
    if (m->head_dim != 64 && m->head_dim != 128 && m->head_dim != 256) return KVCOMM_EUNSUPPORTED;
    if (m->n_q_heads % m->n_kv_heads != 0) return KVCOMM_EUNSUPPORTED;
    return KVCOMM_OK;
}

// A tensor whose rows are moved with 16-byte accesses.  `need_ptr` is false for layouts
// whose ptr field is ignored (anchor layouts).
static inline int check_tensor(const kvcomm_tensor &t, int dtype, bool need_ptr)
{
    const int64_t epv = 16 / elem_size(dtype);
    if (need_ptr && (!t.ptr || !aligned16(t.ptr))) return KVCOMM_EINVAL;
    if (t.stride_layer < 0 || t.stride_head < 0 || t.stride_token < 0) return KVCOMM_EINVAL;
    if (t.stride_layer % epv || t.stride_head % epv || t.stride_token % epv) return KVCOMM_EINVAL;
    return KVCOMM_OK;
}

static inline int check_gran(int gran)
{
    return (gran == KVCOMM_W_TOKEN || gran == KVCOMM_W_LAYER_HEAD_TOKEN || gran == KVCOMM_W_SEGMENT) ? KVCOMM_OK
                                                                                                       : KVCOMM_EINVAL;
}

// ----------------------------------------------------------------- host-side aliasing checks
// A [L, H, n, D] tensor as the caller described it: the bytes it touches are L * H runs ("blocks"), one per
// (layer, head), each reaching from the block's first element to the last element of its last token.
struct Extent {
    uintptr_t base;
    int64_t sl, sh;      // layer / head strides in bytes
    int64_t run;         // bytes from a block's first to one past its last element
    int32_t L, H;
    uintptr_t lo() const { return base; }
    uintptr_t hi() const { return base + (uintptr_t)((L - 1) * sl + (H - 1) * sh + run); }
};

static inline Extent extent_of(const kvcomm_tensor &t, int L, int H, int64_t n_tokens, int D, int es)
{
    return Extent{reinterpret_cast<uintptr_t>(t.ptr), t.stride_layer * es, t.stride_head * es,
                  ((n_tokens - 1) * t.stride_token + D) * es, L, H};
}

static inline Extent extent_of(const void *ptr, const kvcomm_tensor &layout, int L, int H, int64_t n_tokens, int D, int es)
{
    kvcomm_tensor t = layout;
    t.ptr = const_cast<void *>(ptr);
    return extent_of(t, L, H, n_tokens, D, es);
}

static inline Extent extent_flat(const void *ptr, size_t bytes)
{
    return Extent{reinterpret_cast<uintptr_t>(ptr), 0, 0, (int64_t)bytes, 1, 1};
}

// Same description (pointer, strides, shape): the in-place case.
static inline bool same_extent(const Extent &a, const Extent &b)
{
    return a.base == b.base && a.sl == b.sl && a.sh == b.sh && a.run == b.run && a.L == b.L && a.H == b.H;
}

// Do two tensors touch a common byte?  Exact at the granularity of blocks (gaps between the tokens of one
// block count as touched).  Cheap when the whole ranges are disjoint, which is the usual case.
static inline bool extents_overlap(const Extent &a, const Extent &b)
{
    if (a.hi() <= b.lo() || b.hi() <= a.lo()) return false;
    if (a.sl == b.sl && a.sh == b.sh) {
        // Views of one allocation: block (l, h) of a meets block (l', h') of b iff the distance of their
        // first bytes lies in (-run_b, run_a); only the index differences matter.
        const int64_t d0 = (int64_t)(b.base - a.base);
        const int Lm = std::max(a.L, b.L), Hm = std::max(a.H, b.H);
        for (int dl = -(Lm - 1); dl <= Lm - 1; ++dl)
            for (int dh = -(Hm - 1); dh <= Hm - 1; ++dh) {
                // b's block (l + dl, h + dh) against a's block (l, h), for some l, h that keep both in range
                if (a.L - std::max(0, -dl) - std::max(0, dl + a.L - b.L) <= 0) continue;
                if (a.H - std::max(0, -dh) - std::max(0, dh + a.H - b.H) <= 0) continue;
                const int64_t d = d0 + dl * a.sl + dh * a.sh;
                if (d > -b.run && d < a.run) return true;
            }
        return false;
    }
    std::vector<std::pair<uintptr_t, uintptr_t>> blocks;
    blocks.reserve((size_t)a.L * a.H);
    for (int l = 0; l < a.L; ++l)
        for (int h = 0; h < a.H; ++h) {
            const uintptr_t lo = a.base + (uintptr_t)(l * a.sl + h * a.sh);
            blocks.emplace_back(lo, lo + (uintptr_t)a.run);
        }
    std::sort(blocks.begin(), blocks.end());
    uintptr_t reach = 0;   // running maximum of the ends, so that nested blocks are handled too
    std::vector<uintptr_t> max_end(blocks.size());
    for (size_t i = 0; i < blocks.size(); ++i) {
        reach = std::max(reach, blocks[i].second);
        max_end[i] = reach;
    }
    for (int l = 0; l < b.L; ++l)
        for (int h = 0; h < b.H; ++h) {
            const uintptr_t lo = b.base + (uintptr_t)(l * b.sl + h * b.sh), hi = lo + (uintptr_t)b.run;
            // blocks of a that start before hi: does any of them end after lo?
            const size_t n = std::lower_bound(blocks.begin(), blocks.end(), std::make_pair(hi, (uintptr_t)0)) - blocks.begin();
            if (n > 0 && max_end[n - 1] > lo) return true;
        }
    return false;
}

// Launches a kernel that takes its parameter block by value and maps THIS launch's own return code: an
// error that an earlier, unrelated HIP call left on the thread is neither reported nor cleared.
template <typename P>
static inline int launch(void (*kernel)(P), dim3 grid, dim3 block, size_t lds_bytes, hipStream_t stream, const P &params)
{
    void *args[] = {const_cast<void *>(static_cast<const void *>(&params))};
    return hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, args, lds_bytes, stream) == hipSuccess
               ? KVCOMM_OK
               : KVCOMM_EHIP;
}

}  // namespace kvc
