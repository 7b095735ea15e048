// Device-side helpers shared by the three gfx950 kernels of libkvcomm: 16-byte vector
// moves, bf16 <-> fp32 conversion and host-side argument checks.  Nothing here is used by
// (or shared with) the CPU oracle.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

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

static inline int launch_status()
{
    return hipGetLastError() == hipSuccess ? KVCOMM_OK : KVCOMM_EHIP;
}

}  // namespace kvc
