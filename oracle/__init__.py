"""float64 CPU oracle for the KVComm cache-reuse step: Python face of kvcomm_oracle.c.

TEST INFRASTRUCTURE ONLY.  Imported by the tests, by the smoke check and by the
benchmark's CPU-baseline leg.  The product package never imports this module and
this module never imports the product package; the two share no code.

The arithmetic lives in kvcomm_oracle.c (plain C, double precision).  This file
only compiles that one source with gcc, converts arguments to contiguous
float64 numpy arrays (an exact upcast from bf16 / fp32) and allocates outputs.

Array conventions (see the header of kvcomm_oracle.c):
    caches  [L, H, S, D];  anchor tensors [L, H, S_a, D] each with its own S_a;
    distances / weights [A, n] with n = S (gran 0), L*H*S (gran 1) or 1 (gran 2).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kvcomm_oracle.c")
_LIB = os.path.join(_HERE, "libkvcomm_oracle.so")

GRAN_TOKEN = 0
GRAN_LAYER_HEAD_TOKEN = 1
GRAN_SEGMENT = 2

_lib = None


def build(force=False):
    """Compile kvcomm_oracle.c into libkvcomm_oracle.so next to it."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
           "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int)
        dpp = ctypes.POINTER(dp)
        lib.kvo_rope_rotate.argtypes = [dp, dp, ctypes.c_int, ctypes.c_double, ctypes.c_double]
        lib.kvo_rope_rotate.restype = None
        lib.kvo_distances.argtypes = [dp, dpp, ip] + [ctypes.c_int] * 6 + [dp, ip]
        lib.kvo_distances.restype = None
        lib.kvo_weights.argtypes = [dp, ip, ctypes.c_int, ctypes.c_size_t, ctypes.c_double, dp, ip]
        lib.kvo_weights.restype = None
        lib.kvo_align.argtypes = ([dp, dp, dpp, dpp, ip, dp] + [ctypes.c_int] * 6 +
                                  [ctypes.c_double, dp, ctypes.c_double, dp, dp])
        lib.kvo_align.restype = None
        lib.kvo_suffix_attn.argtypes = [dp, dp, dp] + [ctypes.c_int] * 6 + [ctypes.c_double, dp, dp]
        lib.kvo_suffix_attn.restype = None
        lib.kvo_capture.argtypes = [dp, dp, dp, dp] + [ctypes.c_int] * 4 + [ctypes.c_double, ctypes.c_double, dp, dp]
        lib.kvo_capture.restype = None
        lib.kvo_predict.argtypes = [dp, ip, ip, ctypes.c_int, ctypes.c_size_t, ctypes.c_int, ctypes.c_double, dp, dp]
        lib.kvo_predict.restype = ctypes.c_int
        lib.kvo_cosine.argtypes = [dp, dpp, ip] + [ctypes.c_int] * 6 + [dp, ip]
        lib.kvo_cosine.restype = None
        lib.kvo_weights_from_sim.argtypes = [dp, ip, ctypes.c_int, ctypes.c_size_t, ctypes.c_double, dp, ip]
        lib.kvo_weights_from_sim.restype = None
        lib.kvo_weights_nearest.argtypes = [dp, ip, ctypes.c_int, ctypes.c_size_t, dp, ip]
        lib.kvo_weights_nearest.restype = None
        ub = ctypes.POINTER(ctypes.c_ubyte)
        lib.kvo_e4m3_decode.argtypes = [ctypes.c_ubyte]
        lib.kvo_e4m3_decode.restype = ctypes.c_double
        lib.kvo_e4m3_encode.argtypes = [ctypes.c_double]
        lib.kvo_e4m3_encode.restype = ctypes.c_ubyte
        lib.kvo_quantize.argtypes = [dp, ctypes.c_size_t, ctypes.c_double, ub]
        lib.kvo_quantize.restype = None
        lib.kvo_dequantize.argtypes = [ub, ctypes.c_size_t, ctypes.c_double, dp]
        lib.kvo_dequantize.restype = None
        lib.kvo_num_threads.argtypes = []
        lib.kvo_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _f64(x):
    return np.ascontiguousarray(np.asarray(x, dtype=np.float64))


def _dptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _iptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int))


def _ptr_array(arrs):
    dp = ctypes.POINTER(ctypes.c_double)
    return (dp * len(arrs))(*[_dptr(a) for a in arrs])


def gran_count(gran, L, H, S):
    return {GRAN_TOKEN: S, GRAN_LAYER_HEAD_TOKEN: L * H * S, GRAN_SEGMENT: 1}[gran]


def num_threads():
    return int(_load().kvo_num_threads())


def rope_rotate(x, delta, theta):
    """Rotate the last axis of x (length D, pairs (i, i+D/2)) by position delta."""
    x = _f64(x)
    D = x.shape[-1]
    assert D % 2 == 0
    flat = x.reshape(-1, D)
    out = np.empty_like(flat)
    lib = _load()
    for r in range(flat.shape[0]):
        lib.kvo_rope_rotate(_dptr(flat[r]), _dptr(out[r]), D, float(delta), float(theta))
    return out.reshape(x.shape)


def distances(seg_k, anc_k, gran=GRAN_TOKEN):
    """seg_k [L,H,S,D]; anc_k list of [L,H,S_a,D].  Returns (dist [A,n], selected [A])."""
    seg_k = _f64(seg_k)
    L, H, S, D = seg_k.shape
    anc = [_f64(a) for a in anc_k]
    for a in anc:
        assert a.shape[0] == L and a.shape[1] == H and a.shape[3] == D
    A = len(anc)
    anc_len = np.array([a.shape[2] for a in anc], dtype=np.intc)
    n = gran_count(gran, L, H, S)
    dist = np.zeros((A, n), dtype=np.float64)
    selected = np.zeros(A, dtype=np.intc)
    _load().kvo_distances(_dptr(seg_k), _ptr_array(anc), _iptr(anc_len), A, L, H, S, D, gran,
                          _dptr(dist), _iptr(selected))
    return dist, selected


def weights(dist, selected, tau=1.0):
    """dist [A,n], selected [A] -> (w [A,n], nearest [n])."""
    dist = _f64(dist)
    A, n = dist.shape
    selected = np.ascontiguousarray(np.asarray(selected, dtype=np.intc))
    w = np.zeros((A, n), dtype=np.float64)
    nearest = np.zeros(n, dtype=np.intc)
    _load().kvo_weights(_dptr(dist), _iptr(selected), A, n, float(tau), _dptr(w), _iptr(nearest))
    return w, nearest


def align(base_k, base_v, anc_dk, anc_dv, w, delta, theta, anc_delta=None, gran=GRAN_TOKEN):
    """Offset approximation.  Returns (K^, V^) as float64 [L,H,S,D]."""
    base_k = _f64(base_k)
    base_v = _f64(base_v)
    L, H, S, D = base_k.shape
    dk = [_f64(a) for a in anc_dk]
    dv = [_f64(a) for a in anc_dv]
    A = len(dk)
    assert len(dv) == A
    anc_len = np.array([a.shape[2] for a in dk], dtype=np.intc)
    for a, b in zip(dk, dv):
        assert a.shape == b.shape and a.shape[0] == L and a.shape[1] == H and a.shape[3] == D
    w = _f64(w)
    assert w.shape == (A, gran_count(gran, L, H, S))
    ad = None if anc_delta is None else _f64(anc_delta)
    if ad is not None:
        assert ad.shape == (A,)
    out_k = np.empty_like(base_k)
    out_v = np.empty_like(base_v)
    _load().kvo_align(_dptr(base_k), _dptr(base_v), _ptr_array(dk), _ptr_array(dv), _iptr(anc_len),
                      _dptr(w), gran, A, L, H, S, D, float(delta),
                      None if ad is None else _dptr(ad), float(theta), _dptr(out_k), _dptr(out_v))
    return out_k, out_v


def suffix_attn(q, k, v, n_ctx, scale=None, want_lse=False):
    """q [L,Hq,Tq,D]; k, v [L,Hkv,n_ctx+Tq,D].  Returns out [L,Hq,Tq,D] (and lse [L,Hq,Tq])."""
    q = _f64(q)
    k = _f64(k)
    v = _f64(v)
    L, Hq, Tq, D = q.shape
    Hkv = k.shape[1]
    assert k.shape == v.shape == (L, Hkv, n_ctx + Tq, D) and Hq % Hkv == 0
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    out = np.empty_like(q)
    lse = np.empty((L, Hq, Tq), dtype=np.float64)
    _load().kvo_suffix_attn(_dptr(q), _dptr(k), _dptr(v), L, Hq, Hkv, D, n_ctx, Tq, float(scale),
                            _dptr(out), _dptr(lse))
    return (out, lse) if want_lse else out


def reuse_step(seg_k, seg_v, anc_k, anc_dk, anc_dv, delta, theta, tau=1.0, anc_delta=None,
               gran=GRAN_TOKEN):
    """Distances -> weights -> offset approximation for one segment (reuse branch of Algorithm 1)."""
    dist, selected = distances(seg_k, anc_k, gran)
    w, nearest = weights(dist, selected, tau)
    out_k, out_v = align(seg_k, seg_v, anc_dk, anc_dv, w, delta, theta, anc_delta, gran)
    return dict(dist=dist, selected=selected, w=w, nearest=nearest, out_k=out_k, out_v=out_v)


def capture(base_k, base_v, real_k, real_v, delta, theta):
    """Offset capture: (dK, dV) such that align with this single anchor and weight 1 returns the real cache."""
    base_k, base_v, real_k, real_v = _f64(base_k), _f64(base_v), _f64(real_k), _f64(real_v)
    L, H, S, D = base_k.shape
    assert base_v.shape == real_k.shape == real_v.shape == base_k.shape
    dk, dv = np.empty_like(base_k), np.empty_like(base_k)
    _load().kvo_capture(_dptr(base_k), _dptr(base_v), _dptr(real_k), _dptr(real_v), L, H, S, D,
                        float(delta), float(theta), _dptr(dk), _dptr(dv))
    return dk, dv


def predict(w, selected, anc_len, seg_len, gamma):
    """Anchor prediction of Eq. "pred".  w [A,n].  Returns (new_anchor 0/1, entropy [n], mean entropy)."""
    w = _f64(w)
    A, n = w.shape
    selected = np.ascontiguousarray(np.asarray(selected, dtype=np.intc))
    anc_len = np.ascontiguousarray(np.asarray(anc_len, dtype=np.intc))
    ent = np.zeros(n, dtype=np.float64)
    mean = ctypes.c_double(0.0)
    r = _load().kvo_predict(_dptr(w), _iptr(selected), _iptr(anc_len), A, n, int(seg_len), float(gamma),
                            _dptr(ent), ctypes.byref(mean))
    return int(r), ent, mean.value


def cosine(seg_k, anc_k, gran=GRAN_TOKEN):
    """Cosine similarity of base keys per weight slot.  Returns (sim [A,n], selected [A])."""
    seg_k = _f64(seg_k)
    L, H, S, D = seg_k.shape
    anc = [_f64(a) for a in anc_k]
    A = len(anc)
    anc_len = np.array([a.shape[2] for a in anc], dtype=np.intc)
    n = gran_count(gran, L, H, S)
    sim = np.zeros((A, n), dtype=np.float64)
    selected = np.zeros(A, dtype=np.intc)
    _load().kvo_cosine(_dptr(seg_k), _ptr_array(anc), _iptr(anc_len), A, L, H, S, D, gran, _dptr(sim), _iptr(selected))
    return sim, selected


def weights_from_sim(sim, selected, tau=1.0):
    """softmax(sim / tau) over selected anchors.  Returns (w [A,n], best [n])."""
    sim = _f64(sim)
    A, n = sim.shape
    selected = np.ascontiguousarray(np.asarray(selected, dtype=np.intc))
    w = np.zeros((A, n), dtype=np.float64)
    best = np.zeros(n, dtype=np.intc)
    _load().kvo_weights_from_sim(_dptr(sim), _iptr(selected), A, n, float(tau), _dptr(w), _iptr(best))
    return w, best


def weights_nearest(dist, selected):
    """One-hot weights at the selected anchor of smallest distance.  Returns (w [A,n], nearest [n])."""
    dist = _f64(dist)
    A, n = dist.shape
    selected = np.ascontiguousarray(np.asarray(selected, dtype=np.intc))
    w = np.zeros((A, n), dtype=np.float64)
    nearest = np.zeros(n, dtype=np.intc)
    _load().kvo_weights_nearest(_dptr(dist), _iptr(selected), A, n, _dptr(w), _iptr(nearest))
    return w, nearest


def e4m3_decode(byte):
    """One OCP E4M3 byte -> float (NaN for S.1111.111)."""
    return float(_load().kvo_e4m3_decode(int(byte) & 0xff))


def e4m3_encode(x):
    """Nearest E4M3 byte (ties to even, saturating at +-448)."""
    return int(_load().kvo_e4m3_encode(float(x)))


def quantize(x, scale):
    """Array -> uint8 array of E4M3 codes of x / scale."""
    x = _f64(x)
    out = np.empty(x.shape, dtype=np.uint8)
    _load().kvo_quantize(_dptr(x), x.size, float(scale), out.ctypes.data_as(ctypes.POINTER(ctypes.c_ubyte)))
    return out


def dequantize(b, scale):
    """uint8 array of E4M3 codes -> float64 array scale * value."""
    b = np.ascontiguousarray(np.asarray(b, dtype=np.uint8))
    out = np.empty(b.shape, dtype=np.float64)
    _load().kvo_dequantize(b.ctypes.data_as(ctypes.POINTER(ctypes.c_ubyte)), b.size, float(scale), _dptr(out))
    return out
