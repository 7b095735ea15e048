"""ctypes binding of libkvcomm.so: argument marshalling only.

Every function here has the name of the C entry point it calls (include/kvcomm.h) and does
nothing but turn torch tensors into (pointer, strides) descriptors, allocate outputs that
the caller did not pass, and raise on a non-zero status.  All arithmetic of the reuse step
runs inside the library's HIP kernels.  torch is used for device memory and streams only.
"""
import ctypes
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# KVCOMM_LIBRARY selects another build of the same library (e.g. a tuning variant); default: the in-tree build
_LIB_PATH = os.environ.get("KVCOMM_LIBRARY") or os.path.join(_HERE, "libkvcomm.so")

W_TOKEN = 0
W_LAYER_HEAD_TOKEN = 1
W_SEGMENT = 2
MAX_ANCHORS = 64
MAX_BATCH = 8
RULE_L2_SOFTMAX = 0
RULE_NEAREST = 1
RULE_COSINE_SOFTMAX = 2

_DTYPES = {torch.float32: 0, torch.bfloat16: 1}


class KVCommError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"libkvcomm: {message} (status {status})")
        self.status = status


class _CModel(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("dtype", ctypes.c_int32), ("rope_theta", ctypes.c_double)]


class _CTensor(ctypes.Structure):
    _fields_ = [("ptr", ctypes.c_void_p), ("stride_layer", ctypes.c_int64), ("stride_head", ctypes.c_int64),
                ("stride_token", ctypes.c_int64)]


class _CAlignJob(ctypes.Structure):
    _fields_ = [("base_k", _CTensor), ("base_v", _CTensor), ("out_k", _CTensor), ("out_v", _CTensor),
                ("seg_len", ctypes.c_int32), ("delta_pos", ctypes.c_int32),
                ("anchor_dk", ctypes.POINTER(ctypes.c_void_p)), ("anchor_dv", ctypes.POINTER(ctypes.c_void_p)),
                ("anchor_len", ctypes.POINTER(ctypes.c_int32)), ("anchor_delta_pos", ctypes.POINTER(ctypes.c_int32)),
                ("n_anchors", ctypes.c_int32), ("weights", ctypes.c_void_p), ("weights_slots", ctypes.c_int64)]


class _CAlignQ8Job(ctypes.Structure):
    _fields_ = [("base_k", _CTensor), ("base_v", _CTensor), ("out_k", _CTensor), ("out_v", _CTensor),
                ("seg_len", ctypes.c_int32), ("delta_pos", ctypes.c_int32),
                ("anchor_dk", ctypes.POINTER(ctypes.c_void_p)), ("anchor_dv", ctypes.POINTER(ctypes.c_void_p)),
                ("anchor_len", ctypes.POINTER(ctypes.c_int32)), ("anchor_delta_pos", ctypes.POINTER(ctypes.c_int32)),
                ("anchor_scale_k", ctypes.POINTER(ctypes.c_float)), ("anchor_scale_v", ctypes.POINTER(ctypes.c_float)),
                ("n_anchors", ctypes.c_int32), ("weights", ctypes.c_void_p), ("weights_slots", ctypes.c_int64)]


class _CWeightsJob(ctypes.Structure):
    _fields_ = [("seg_base_k", _CTensor), ("seg_len", ctypes.c_int32),
                ("anchor_base_k", ctypes.POINTER(ctypes.c_void_p)), ("anchor_len", ctypes.POINTER(ctypes.c_int32)),
                ("n_anchors", ctypes.c_int32), ("weights_out", ctypes.c_void_p), ("nearest_out", ctypes.c_void_p),
                ("selected_out", ctypes.c_void_p)]


@dataclass(frozen=True)
class Model:
    """Shape of the model whose KV-cache is handled (kvcomm_model of the C header)."""
    n_layers: int
    n_kv_heads: int
    n_q_heads: int
    head_dim: int
    dtype: torch.dtype
    rope_theta: float

    def c(self):
        if self.dtype not in _DTYPES:
            raise KVCommError(-2, f"unsupported dtype {self.dtype}")
        return _CModel(self.n_layers, self.n_kv_heads, self.n_q_heads, self.head_dim, _DTYPES[self.dtype],
                       float(self.rope_theta))


_lib = None


def library_path():
    return _LIB_PATH


def load_library():
    """Load libkvcomm.so (built by paper_2510_12872_amd.build); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2510_12872_amd.build` "
                           "(there is no fallback path)")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
    mp = ctypes.POINTER(_CModel)
    lib.kvcomm_weight_slots.argtypes = [mp, i32, i32]
    lib.kvcomm_weight_slots.restype = sz
    lib.kvcomm_anchor_weights_workspace.argtypes = [mp, i32, i32, i32]
    lib.kvcomm_anchor_weights_workspace.restype = sz
    lib.kvcomm_anchor_weights.argtypes = [mp, i32, f32, _CTensor, i32, ctypes.POINTER(vp), _CTensor,
                                          ctypes.POINTER(i32), i32, vp, vp, vp, vp, sz, vp]
    lib.kvcomm_anchor_weights.restype = ctypes.c_int
    lib.kvcomm_anchor_weights_static_capacity.argtypes = []
    lib.kvcomm_anchor_weights_static_capacity.restype = sz
    lib.kvcomm_anchor_weights_static.argtypes = [mp, i32, f32, _CTensor, i32, ctypes.POINTER(vp), _CTensor,
                                                 ctypes.POINTER(i32), i32, vp, vp, vp, vp]
    lib.kvcomm_anchor_weights_static.restype = ctypes.c_int
    lib.kvcomm_align_kv.argtypes = [mp, i32, _CTensor, _CTensor, i32, ctypes.POINTER(vp), ctypes.POINTER(vp),
                                    _CTensor, ctypes.POINTER(i32), i32, vp, i32, ctypes.POINTER(i32),
                                    _CTensor, _CTensor, vp]
    lib.kvcomm_align_kv.restype = ctypes.c_int
    lib.kvcomm_suffix_attn_workspace.argtypes = [mp, i32, i32]
    lib.kvcomm_suffix_attn_workspace.restype = sz
    lib.kvcomm_suffix_attn.argtypes = [mp, _CTensor, _CTensor, _CTensor, i32, i32, f32, _CTensor, vp, vp, sz, vp]
    lib.kvcomm_suffix_attn.restype = ctypes.c_int
    lib.kvcomm_suffix_attn_confined.argtypes = [mp, _CTensor, _CTensor, _CTensor, i32, i32, f32, _CTensor, vp, i32, vp]
    lib.kvcomm_suffix_attn_confined.restype = ctypes.c_int
    lib.kvcomm_anchor_weights_rule_workspace.argtypes = [mp, i32, i32, i32, i32]
    lib.kvcomm_anchor_weights_rule_workspace.restype = sz
    lib.kvcomm_anchor_weights_rule.argtypes = [mp, i32, i32, f32, _CTensor, i32, ctypes.POINTER(vp), _CTensor,
                                               ctypes.POINTER(i32), i32, vp, vp, vp, vp, sz, vp]
    lib.kvcomm_anchor_weights_rule.restype = ctypes.c_int
    lib.kvcomm_anchor_predict_workspace.argtypes = [ctypes.c_int64]
    lib.kvcomm_anchor_predict_workspace.restype = sz
    lib.kvcomm_anchor_predict.argtypes = [vp, ctypes.c_int64, ctypes.POINTER(i32), i32, i32, f32, vp, vp, vp, sz, vp]
    lib.kvcomm_anchor_predict.restype = ctypes.c_int
    lib.kvcomm_capture_offsets.argtypes = [mp, _CTensor, _CTensor, _CTensor, _CTensor, i32, i32, _CTensor, _CTensor,
                                           vp]
    lib.kvcomm_capture_offsets.restype = ctypes.c_int
    lib.kvcomm_align_kv_batch.argtypes = [mp, i32, _CTensor, ctypes.POINTER(_CAlignJob), i32, vp]
    lib.kvcomm_align_kv_batch.restype = ctypes.c_int
    lib.kvcomm_anchor_weights_batch_workspace.argtypes = [mp, i32, i32, ctypes.POINTER(i32), ctypes.POINTER(i32), i32]
    lib.kvcomm_anchor_weights_batch_workspace.restype = sz
    lib.kvcomm_anchor_weights_batch.argtypes = [mp, i32, i32, f32, _CTensor, ctypes.POINTER(_CWeightsJob), i32, vp,
                                                sz, vp]
    lib.kvcomm_anchor_weights_batch.restype = ctypes.c_int
    lib.kvcomm_quantize_deltas.argtypes = [mp, _CTensor, i32, f32, _CTensor, vp]
    lib.kvcomm_quantize_deltas.restype = ctypes.c_int
    lib.kvcomm_align_kv_q8.argtypes = [mp, i32, _CTensor, _CTensor, i32, ctypes.POINTER(vp), ctypes.POINTER(vp),
                                       _CTensor, ctypes.POINTER(i32), ctypes.POINTER(f32), ctypes.POINTER(f32), i32,
                                       vp, i32, ctypes.POINTER(i32), _CTensor, _CTensor, vp]
    lib.kvcomm_align_kv_q8.restype = ctypes.c_int
    lib.kvcomm_align_kv_q8_batch.argtypes = [mp, i32, _CTensor, ctypes.POINTER(_CAlignQ8Job), i32, vp]
    lib.kvcomm_align_kv_q8_batch.restype = ctypes.c_int
    lib.kvcomm_status_string.argtypes = [ctypes.c_int]
    lib.kvcomm_status_string.restype = ctypes.c_char_p
    lib.kvcomm_version.argtypes = []
    lib.kvcomm_version.restype = ctypes.c_int
    _lib = lib
    return lib


def _check(status):
    if status != 0:
        raise KVCommError(status, load_library().kvcomm_status_string(status).decode())


def _desc(t, dtype, what):
    """[layer, head, token, channel] tensor -> kvcomm_tensor."""
    if t.dim() != 4 or t.dtype != dtype or not t.is_cuda or t.stride(3) != 1:
        raise KVCommError(-1, f"{what}: expected a 4-d {dtype} device tensor with contiguous channels")
    return _CTensor(t.data_ptr(), t.stride(0), t.stride(1), t.stride(2))


def _stream_ptr(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _anchor_args(anchors, anchor_len, dtype, what):
    """List of same-layout anchor tensors -> (host pointer array, layout descriptor, host length array)."""
    n = len(anchors)
    if n == 0:
        return None, _CTensor(None, 0, 0, 0), None
    layout = _desc(anchors[0], dtype, what)
    for a in anchors:
        d = _desc(a, dtype, what)
        if (d.stride_layer, d.stride_head, d.stride_token) != (layout.stride_layer, layout.stride_head,
                                                               layout.stride_token):
            raise KVCommError(-1, f"{what}: all anchors must share one layout (pad them to a common capacity)")
    ptrs = (ctypes.c_void_p * n)(*[a.data_ptr() for a in anchors])
    if anchor_len is None:
        anchor_len = [a.shape[2] for a in anchors]
    lens = (ctypes.c_int32 * n)(*[int(x) for x in anchor_len])
    return ptrs, layout, lens


def kvcomm_weight_slots(model, seg_len, gran=W_TOKEN):
    return int(load_library().kvcomm_weight_slots(ctypes.byref(model.c()), seg_len, gran))


def kvcomm_anchor_weights_workspace(model, seg_len, n_anchors, gran=W_TOKEN):
    return int(load_library().kvcomm_anchor_weights_workspace(ctypes.byref(model.c()), seg_len, n_anchors, gran))


def kvcomm_anchor_weights(model, seg_base_k, anchor_base_k, anchor_len=None, temperature=1.0, gran=W_TOKEN,
                          weights_out=None, nearest_out=None, selected_out=None, workspace=None, stream=None):
    """Anchor matching.  Returns (weights [n, A] fp32, nearest [n] int32, selected [A] int32)."""
    lib = load_library()
    seg_len = seg_base_k.shape[2]
    A = len(anchor_base_k)
    dev = seg_base_k.device
    n = kvcomm_weight_slots(model, seg_len, gran)
    if weights_out is None:
        weights_out = torch.empty((n, A), dtype=torch.float32, device=dev)
    if nearest_out is None:
        nearest_out = torch.empty((n,), dtype=torch.int32, device=dev)
    if selected_out is None:
        selected_out = torch.empty((A,), dtype=torch.int32, device=dev)
    need = kvcomm_anchor_weights_workspace(model, seg_len, A, gran)
    if workspace is None:
        workspace = torch.empty((max(need, 1),), dtype=torch.uint8, device=dev)
    ptrs, layout, lens = _anchor_args(anchor_base_k, anchor_len, model.dtype, "anchor_base_k")
    _check(lib.kvcomm_anchor_weights(ctypes.byref(model.c()), gran, float(temperature),
                                     _desc(seg_base_k, model.dtype, "seg_base_k"), seg_len, ptrs, layout, lens, A,
                                     weights_out.data_ptr(), nearest_out.data_ptr(), selected_out.data_ptr(),
                                     workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                     _stream_ptr(stream)))
    return weights_out, nearest_out, selected_out


def kvcomm_anchor_weights_static_capacity():
    return int(load_library().kvcomm_anchor_weights_static_capacity())


def kvcomm_anchor_weights_static(model, seg_base_k, anchor_base_k, weights_out, nearest_out, selected_out,
                                 anchor_len=None, temperature=1.0, gran=W_TOKEN, stream=None):
    """kvcomm_anchor_weights without a workspace argument (the library's fixed scratch array).  The caller
    passes every output; nothing is allocated here or in the library."""
    lib = load_library()
    ptrs, layout, lens = _anchor_args(anchor_base_k, anchor_len, model.dtype, "anchor_base_k")
    _check(lib.kvcomm_anchor_weights_static(ctypes.byref(model.c()), gran, float(temperature),
                                            _desc(seg_base_k, model.dtype, "seg_base_k"), seg_base_k.shape[2], ptrs,
                                            layout, lens, len(anchor_base_k), weights_out.data_ptr(),
                                            None if nearest_out is None else nearest_out.data_ptr(),
                                            None if selected_out is None else selected_out.data_ptr(),
                                            _stream_ptr(stream)))
    return weights_out, nearest_out, selected_out


def kvcomm_align_kv(model, base_k, base_v, anchor_dk, anchor_dv, weights, delta_pos, out_k, out_v,
                    anchor_len=None, anchor_delta_pos=None, gran=W_TOKEN, stream=None):
    """Positional alignment + offset approximation into out_k / out_v (views of the agent cache)."""
    lib = load_library()
    seg_len = base_k.shape[2]
    A = len(anchor_dk)
    if len(anchor_dv) != A:
        raise KVCommError(-1, "anchor_dk and anchor_dv differ in length")
    pk, layout, lens = _anchor_args(anchor_dk, anchor_len, model.dtype, "anchor_dk")
    pv, layout_v, _ = _anchor_args(anchor_dv, anchor_len, model.dtype, "anchor_dv")
    if A and (layout.stride_layer, layout.stride_head, layout.stride_token) != (
            layout_v.stride_layer, layout_v.stride_head, layout_v.stride_token):
        raise KVCommError(-1, "anchor_dk and anchor_dv must share one layout")
    adp = None
    if anchor_delta_pos is not None:
        if len(anchor_delta_pos) != A:
            raise KVCommError(-1, "anchor_delta_pos must have one entry per anchor")
        adp = (ctypes.c_int32 * max(A, 1))(*[int(x) for x in anchor_delta_pos])
    if A:
        if weights is None or weights.dtype != torch.float32 or not weights.is_contiguous():
            raise KVCommError(-1, "weights: expected a contiguous fp32 device tensor [n, A]")
        if weights.numel() != kvcomm_weight_slots(model, seg_len, gran) * A:
            raise KVCommError(-1, "weights: wrong number of elements for this granularity")
    _check(lib.kvcomm_align_kv(ctypes.byref(model.c()), gran, _desc(base_k, model.dtype, "base_k"),
                               _desc(base_v, model.dtype, "base_v"), seg_len, pk, pv, layout, lens, A,
                               None if weights is None else weights.data_ptr(), int(delta_pos), adp,
                               _desc(out_k, model.dtype, "out_k"), _desc(out_v, model.dtype, "out_v"),
                               _stream_ptr(stream)))
    return out_k, out_v


def kvcomm_suffix_attn_workspace(model, n_ctx, tq):
    return int(load_library().kvcomm_suffix_attn_workspace(ctypes.byref(model.c()), int(n_ctx), int(tq)))


def kvcomm_suffix_attn(model, q, cache_k, cache_v, n_ctx, softmax_scale=0.0, out=None, lse_out=None,
                       want_lse=False, stream=None):
    """Causal attention of the suffix queries q [L,Hq,Tq,D] over cache_k/v [L,Hkv,n_ctx+Tq,D]."""
    lib = load_library()
    tq = q.shape[2]
    if cache_k.shape[2] != n_ctx + tq or cache_v.shape[2] != n_ctx + tq:
        raise KVCommError(-1, "cache_k / cache_v must hold n_ctx + tq tokens")
    if out is None:
        out = torch.empty_like(q)
    if want_lse and lse_out is None:
        lse_out = torch.empty(q.shape[:3], dtype=torch.float32, device=q.device)
    _check(lib.kvcomm_suffix_attn(ctypes.byref(model.c()), _desc(q, model.dtype, "q"),
                                  _desc(cache_k, model.dtype, "cache_k"), _desc(cache_v, model.dtype, "cache_v"),
                                  int(n_ctx), tq, float(softmax_scale), _desc(out, model.dtype, "out"),
                                  None if lse_out is None else lse_out.data_ptr(), None, 0, _stream_ptr(stream)))
    return (out, lse_out) if want_lse else out


def kvcomm_suffix_attn_confined(model, q, cache_k, cache_v, n_ctx, max_blocks, softmax_scale=0.0, out=None,
                                lse_out=None, want_lse=False, stream=None):
    """kvcomm_suffix_attn as at most max_blocks persistent thread blocks (one per compute unit)."""
    lib = load_library()
    tq = q.shape[2]
    if cache_k.shape[2] != n_ctx + tq or cache_v.shape[2] != n_ctx + tq:
        raise KVCommError(-1, "cache_k / cache_v must hold n_ctx + tq tokens")
    if out is None:
        out = torch.empty_like(q)
    if want_lse and lse_out is None:
        lse_out = torch.empty(q.shape[:3], dtype=torch.float32, device=q.device)
    _check(lib.kvcomm_suffix_attn_confined(ctypes.byref(model.c()), _desc(q, model.dtype, "q"),
                                           _desc(cache_k, model.dtype, "cache_k"),
                                           _desc(cache_v, model.dtype, "cache_v"), int(n_ctx), tq,
                                           float(softmax_scale), _desc(out, model.dtype, "out"),
                                           None if lse_out is None else lse_out.data_ptr(), int(max_blocks),
                                           _stream_ptr(stream)))
    return (out, lse_out) if want_lse else out


def kvcomm_anchor_weights_rule_workspace(model, seg_len, n_anchors, gran=W_TOKEN, rule=RULE_L2_SOFTMAX):
    return int(load_library().kvcomm_anchor_weights_rule_workspace(ctypes.byref(model.c()), seg_len, n_anchors, gran,
                                                                   rule))


def kvcomm_anchor_weights_rule(model, rule, seg_base_k, anchor_base_k, anchor_len=None, temperature=1.0, gran=W_TOKEN,
                               weights_out=None, nearest_out=None, selected_out=None, workspace=None, stream=None):
    """Anchor matching under one of the weighting variants.  Returns (weights, nearest, selected)."""
    lib = load_library()
    seg_len = seg_base_k.shape[2]
    A = len(anchor_base_k)
    dev = seg_base_k.device
    n = kvcomm_weight_slots(model, seg_len, gran)
    if weights_out is None:
        weights_out = torch.empty((n, A), dtype=torch.float32, device=dev)
    if nearest_out is None:
        nearest_out = torch.empty((n,), dtype=torch.int32, device=dev)
    if selected_out is None:
        selected_out = torch.empty((A,), dtype=torch.int32, device=dev)
    if workspace is None:
        need = kvcomm_anchor_weights_rule_workspace(model, seg_len, A, gran, rule)
        workspace = torch.empty((max(need, 1),), dtype=torch.uint8, device=dev)
    ptrs, layout, lens = _anchor_args(anchor_base_k, anchor_len, model.dtype, "anchor_base_k")
    _check(lib.kvcomm_anchor_weights_rule(ctypes.byref(model.c()), gran, int(rule), float(temperature),
                                          _desc(seg_base_k, model.dtype, "seg_base_k"), seg_len, ptrs, layout, lens,
                                          A, weights_out.data_ptr(), nearest_out.data_ptr(), selected_out.data_ptr(),
                                          workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                          _stream_ptr(stream)))
    return weights_out, nearest_out, selected_out


def kvcomm_anchor_predict_workspace(n_slots):
    return int(load_library().kvcomm_anchor_predict_workspace(int(n_slots)))


def kvcomm_anchor_predict(weights, anchor_len, seg_len, gamma, entropy_out=None, result_out=None, workspace=None,
                          want_entropy=False, stream=None):
    """Eq. "pred" on the device.  weights [n, A] fp32.  Returns result [2] (decision, mean entropy)
    and, with want_entropy, the per-slot entropies [n]."""
    lib = load_library()
    if weights.dim() != 2 or weights.dtype != torch.float32 or not weights.is_contiguous() or not weights.is_cuda:
        raise KVCommError(-1, "weights: expected a contiguous fp32 device tensor [n, A]")
    n, A = weights.shape
    if len(anchor_len) != A:
        raise KVCommError(-1, "anchor_len must have one entry per anchor")
    dev = weights.device
    if want_entropy and entropy_out is None:
        entropy_out = torch.empty((n,), dtype=torch.float32, device=dev)
    if result_out is None:
        result_out = torch.empty((2,), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = torch.empty((max(kvcomm_anchor_predict_workspace(n), 8),), dtype=torch.uint8, device=dev)
    lens = (ctypes.c_int32 * max(A, 1))(*[int(x) for x in anchor_len])
    _check(lib.kvcomm_anchor_predict(weights.data_ptr(), n, lens, A, int(seg_len), float(gamma),
                                     None if entropy_out is None else entropy_out.data_ptr(), result_out.data_ptr(),
                                     workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                     _stream_ptr(stream)))
    return (result_out, entropy_out) if want_entropy else result_out


def kvcomm_capture_offsets(model, base_k, base_v, real_k, real_v, delta_pos, out_dk=None, out_dv=None, stream=None):
    """Offset capture: (real - re-positioned base) for keys and values of one segment."""
    lib = load_library()
    seg_len = base_k.shape[2]
    for t in (base_v, real_k, real_v):
        if t.shape != base_k.shape:
            raise KVCommError(-1, "base and real tensors must have one shape")
    if out_dk is None:
        out_dk = torch.empty(base_k.shape, dtype=model.dtype, device=base_k.device)
    if out_dv is None:
        out_dv = torch.empty(base_k.shape, dtype=model.dtype, device=base_k.device)
    d = lambda t, what: _desc(t, model.dtype, what)
    _check(lib.kvcomm_capture_offsets(ctypes.byref(model.c()), d(base_k, "base_k"), d(base_v, "base_v"),
                                      d(real_k, "real_k"), d(real_v, "real_v"), seg_len, int(delta_pos),
                                      d(out_dk, "out_dk"), d(out_dv, "out_dv"), _stream_ptr(stream)))
    return out_dk, out_dv


def _same_layout(a, b):
    return (a.stride_layer, a.stride_head, a.stride_token) == (b.stride_layer, b.stride_head, b.stride_token)


def kvcomm_anchor_weights_batch_workspace(model, seg_lens, n_anchors, gran=W_TOKEN, rule=RULE_L2_SOFTMAX):
    n = len(seg_lens)
    sl = (ctypes.c_int32 * n)(*[int(x) for x in seg_lens])
    na = (ctypes.c_int32 * n)(*[int(x) for x in n_anchors])
    return int(load_library().kvcomm_anchor_weights_batch_workspace(ctypes.byref(model.c()), gran, rule, sl, na, n))


def kvcomm_anchor_weights_batch(model, jobs, temperature=1.0, gran=W_TOKEN, rule=RULE_L2_SOFTMAX, workspace=None,
                                stream=None):
    """Anchor matching of several segments in one launch per stage.

    jobs: list of dicts with seg_base_k, anchor_base_k (list of tensors) and optionally anchor_len,
    weights_out, nearest_out, selected_out.  Returns a list of (weights, nearest, selected)."""
    lib = load_library()
    n = len(jobs)
    cjobs = (_CWeightsJob * max(n, 1))()
    keep, outs, layout = [], [], None
    for j, jd in enumerate(jobs):
        seg = jd["seg_base_k"]
        S, A, dev = seg.shape[2], len(jd["anchor_base_k"]), seg.device
        slots = kvcomm_weight_slots(model, S, gran)
        w = jd.get("weights_out")
        w = torch.empty((slots, A), dtype=torch.float32, device=dev) if w is None else w
        nr = jd.get("nearest_out")
        nr = torch.empty((slots,), dtype=torch.int32, device=dev) if nr is None else nr
        so = jd.get("selected_out")
        so = torch.empty((A,), dtype=torch.int32, device=dev) if so is None else so
        ptrs, lay, lens = _anchor_args(jd["anchor_base_k"], jd.get("anchor_len"), model.dtype, "anchor_base_k")
        if layout is None:
            layout = lay
        elif A and not _same_layout(layout, lay):
            raise KVCommError(-1, "all anchors of a batched call must share one layout")
        keep.append((ptrs, lens))
        cjobs[j] = _CWeightsJob(_desc(seg, model.dtype, "seg_base_k"), S, ptrs, lens, A, w.data_ptr(), nr.data_ptr(),
                                so.data_ptr())
        outs.append((w, nr, so))
    if workspace is None:
        need = kvcomm_anchor_weights_batch_workspace(model, [jd["seg_base_k"].shape[2] for jd in jobs],
                                                     [len(jd["anchor_base_k"]) for jd in jobs], gran, rule)
        workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=jobs[0]["seg_base_k"].device)
    _check(lib.kvcomm_anchor_weights_batch(ctypes.byref(model.c()), gran, int(rule), float(temperature),
                                           layout if layout is not None else _CTensor(None, 0, 0, 0), cjobs, n,
                                           workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                           _stream_ptr(stream)))
    return outs


def kvcomm_align_kv_batch(model, jobs, gran=W_TOKEN, stream=None):
    """Positional alignment + offset approximation of several segments in one launch.

    jobs: list of dicts with base_k, base_v, anchor_dk, anchor_dv (lists of tensors), weights, delta_pos,
    out_k, out_v and optionally anchor_len, anchor_delta_pos."""
    lib = load_library()
    n = len(jobs)
    cjobs = (_CAlignJob * max(n, 1))()
    keep, layout = [], None
    for j, jd in enumerate(jobs):
        A = len(jd["anchor_dk"])
        if len(jd["anchor_dv"]) != A:
            raise KVCommError(-1, "anchor_dk and anchor_dv differ in length")
        pk, lay, lens = _anchor_args(jd["anchor_dk"], jd.get("anchor_len"), model.dtype, "anchor_dk")
        pv, lay_v, _ = _anchor_args(jd["anchor_dv"], jd.get("anchor_len"), model.dtype, "anchor_dv")
        if A:
            if not _same_layout(lay, lay_v) or (layout is not None and not _same_layout(layout, lay)):
                raise KVCommError(-1, "all anchors of a batched call must share one layout")
            layout = lay
        adp = None
        if jd.get("anchor_delta_pos") is not None:
            if len(jd["anchor_delta_pos"]) != A:
                raise KVCommError(-1, "anchor_delta_pos must have one entry per anchor")
            adp = (ctypes.c_int32 * max(A, 1))(*[int(x) for x in jd["anchor_delta_pos"]])
        w = jd.get("weights")
        S = jd["base_k"].shape[2]
        if A:
            if w is None or w.dtype != torch.float32 or not w.is_contiguous():
                raise KVCommError(-1, "weights: expected a contiguous fp32 device tensor [n, A]")
            if w.numel() % A:
                raise KVCommError(-1, "weights: expected [n, A]")
        keep.append((pk, pv, lens, adp))
        d = lambda t, what: _desc(t, model.dtype, what)
        cjobs[j] = _CAlignJob(d(jd["base_k"], "base_k"), d(jd["base_v"], "base_v"), d(jd["out_k"], "out_k"),
                              d(jd["out_v"], "out_v"), S, int(jd["delta_pos"]), pk, pv, lens, adp, A,
                              None if w is None else w.data_ptr(), 0 if (w is None or not A) else w.numel() // A)
    _check(lib.kvcomm_align_kv_batch(ctypes.byref(model.c()), gran,
                                     layout if layout is not None else _CTensor(None, 0, 0, 0), cjobs, n,
                                     _stream_ptr(stream)))


def _desc_q8(t, what):
    """[layer, head, token, channel] uint8 tensor of E4M3 codes -> kvcomm_tensor (strides in bytes)."""
    if t.dim() != 4 or t.dtype != torch.uint8 or not t.is_cuda or t.stride(3) != 1:
        raise KVCommError(-1, f"{what}: expected a 4-d uint8 device tensor with contiguous channels")
    return _CTensor(t.data_ptr(), t.stride(0), t.stride(1), t.stride(2))


def kvcomm_quantize_deltas(model, x, scale, out=None, stream=None):
    """Stored deviation x [L,Hkv,n,D] (model dtype) -> E4M3 codes (uint8) of x / scale; scale a power of two."""
    lib = load_library()
    if out is None:
        out = torch.empty(x.shape, dtype=torch.uint8, device=x.device)
    _check(lib.kvcomm_quantize_deltas(ctypes.byref(model.c()), _desc(x, model.dtype, "x"), x.shape[2], float(scale),
                                      _desc_q8(out, "out"), _stream_ptr(stream)))
    return out


def kvcomm_align_kv_q8(model, base_k, base_v, anchor_dk8, anchor_dv8, scale_k, scale_v, weights, delta_pos, out_k,
                       out_v, anchor_len=None, anchor_delta_pos=None, gran=W_TOKEN, stream=None):
    """kvcomm_align_kv with E4M3-compressed deviations (uint8 tensors) and their per-anchor scales."""
    lib = load_library()
    seg_len = base_k.shape[2]
    A = len(anchor_dk8)
    if len(anchor_dv8) != A or len(scale_k) != A or len(scale_v) != A:
        raise KVCommError(-1, "anchor lists and scales differ in length")
    if A:
        layout = _desc_q8(anchor_dk8[0], "anchor_dk8")
        for a in list(anchor_dk8) + list(anchor_dv8):
            if not _same_layout(layout, _desc_q8(a, "anchor deviations")):
                raise KVCommError(-1, "all compressed anchors must share one layout")
        pk = (ctypes.c_void_p * A)(*[a.data_ptr() for a in anchor_dk8])
        pv = (ctypes.c_void_p * A)(*[a.data_ptr() for a in anchor_dv8])
        lens = (ctypes.c_int32 * A)(*[int(x) for x in (anchor_len if anchor_len is not None
                                                        else [a.shape[2] for a in anchor_dk8])])
        sk = (ctypes.c_float * A)(*[float(x) for x in scale_k])
        sv = (ctypes.c_float * A)(*[float(x) for x in scale_v])
        if weights is None or weights.dtype != torch.float32 or not weights.is_contiguous():
            raise KVCommError(-1, "weights: expected a contiguous fp32 device tensor [n, A]")
        if weights.numel() != kvcomm_weight_slots(model, seg_len, gran) * A:
            raise KVCommError(-1, "weights: wrong number of elements for this granularity")
    else:
        layout, pk, pv, lens, sk, sv = _CTensor(None, 0, 0, 0), None, None, None, None, None
    adp = None
    if anchor_delta_pos is not None:
        adp = (ctypes.c_int32 * max(A, 1))(*[int(x) for x in anchor_delta_pos])
    _check(lib.kvcomm_align_kv_q8(ctypes.byref(model.c()), gran, _desc(base_k, model.dtype, "base_k"),
                                  _desc(base_v, model.dtype, "base_v"), seg_len, pk, pv, layout, lens, sk, sv, A,
                                  None if weights is None else weights.data_ptr(), int(delta_pos), adp,
                                  _desc(out_k, model.dtype, "out_k"), _desc(out_v, model.dtype, "out_v"),
                                  _stream_ptr(stream)))
    return out_k, out_v


def kvcomm_align_kv_q8_batch(model, jobs, gran=W_TOKEN, stream=None):
    """The compressed update of several segments in one launch.

    jobs: list of dicts with base_k, base_v, anchor_dk8, anchor_dv8 (lists of uint8 tensors), scale_k, scale_v
    (lists of floats), weights, delta_pos, out_k, out_v and optionally anchor_len, anchor_delta_pos."""
    lib = load_library()
    n = len(jobs)
    cjobs = (_CAlignQ8Job * max(n, 1))()
    keep, layout = [], None
    for j, jd in enumerate(jobs):
        dk8, dv8 = jd["anchor_dk8"], jd["anchor_dv8"]
        A = len(dk8)
        if len(dv8) != A or len(jd["scale_k"]) != A or len(jd["scale_v"]) != A:
            raise KVCommError(-1, "anchor lists and scales differ in length")
        pk = pv = lens = sk = sv = adp = None
        if A:
            lay = _desc_q8(dk8[0], "anchor_dk8")
            for a in list(dk8) + list(dv8):
                if not _same_layout(lay, _desc_q8(a, "anchor deviations")):
                    raise KVCommError(-1, "all compressed anchors must share one layout")
            if layout is not None and not _same_layout(layout, lay):
                raise KVCommError(-1, "all anchors of a batched call must share one layout")
            layout = lay
            pk = (ctypes.c_void_p * A)(*[a.data_ptr() for a in dk8])
            pv = (ctypes.c_void_p * A)(*[a.data_ptr() for a in dv8])
            al = jd.get("anchor_len")
            lens = (ctypes.c_int32 * A)(*[int(x) for x in (al if al is not None else [a.shape[2] for a in dk8])])
            sk = (ctypes.c_float * A)(*[float(x) for x in jd["scale_k"]])
            sv = (ctypes.c_float * A)(*[float(x) for x in jd["scale_v"]])
        if jd.get("anchor_delta_pos") is not None:
            if len(jd["anchor_delta_pos"]) != A:
                raise KVCommError(-1, "anchor_delta_pos must have one entry per anchor")
            adp = (ctypes.c_int32 * max(A, 1))(*[int(x) for x in jd["anchor_delta_pos"]])
        w = jd.get("weights")
        if A and (w is None or w.dtype != torch.float32 or not w.is_contiguous() or w.numel() % A):
            raise KVCommError(-1, "weights: expected a contiguous fp32 device tensor [n, A]")
        keep.append((pk, pv, lens, sk, sv, adp))
        d = lambda t, what: _desc(t, model.dtype, what)
        cjobs[j] = _CAlignQ8Job(d(jd["base_k"], "base_k"), d(jd["base_v"], "base_v"), d(jd["out_k"], "out_k"),
                                d(jd["out_v"], "out_v"), jd["base_k"].shape[2], int(jd["delta_pos"]), pk, pv, lens, adp,
                                sk, sv, A, None if w is None else w.data_ptr(),
                                0 if (w is None or not A) else w.numel() // A)
    _check(lib.kvcomm_align_kv_q8_batch(ctypes.byref(model.c()), gran,
                                        layout if layout is not None else _CTensor(None, 0, 0, 0), cjobs, n,
                                        _stream_ptr(stream)))
