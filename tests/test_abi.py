"""CPU-only checks of the C-ABI boundary: the built library loads without a GPU, exports every
symbol the header declares, and turns bad arguments into status codes on the host before
anything is enqueued (so none of these calls touches a device)."""
import ctypes
import os
import re

import pytest
import torch

import paper_2510_12872_amd as kv
from paper_2510_12872_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "kvcomm.h")

EINVAL, EUNSUPPORTED, EWORKSPACE = -1, -2, -3


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(kv.library_path()):
        from paper_2510_12872_amd import build
        build.build()
    return kv.load_library()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kvcomm_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = declared_functions()
    assert {"kvcomm_anchor_weights", "kvcomm_align_kv", "kvcomm_suffix_attn", "kvcomm_anchor_weights_workspace",
            "kvcomm_suffix_attn_workspace", "kvcomm_weight_slots", "kvcomm_status_string",
            "kvcomm_version"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in kvcomm.h but not exported"
    assert lib.kvcomm_version() >= 120
    for st in (0, -1, -2, -3, -4, 17):
        assert lib.kvcomm_status_string(st)


def test_every_entry_point_has_a_binding_of_the_same_name():
    """The Python layer is a thin binding: one function per C entry point, same name."""
    for n in declared_functions():
        if n in ("kvcomm_status_string", "kvcomm_version"):
            continue                      # used through load_library() / KVCommError
        assert callable(getattr(kv, n, None)), f"{n} has no binding of the same name"


def test_header_is_plain_c(tmp_path):
    src = tmp_path / "t.c"
    src.write_text('#include "kvcomm.h"\nint main(void){ kvcomm_model m; (void)m; return KVCOMM_MAX_ANCHORS == 64 ? 0 : 1; }\n')
    import subprocess
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    "-c", str(src), "-o", str(tmp_path / "t.o")], check=True)


def _model(**kw):
    d = dict(n_layers=2, n_kv_heads=2, n_q_heads=4, head_dim=128, dtype=1, rope_theta=5e5)
    d.update(kw)
    return binding._CModel(d["n_layers"], d["n_kv_heads"], d["n_q_heads"], d["head_dim"], d["dtype"], d["rope_theta"])


def _tensor(ptr=0x1000, sl=1 << 20, sh=1 << 16, st=128):
    return binding._CTensor(ptr, sl, sh, st)


def _aw(lib, m, gran=0, tau=1.0, seg=None, seg_len=16, ptrs=(0x2000, 0x3000), lens=(16, 16), layout=None,
        weights=0x4000, ws=0x10000, ws_bytes=1 << 30):
    A = len(ptrs)
    parr = (ctypes.c_void_p * max(A, 1))(*ptrs)
    larr = (ctypes.c_int32 * max(A, 1))(*lens)
    return lib.kvcomm_anchor_weights(ctypes.byref(m), gran, tau, seg or _tensor(), seg_len, parr,
                                     layout or _tensor(None), larr, A, weights, None, None, ws, ws_bytes, None)


def test_model_validation(lib):
    assert _aw(lib, _model(head_dim=96)) == EUNSUPPORTED
    assert _aw(lib, _model(head_dim=0)) == EINVAL
    assert _aw(lib, _model(n_q_heads=3)) == EUNSUPPORTED
    assert _aw(lib, _model(dtype=7)) == EINVAL
    assert _aw(lib, _model(rope_theta=0.0)) == EINVAL
    assert _aw(lib, _model(n_layers=0)) == EINVAL
    assert lib.kvcomm_anchor_weights(None, 0, 1.0, _tensor(), 16, None, _tensor(None), None, 1, None, None, None,
                                     None, 0, None) == EINVAL


def test_anchor_weights_argument_errors(lib):
    m = _model()
    assert _aw(lib, m, tau=0.0) == EINVAL
    assert _aw(lib, m, tau=-1.0) == EINVAL
    assert _aw(lib, m, tau=float("nan")) == EINVAL
    assert _aw(lib, m, gran=3) == EINVAL
    assert _aw(lib, m, seg_len=0) == EINVAL
    assert _aw(lib, m, ptrs=(), lens=()) == EINVAL
    assert _aw(lib, m, ptrs=(0x2000,) * 65, lens=(16,) * 65) == EUNSUPPORTED
    assert _aw(lib, m, seg=_tensor(ptr=None)) == EINVAL
    assert _aw(lib, m, seg=_tensor(ptr=0x1008)) == EINVAL          # not 16-byte aligned
    assert _aw(lib, m, seg=_tensor(st=4)) == EINVAL                # token stride not a multiple of 8 bf16
    assert _aw(lib, m, ptrs=(0x2000, 0x3004)) == EINVAL            # misaligned selected anchor
    assert _aw(lib, m, ptrs=(0x2000, 0)) == EINVAL                 # null selected anchor
    assert _aw(lib, m, lens=(16, -1)) == EINVAL
    assert _aw(lib, m, weights=None) == EINVAL
    assert _aw(lib, m, ws=None) == EWORKSPACE
    assert _aw(lib, m, ws=0x10010) == EWORKSPACE                   # not 256-byte aligned
    need = lib.kvcomm_anchor_weights_workspace(ctypes.byref(m), 16, 2, 0)
    assert need > 0
    assert _aw(lib, m, ws_bytes=need - 1) == EWORKSPACE


def test_workspace_and_slot_queries(lib):
    m = _model()
    assert lib.kvcomm_weight_slots(ctypes.byref(m), 100, 0) == 100
    assert lib.kvcomm_weight_slots(ctypes.byref(m), 100, 1) == 2 * 2 * 100
    assert lib.kvcomm_weight_slots(ctypes.byref(m), 100, 2) == 1
    assert lib.kvcomm_weight_slots(ctypes.byref(m), 0, 0) == 0
    assert lib.kvcomm_weight_slots(ctypes.byref(m), 100, 5) == 0
    assert lib.kvcomm_anchor_weights_workspace(ctypes.byref(m), 100, 0, 0) == 0
    assert lib.kvcomm_anchor_weights_workspace(ctypes.byref(m), 100, 65, 0) == 0
    # per-(layer, head, token) weights need one partial per (layer, head)
    assert lib.kvcomm_anchor_weights_workspace(ctypes.byref(m), 100, 3, 1) == 8 * 4 * 100 * 3
    assert lib.kvcomm_suffix_attn_workspace(ctypes.byref(m), 100, 10) == 0


def test_rule_predict_capture_argument_errors(lib):
    m = _model()
    parr = (ctypes.c_void_p * 2)(0x2000, 0x3000)
    larr = (ctypes.c_int32 * 2)(16, 16)
    rule = lambda r, ws_bytes=1 << 30: lib.kvcomm_anchor_weights_rule(
        ctypes.byref(m), 0, r, 1.0, _tensor(), 16, parr, _tensor(None), larr, 2, 0x4000, None, None, 0x10000,
        ws_bytes, None)
    assert rule(3) == EINVAL and rule(-1) == EINVAL
    need_l2 = lib.kvcomm_anchor_weights_rule_workspace(ctypes.byref(m), 16, 2, 0, 0)
    need_cos = lib.kvcomm_anchor_weights_rule_workspace(ctypes.byref(m), 16, 2, 0, 2)
    assert need_l2 == lib.kvcomm_anchor_weights_workspace(ctypes.byref(m), 16, 2, 0)
    assert need_l2 == lib.kvcomm_anchor_weights_rule_workspace(ctypes.byref(m), 16, 2, 0, 1)
    assert need_cos == 3 * need_l2
    assert lib.kvcomm_anchor_weights_rule_workspace(ctypes.byref(m), 16, 2, 0, 7) == 0
    assert rule(2, need_cos - 1) == EWORKSPACE

    pred = lambda wts=0x4000, n=10, lens=(16, 16), seg_len=16, gamma=0.3, res=0x5000, ws=0x6000, ws_bytes=1 << 20: \
        lib.kvcomm_anchor_predict(wts, n, (ctypes.c_int32 * max(len(lens), 1))(*lens), len(lens), seg_len, gamma,
                                  None, res, ws, ws_bytes, None)
    assert pred(wts=None) == EINVAL and pred(res=None) == EINVAL
    assert pred(n=0) == EINVAL and pred(lens=()) == EINVAL and pred(seg_len=0) == EINVAL
    assert pred(gamma=-0.1) == EINVAL and pred(gamma=float("nan")) == EINVAL
    assert pred(lens=(16, -2)) == EINVAL
    assert pred(lens=(16,) * 65) == EUNSUPPORTED
    assert pred(ws=None) == EWORKSPACE and pred(ws=0x6004) == EWORKSPACE
    assert lib.kvcomm_anchor_predict_workspace(10) == 8
    assert lib.kvcomm_anchor_predict_workspace(257) == 16
    assert lib.kvcomm_anchor_predict_workspace(10 ** 9) == 8 * 1024
    assert lib.kvcomm_anchor_predict_workspace(0) == 0
    assert pred(n=1000, ws_bytes=8 * 4 - 1) == EWORKSPACE

    cap = lambda mm=m, seg_len=16, bk=None, out=None: lib.kvcomm_capture_offsets(
        ctypes.byref(mm), bk or _tensor(), _tensor(0x2000), _tensor(0x3000), _tensor(0x4000), seg_len, 5,
        out or _tensor(0x5000), _tensor(0x6000), None)
    assert cap(seg_len=0) == EINVAL
    assert cap(bk=_tensor(ptr=None)) == EINVAL
    assert cap(out=_tensor(ptr=0x5008)) == EINVAL
    assert cap(mm=_model(head_dim=72)) == EUNSUPPORTED
    assert lib.kvcomm_capture_offsets(None, _tensor(), _tensor(), _tensor(), _tensor(), 16, 0, _tensor(), _tensor(),
                                      None) == EINVAL


def test_compressed_deviation_argument_errors(lib):
    m = _model()
    q = lambda scale=2.0 ** -10, n=16, inp=None, out=None: lib.kvcomm_quantize_deltas(
        ctypes.byref(m), inp or _tensor(), n, scale, out or _tensor(0x2000, st=128), None)
    assert q(scale=0.003) == EINVAL and q(scale=0.0) == EINVAL and q(scale=-0.5) == EINVAL
    assert q(scale=float("inf")) == EINVAL and q(scale=float("nan")) == EINVAL
    assert q(n=0) == EINVAL
    assert q(out=_tensor(0x2008, st=128)) == EINVAL           # byte tensors need 16-byte alignment too
    assert q(out=_tensor(0x2000, st=72)) == EINVAL
    assert q(inp=_tensor(ptr=None)) == EINVAL
    parr = (ctypes.c_void_p * 2)(0x2000, 0x3000)
    larr = (ctypes.c_int32 * 2)(16, 16)
    good = (ctypes.c_float * 2)(2.0 ** -10, 2.0 ** -9)
    bad = (ctypes.c_float * 2)(2.0 ** -10, 0.3)
    a8 = lambda sk=good, sv=good, layout=None, weights=0x4000: lib.kvcomm_align_kv_q8(
        ctypes.byref(m), 0, _tensor(), _tensor(0x5000), 16, parr, parr, layout or _tensor(None, st=128), larr, sk, sv, 2,
        weights, 64, None, _tensor(0x6000), _tensor(0x7000), None)
    assert a8(sk=bad) == EINVAL and a8(sv=bad) == EINVAL and a8(sk=None) == EINVAL
    assert a8(layout=_tensor(None, st=24)) == EINVAL
    assert a8(weights=None) == EINVAL


def test_compressed_batch_argument_errors(lib):
    m = _model()
    parr = (ctypes.c_void_p * 2)(0x2000, 0x3000)
    larr = (ctypes.c_int32 * 2)(16, 16)
    good = (ctypes.c_float * 2)(2.0 ** -10, 2.0 ** -9)
    bad = (ctypes.c_float * 2)(2.0 ** -10, 0.3)
    tiny = (ctypes.c_float * 2)(2.0 ** -10, 2.0 ** -130)      # a subnormal power of two has no exponent to pass on

    def job(sk=good, sv=good, out=0x6000, slots=16, weights=0x4000):
        return binding._CAlignQ8Job(_tensor(), _tensor(0x5000), _tensor(out), _tensor(out + 0x1000), 16, 64, parr, parr,
                                    larr, None, sk, sv, 2, weights, slots)

    def call(jobs, layout=None):
        arr = (binding._CAlignQ8Job * max(len(jobs), 1))(*jobs)
        return lib.kvcomm_align_kv_q8_batch(ctypes.byref(m), 0, layout or _tensor(None, st=128), arr, len(jobs), None)

    assert call([]) == EINVAL
    assert call([job()] * 9) == EUNSUPPORTED
    assert call([job(), job(sk=bad, out=0x8000)]) == EINVAL
    assert call([job(sv=tiny)]) == EINVAL
    assert call([job(sk=None)]) == EINVAL
    assert call([job(slots=3)]) == EINVAL
    assert call([job(), job()]) == EINVAL                       # both jobs write the same rows
    assert call([job()], layout=_tensor(None, st=24)) == EINVAL
    assert call([job(), job(out=0x8000)]) != EINVAL


def test_static_scratch_entry_point_argument_errors(lib):
    """The entry point without a workspace argument refuses what does not fit its fixed array before it
    looks at anything else, and validates like kvcomm_anchor_weights otherwise."""
    m = _model(n_layers=32, n_kv_heads=8, n_q_heads=32)
    cap = lib.kvcomm_anchor_weights_static_capacity()
    assert cap == 16 << 20

    def call(seg_len=16, A=2, gran=0, tau=1.0, weights=0x4000, model=m):
        parr = (ctypes.c_void_p * A)(*[0x2000 + 0x1000 * i for i in range(A)])
        larr = (ctypes.c_int32 * A)(*[seg_len] * A)
        return lib.kvcomm_anchor_weights_static(ctypes.byref(model), gran, tau, _tensor(), seg_len, parr, _tensor(None),
                                                larr, A, weights, None, None, None)

    assert lib.kvcomm_anchor_weights_workspace(ctypes.byref(m), 1024, 64, 0) <= cap
    assert lib.kvcomm_anchor_weights_workspace(ctypes.byref(m), 2048, 16, 0) <= cap
    assert lib.kvcomm_anchor_weights_workspace(ctypes.byref(m), 32768, 64, 0) <= cap    # the per-token cut adapts
    big = (65536, 64, 0)
    assert lib.kvcomm_anchor_weights_workspace(ctypes.byref(m), *big) > cap
    assert call(seg_len=big[0], A=big[1], gran=big[2]) == EWORKSPACE
    assert call(seg_len=2048, A=8, gran=1) == EWORKSPACE         # one partial per (layer, head, token, anchor): 32 MiB
    assert call(seg_len=0) == EINVAL
    assert call(gran=7) == EINVAL
    assert call(A=0) == EINVAL
    assert call(A=65) == EUNSUPPORTED
    assert call(model=_model(head_dim=80)) == EUNSUPPORTED
    # what fits goes on to the checks of kvcomm_anchor_weights itself, still on the host
    assert call(tau=0.0) in (EINVAL, -4)
    assert call(weights=None) in (EINVAL, -4)


def test_batch_argument_errors(lib):
    m = _model()
    parr = (ctypes.c_void_p * 40)(*[0x2000 + 0x100 * i for i in range(40)])
    larr = (ctypes.c_int32 * 40)(*[16] * 40)

    def ajob(n_anchors=2, seg_len=16, weights=0x4000, out=0x6000, slots=16, gran_slots=None):
        return binding._CAlignJob(_tensor(), _tensor(0x5000), _tensor(out), _tensor(out + 0x1000), seg_len, 64, parr, parr,
                                  larr, None, n_anchors, weights, slots)

    def acall(jobs, gran=0):
        arr = (binding._CAlignJob * max(len(jobs), 1))(*jobs)
        return lib.kvcomm_align_kv_batch(ctypes.byref(m), gran, _tensor(None), arr, len(jobs), None)

    assert acall([]) == EINVAL
    assert acall([ajob()] * 9) == EUNSUPPORTED                     # more than KVCOMM_MAX_BATCH jobs
    assert acall([ajob(), ajob(seg_len=0, out=0x8000)]) == EINVAL
    assert acall([ajob(), ajob(weights=None, out=0x8000)]) == EINVAL
    assert acall([ajob(n_anchors=40), ajob(n_anchors=40, out=0x8000)]) == EUNSUPPORTED   # 80 selected anchors in one launch
    assert lib.kvcomm_align_kv_batch(ctypes.byref(m), 0, _tensor(None), None, 1, None) == EINVAL
    # a job's weight buffer must have the rows its own segment length asks for (a prefix segment that borrows a
    # placeholder's per-token weights of another length is refused; per-segment weights fit any length)
    assert acall([ajob(slots=15)]) == EINVAL
    assert acall([ajob(), ajob(out=0x8000, slots=1)]) == EINVAL
    assert acall([ajob(slots=1)], gran=2) != EINVAL
    assert acall([ajob(slots=16)], gran=2) == EINVAL
    assert acall([ajob(slots=2 * 2 * 16)], gran=1) != EINVAL
    # two jobs that write the same rows
    assert acall([ajob(), ajob()]) == EINVAL
    assert acall([ajob(), ajob(out=0x6800)]) == EINVAL

    def wjob(n_anchors=2, seg_len=16, weights=0x4000):
        return binding._CWeightsJob(_tensor(), seg_len, parr, larr, n_anchors, weights, None, None)

    def wcall(jobs, ws=0x10000, ws_bytes=1 << 30, tau=1.0):
        arr = (binding._CWeightsJob * max(len(jobs), 1))(*jobs)
        return lib.kvcomm_anchor_weights_batch(ctypes.byref(m), 0, 0, tau, _tensor(None), arr, len(jobs), ws, ws_bytes,
                                               None)

    assert wcall([]) == EINVAL
    assert wcall([wjob()] * 9) == EUNSUPPORTED
    assert wcall([wjob(), wjob(weights=None)]) == EINVAL
    assert wcall([wjob(n_anchors=40), wjob(n_anchors=40)]) == EUNSUPPORTED
    assert wcall([wjob(), wjob()], tau=0.0) == EINVAL
    sl = (ctypes.c_int32 * 2)(16, 100)
    na = (ctypes.c_int32 * 2)(2, 5)
    need = lib.kvcomm_anchor_weights_batch_workspace(ctypes.byref(m), 0, 0, sl, na, 2)
    assert need > 0 and need % 256 == 0
    assert wcall([wjob(), wjob(n_anchors=5, seg_len=100)], ws_bytes=need - 1) == EWORKSPACE
    assert wcall([wjob(), wjob()], ws=None) == EWORKSPACE
    assert lib.kvcomm_anchor_weights_batch_workspace(ctypes.byref(m), 0, 0, sl, na, 9) == 0
    assert lib.kvcomm_anchor_weights_batch_workspace(ctypes.byref(m), 0, 0, sl, None, 2) == 0


def _align(lib, m, gran=0, seg_len=16, ptrs=(0x2000,), lens=(16,), weights=0x4000, bk=None, out=None, adp=None):
    A = len(ptrs)
    parr = (ctypes.c_void_p * max(A, 1))(*ptrs)
    larr = (ctypes.c_int32 * max(A, 1))(*lens)
    aarr = None if adp is None else (ctypes.c_int32 * max(A, 1))(*adp)
    return lib.kvcomm_align_kv(ctypes.byref(m), gran, bk or _tensor(), _tensor(0x5000), seg_len, parr, parr,
                               _tensor(None), larr, A, weights, 64, aarr, out or _tensor(0x6000), _tensor(0x7000),
                               None)


def test_align_aliasing_rules(lib):
    """An output may be exactly its base tensor (in place); any other sharing of bytes with another tensor of the
    call is an argument error found on the host.  (Every call that passes the checks here would launch; the
    accepted cases therefore use status != EINVAL on a machine without a GPU.)"""
    m = _model()
    parr = (ctypes.c_void_p * 1)(0x2000)
    larr = (ctypes.c_int32 * 1)(16)

    def call(bk=0x1000, bv=0x5000, ok=0x6000, ov=0x7000, dk=0x2000, dv=0x3000, w=0x4000, ok_t=None, layout=None):
        pk, pv = (ctypes.c_void_p * 1)(dk), (ctypes.c_void_p * 1)(dv)
        return lib.kvcomm_align_kv(ctypes.byref(m), 0, _tensor(bk), _tensor(bv), 16, pk, pv, layout or _tensor(None), larr,
                                   1, w, 64, None, ok_t or _tensor(ok), _tensor(ov), None)

    assert call(ok=0x1000 + 0x800) == EINVAL            # out_k starts inside base_k's first block
    assert call(ok=0x1000 - 0x800) == EINVAL            # ... or ends inside it
    assert call(ok=0x5000 + 0x10) == EINVAL             # out_k over base_v
    assert call(ov=0x1000) == EINVAL                    # out_v exactly base_k: only the own base may be shared
    assert call(ok=0x6000, ov=0x6000) == EINVAL         # the two outputs on each other
    assert call(ok=0x6000, ov=0x6800) == EINVAL
    assert call(ok=0x2000 + 0x40) == EINVAL             # out_k over the anchor's key deviations
    assert call(ov=0x3000 - 0x40) == EINVAL             # out_v over its value deviations
    assert call(ok=0x4000 - 0xfc0) == EINVAL            # out_k's last bytes over the weights
    # same pointer, other strides: not the in-place case
    assert call(ok_t=_tensor(0x1000, st=256)) == EINVAL
    # a block of out_k that lands on a LATER block of base_k (other layer / head), same strides
    assert call(ok=0x1000 + (1 << 16) * 2 + 0x100) == EINVAL
    assert call(ok=0x1000 + (1 << 20) * 2 - 0x100) == EINVAL
    # other strides than base_k's (blocks at +0, +0x10000, +0x100000, +0x110000 bytes): the sorted-interval path
    assert call(ok_t=binding._CTensor(0x8000, 1 << 19, 1 << 15, 128)) != EINVAL       # touches nothing
    assert call(ok_t=binding._CTensor(0x11000, 1 << 19, 1 << 15, 128)) == EINVAL      # its block (0, 1) is base_k's (0, 1)
    assert call(ok_t=binding._CTensor(0x101000 + 0x800, 1 << 19, 1 << 15, 128)) == EINVAL   # its (1, 0) ends in base_k's (1, 0)
    # accepted: disjoint tensors, and the in-place update
    assert call() != EINVAL
    assert call(ok=0x1000, ov=0x5000) != EINVAL
    # an anchor that is too short is never read, so it may lie anywhere
    short = (ctypes.c_int32 * 1)(8)
    assert lib.kvcomm_align_kv(ctypes.byref(m), 0, _tensor(), _tensor(0x5000), 16, parr, parr, _tensor(None), short, 1,
                               0x4000, 64, None, _tensor(0x2000), _tensor(0x7000), None) != EINVAL


def test_align_argument_errors(lib):
    m = _model()
    assert _align(lib, m, gran=9) == EINVAL
    assert _align(lib, m, seg_len=-3) == EINVAL
    assert _align(lib, m, bk=_tensor(ptr=None)) == EINVAL
    assert _align(lib, m, out=_tensor(ptr=0x6002)) == EINVAL
    assert _align(lib, m, weights=None) == EINVAL
    assert _align(lib, m, ptrs=(0x2001,)) == EINVAL
    assert _align(lib, m, ptrs=(0x2000,) * 65, lens=(16,) * 65) == EUNSUPPORTED
    assert _align(lib, m, lens=(-5,)) == EINVAL
    assert _align(lib, _model(head_dim=80)) == EUNSUPPORTED
    assert _align(lib, _model(dtype=0), bk=_tensor(st=2)) == EINVAL   # fp32 rows need strides in multiples of 4


def test_suffix_attn_confined_argument_errors(lib):
    m = _model()
    call = lambda max_blocks=64, n_ctx=10, tq=4, q=None: lib.kvcomm_suffix_attn_confined(
        ctypes.byref(m), q or _tensor(), _tensor(0x2000), _tensor(0x3000), n_ctx, tq, 0.0, _tensor(0x4000), None,
        max_blocks, None)
    for bad in (7, 0, -1):
        assert call(max_blocks=bad) == EINVAL       # fewer than one block per XCD
    assert call(tq=0) == EINVAL                     # the checks of kvcomm_suffix_attn come first for valid max_blocks
    assert call(n_ctx=-1) == EINVAL
    assert call(q=_tensor(ptr=None)) == EINVAL


def test_suffix_attn_argument_errors(lib):
    m = _model()
    call = lambda q=None, n_ctx=10, tq=4, out=None: lib.kvcomm_suffix_attn(
        ctypes.byref(m), q or _tensor(), _tensor(0x2000), _tensor(0x3000), n_ctx, tq, 0.0, out or _tensor(0x4000),
        None, None, 0, None)
    assert call(tq=0) == EINVAL
    assert call(n_ctx=-1) == EINVAL
    assert call(q=_tensor(ptr=None)) == EINVAL
    assert call(out=_tensor(ptr=0x4004)) == EINVAL
    assert lib.kvcomm_suffix_attn(ctypes.byref(_model(n_q_heads=5)), _tensor(), _tensor(0x2000), _tensor(0x3000), 1, 1,
                                  0.0, _tensor(0x4000), None, None, 0, None) == EUNSUPPORTED
    # a bf16 cache whose rows are too far apart for the kernel's 32-bit per-lane byte offsets
    far = _tensor(0x2000)
    far.stride_token = 1 << 28
    far.stride_head = 1 << 40
    far.stride_layer = 1 << 44
    assert lib.kvcomm_suffix_attn(ctypes.byref(m), _tensor(), far, _tensor(0x3000), 10, 4, 0.0, _tensor(0x4000),
                                  None, None, 0, None) == EUNSUPPORTED


def test_binding_rejects_host_tensors_and_mixed_layouts(lib):
    model = kv.Model(2, 2, 4, 128, torch.bfloat16, 5e5)
    x = torch.zeros(2, 2, 16, 128, dtype=torch.bfloat16)
    with pytest.raises(kv.KVCommError):
        kv.kvcomm_suffix_attn(model, x, x, x, 0)
    with pytest.raises(kv.KVCommError):
        binding._desc(x, torch.bfloat16, "x")
    with pytest.raises(kv.KVCommError):
        kv.Model(2, 2, 4, 128, torch.float16, 5e5).c()


def test_launch_chunks_respect_segment_and_anchor_limits():
    from paper_2510_12872_amd import hotpath
    assert hotpath.launch_chunks([8, 8, 8, 8]) == [[0, 1, 2, 3]]
    assert hotpath.launch_chunks([3] * 11) == [list(range(8)), [8, 9, 10]]
    assert hotpath.launch_chunks([30, 30, 30]) == [[0, 1], [2]]
    assert hotpath.launch_chunks([64, 1, 63, 64]) == [[0], [1, 2], [3]]
    assert hotpath.launch_chunks([]) == []
    for counts in ([5, 60, 4, 4, 64, 1, 1, 1, 1, 1, 1, 1, 1, 1], [16] * 9):
        chunks = hotpath.launch_chunks(counts)
        assert [j for c in chunks for j in c] == list(range(len(counts)))
        assert all(len(c) <= kv.MAX_BATCH and sum(counts[j] for j in c) <= kv.MAX_ANCHORS for c in chunks)


def test_bench_refuses_more_than_one_gpu():
    """The benchmark runs on one GPU only; asking for more exits with a message (and never touches a device)."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stderr + r.stdout)
