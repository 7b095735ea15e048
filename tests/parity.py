"""Helpers shared by the GPU parity tests: oracle evaluation on (sampled) inputs and the
comparison rules.

Tolerances (stated by the build's target): integer outputs bit-exact; bf16 outputs within
max-abs 2e-2 of the float64 oracle; fp32 outputs within 1e-5 * max(1, max|oracle|) per
tensor.  The fp32 weights are held to the 1e-5 rule for every dtype because distances are
accumulated in double on both sides.
"""
import numpy as np
import torch

import oracle

BF16_ATOL = 2e-2
F32_RTOL = 1e-5


def to_np(t):
    return t.detach().to(torch.float64).cpu().numpy()


def check_close(got, want, dtype, what):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    assert np.all(np.isfinite(got)), f"{what}: non-finite values"
    err = float(np.max(np.abs(got - want))) if got.size else 0.0
    tol = BF16_ATOL if dtype == torch.bfloat16 else F32_RTOL * max(1.0, float(np.max(np.abs(want))) if want.size else 1.0)
    assert err <= tol, f"{what}: max abs err {err:.3e} > {tol:.3e}"
    return err


def check_weights(got, want, what="weights"):
    got = np.asarray(got, dtype=np.float64)
    err = float(np.max(np.abs(got - want))) if got.size else 0.0
    assert np.all(np.isfinite(got)), f"{what}: non-finite values"
    assert err <= F32_RTOL, f"{what}: max abs err {err:.3e} > {F32_RTOL:.1e}"
    return err


def oracle_segment(w, seg, tokens=None, gran=0):
    """Oracle distances/weights/align for one workloads.Segment, optionally on a subset of tokens.

    Per-token granularity treats tokens independently, so a token subset is itself a valid
    (shorter) segment for the oracle; anchors keep only those tokens too.  An anchor shorter
    than the segment is passed with zero tokens so that the oracle leaves it unselected.
    """
    S = seg.base_k.shape[2]
    idx = torch.arange(S) if tokens is None else torch.as_tensor(tokens)
    sel = lambda t: to_np(t[:, :, idx.to(t.device)])
    bk, bv = sel(seg.base_k), sel(seg.base_v)

    def anchors(lst):
        out = []
        for a, n in zip(lst, seg.anchor_len):
            out.append(sel(a) if n >= S else np.zeros(bk.shape[:2] + (0, bk.shape[3])))
        return out

    return oracle.reuse_step(bk, bv, anchors(seg.anchor_k), anchors(seg.anchor_dk), anchors(seg.anchor_dv),
                             seg.delta_pos, w.rope_theta, tau=w.temperature,
                             anc_delta=seg.anchor_delta_pos, gran=gran)


def oracle_attention(w, agent, layer_heads, queries=None):
    """Oracle suffix attention for chosen (layer, q head) pairs; returns {(l, hq): out [Tq', D]}."""
    G = w.n_q_heads // w.n_kv_heads
    res = {}
    for (l, hq) in layer_heads:
        hk = hq // G
        q = to_np(agent.q[l:l + 1, hq:hq + 1])
        k = to_np(agent.cache_k[l:l + 1, hk:hk + 1])
        v = to_np(agent.cache_v[l:l + 1, hk:hk + 1])
        out, lse = oracle.suffix_attn(q, k, v, w.n_ctx, want_lse=True)
        res[(l, hq)] = (out[0, 0], lse[0, 0])
    return res
