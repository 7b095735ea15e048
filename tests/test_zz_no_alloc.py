"""kvcomm_anchor_weights_static: the anchor-matching entry point for callers that cannot allocate (its
partial sums live in a fixed array inside the library).  Through the C ABI against kvcomm_anchor_weights
on the same inputs: bit-identical weights, nearest anchors and selection, on two calls in a row, the
second with a smaller input, so whatever the first call left in the shared array must not matter.  The
first result is also held to the oracle.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_12872_amd as kv
from paper_2510_12872_amd import hotpath, workloads
from paper_2510_12872_amd.workloads import scaled

from parity import check_weights, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _both(model, seg, gran):
    S, A = seg.base_k.shape[2], len(seg.anchor_k)
    n = kv.kvcomm_weight_slots(model, S, gran)
    want = kv.kvcomm_anchor_weights(model, seg.base_k, seg.anchor_k, seg.anchor_len, 1.0, gran)
    got = (torch.full((n, A), -7.0, dtype=torch.float32, device=DEV),
           torch.full((n,), -7, dtype=torch.int32, device=DEV), torch.full((A,), -7, dtype=torch.int32, device=DEV))
    kv.kvcomm_anchor_weights_static(model, seg.base_k, seg.anchor_k, *got, anchor_len=seg.anchor_len, gran=gran)
    torch.cuda.synchronize()
    return got, want


def test_static_scratch_matches_workspace_entry_point_twice():
    big = scaled(workloads.LLAMA8B_5AGENTS, name="noalloc_big", n_layers=4, n_kv_heads=2, n_q_heads=4, n_agents=1,
                 seg_len=333, n_segments=1, n_anchors=9, tq=0, anchor_lens=(333, 400, 333, 100, 333, 333, 350, 333, 333))
    small = scaled(big, name="noalloc_small", seg_len=45, n_anchors=3, anchor_lens=None, seed=3)
    assert kv.kvcomm_anchor_weights_static_capacity() == 16 << 20
    first = True
    for w in (big, small):
        print(f"no-alloc entry point: {w.name}", flush=True)
        model = hotpath.model_of(w)
        seg = workloads.make_segment(w, 0, 0, DEV)
        for gran in (kv.W_TOKEN, kv.W_SEGMENT):
            got, want = _both(model, seg, gran)
            for g, x, what in zip(got, want, ("weights", "nearest", "selected")):
                assert torch.equal(g, x), f"{w.name} gran {gran}: {what} differ from kvcomm_anchor_weights"
        if first:
            S = w.seg_len
            anc = [to_np(a) if n >= S else np.zeros(seg.base_k.shape[:2] + (0, w.head_dim))
                   for a, n in zip(seg.anchor_k, seg.anchor_len)]
            dist, sel = oracle.distances(to_np(seg.base_k), anc, 0)
            wo, near = oracle.weights(dist, sel, 1.0)
            got, _ = _both(model, seg, kv.W_TOKEN)
            check_weights(got[0].cpu().numpy(), wo.T)
            assert np.array_equal(got[1].cpu().numpy(), near) and np.array_equal(got[2].cpu().numpy(), sel)
            first = False


def test_static_scratch_refuses_what_does_not_fit():
    w = scaled(workloads.LLAMA8B_5AGENTS, n_agents=1, n_segments=1, seg_len=2048, n_anchors=8, tq=0)
    model = hotpath.model_of(w)
    assert kv.kvcomm_anchor_weights_workspace(model, 2048, 8, kv.W_LAYER_HEAD_TOKEN) > kv.kvcomm_anchor_weights_static_capacity()
    x = torch.zeros((w.n_layers, w.n_kv_heads, 2048, w.head_dim), dtype=w.dtype, device=DEV)
    n = kv.kvcomm_weight_slots(model, 2048, kv.W_LAYER_HEAD_TOKEN)
    out = torch.full((n, 8), -7.0, dtype=torch.float32, device=DEV)
    with pytest.raises(kv.KVCommError) as e:
        kv.kvcomm_anchor_weights_static(model, x, [x] * 8, out, None, None, gran=kv.W_LAYER_HEAD_TOKEN)
    assert e.value.status == -3
    torch.cuda.synchronize()
    assert float(out.min()) == -7.0 and float(out.max()) == -7.0     # nothing was launched
