"""Host-side sequencing of the reuse step for one agent: three library calls per segment/agent.

Nothing is computed here; the functions only issue the calls of include/kvcomm.h in the
order of the reuse branch of Algorithm 1 (weights -> offset approximation per placeholder,
then attention over the concatenated cache) on the current stream.
"""
import torch

from . import binding as kv


def model_of(w):
    """kvcomm model descriptor of a workloads.Workload."""
    return kv.Model(w.n_layers, w.n_kv_heads, w.n_q_heads, w.head_dim, w.dtype, w.rope_theta)


class Scratch:
    """Reusable device buffers for the weight step (so a timed loop allocates nothing)."""

    def __init__(self, model, seg_len, n_anchors, gran, device):
        n = kv.kvcomm_weight_slots(model, seg_len, gran)
        self.weights = torch.empty((n, n_anchors), dtype=torch.float32, device=device)
        self.nearest = torch.empty((n,), dtype=torch.int32, device=device)
        self.selected = torch.empty((n_anchors,), dtype=torch.int32, device=device)
        need = kv.kvcomm_anchor_weights_workspace(model, seg_len, n_anchors, gran)
        self.workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=device)


def align_segment(model, seg, out_k, out_v, temperature=1.0, gran=kv.W_TOKEN, scratch=None, stream=None):
    """Anchor weights, then aligned K/V of one segment written into out_k / out_v."""
    if scratch is None:
        scratch = Scratch(model, seg.base_k.shape[2], len(seg.anchor_k), gran, seg.base_k.device)
    kv.kvcomm_anchor_weights(model, seg.base_k, seg.anchor_k, seg.anchor_len, temperature, gran,
                             scratch.weights, scratch.nearest, scratch.selected, scratch.workspace, stream)
    kv.kvcomm_align_kv(model, seg.base_k, seg.base_v, seg.anchor_dk, seg.anchor_dv, scratch.weights,
                       seg.delta_pos, out_k, out_v, seg.anchor_len, seg.anchor_delta_pos, gran, stream)
    return scratch


def reuse_agent(w, model, agent, out=None, gran=kv.W_TOKEN, scratches=None, stream=None):
    """Whole hot path for one agent: align every segment into its cache slot, then suffix attention."""
    for j, seg in enumerate(agent.segments):
        p0 = w.seg_offset(j)
        S = seg.base_k.shape[2]
        align_segment(model, seg, agent.cache_k[:, :, p0:p0 + S], agent.cache_v[:, :, p0:p0 + S],
                      w.temperature, gran, None if scratches is None else scratches[j], stream)
    if agent.q is None:
        return None
    return kv.kvcomm_suffix_attn(model, agent.q, agent.cache_k, agent.cache_v, w.n_ctx, out=out, stream=stream)
