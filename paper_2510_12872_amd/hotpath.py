"""Host-side sequencing of the reuse step: three library calls per segment/agent.

Nothing is computed here; the functions only issue the calls of include/kvcomm.h in the
order of the reuse branch of Algorithm 1 (weights -> offset approximation per placeholder,
then attention over the concatenated cache), on the current stream or, for consecutive
agents, on two streams (TwoStreamPipeline).
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


def launch_chunks(n_anchors):
    """Cut the segments of an agent (given by their anchor counts) into launches: one launch carries at
    most MAX_BATCH segments and MAX_ANCHORS anchors over all of them."""
    chunks, cur, n_anc = [], [], 0
    for j, a in enumerate(n_anchors):
        if cur and (len(cur) == kv.MAX_BATCH or n_anc + a > kv.MAX_ANCHORS):
            chunks.append(cur)
            cur, n_anc = [], 0
        cur.append(j)
        n_anc += a
    if cur:
        chunks.append(cur)
    return chunks


class AgentScratch:
    """Reusable device buffers for the batched weight step of all segments of one agent."""

    def __init__(self, model, seg_lens, n_anchors, gran, device, rule=kv.RULE_L2_SOFTMAX):
        self.weights, self.nearest, self.selected = [], [], []
        for S, A in zip(seg_lens, n_anchors):
            n = kv.kvcomm_weight_slots(model, S, gran)
            self.weights.append(torch.empty((n, A), dtype=torch.float32, device=device))
            self.nearest.append(torch.empty((n,), dtype=torch.int32, device=device))
            self.selected.append(torch.empty((A,), dtype=torch.int32, device=device))
        seg_lens, n_anchors = list(seg_lens), list(n_anchors)
        need = max(kv.kvcomm_anchor_weights_batch_workspace(model, [seg_lens[j] for j in c], [n_anchors[j] for j in c],
                                                            gran, rule) for c in launch_chunks(n_anchors))
        self.workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=device)


def align_agent_batched(w, model, agent, gran=kv.W_TOKEN, scratch=None, stream=None):
    """Anchor weights, then aligned K/V of ALL segments of an agent: one batched call per step and
    chunk of segments (a launch holds at most MAX_BATCH segments and MAX_ANCHORS anchors)."""
    segs = agent.segments
    if scratch is None:
        scratch = AgentScratch(model, [s.base_k.shape[2] for s in segs], [len(s.anchor_k) for s in segs], gran,
                               segs[0].base_k.device)
    for idx in launch_chunks([len(s.anchor_k) for s in segs]):
        kv.kvcomm_anchor_weights_batch(model, [dict(
            seg_base_k=segs[j].base_k, anchor_base_k=segs[j].anchor_k, anchor_len=segs[j].anchor_len,
            weights_out=scratch.weights[j], nearest_out=scratch.nearest[j], selected_out=scratch.selected[j])
            for j in idx], w.temperature, gran, workspace=scratch.workspace, stream=stream)
        jobs = []
        for j in idx:
            p0, S = w.seg_offset(j), segs[j].base_k.shape[2]
            jobs.append(dict(base_k=segs[j].base_k, base_v=segs[j].base_v, anchor_dk=segs[j].anchor_dk,
                             anchor_dv=segs[j].anchor_dv, anchor_len=segs[j].anchor_len, weights=scratch.weights[j],
                             delta_pos=segs[j].delta_pos, anchor_delta_pos=segs[j].anchor_delta_pos,
                             out_k=agent.cache_k[:, :, p0:p0 + S], out_v=agent.cache_v[:, :, p0:p0 + S]))
        kv.kvcomm_align_kv_batch(model, jobs, gran, stream)
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


class TwoStreamPipeline:
    """The reuse step of consecutive agents on two streams: weights + alignment of an agent run beside the
    attention of the agent before it.  The attention is launched through kvcomm_suffix_attn_confined as at most
    `attn_blocks` persistent blocks, so that the other compute units are free for the memory-bound alignment
    kernels for the whole launch (attn_blocks = 0: the plain launch, which leaves them only the gaps).

    Ordering: an event per submission puts the attention behind its own alignment; a second one, kept per buffer
    key, puts the next alignment into the same cache behind the attention that still reads it.  HIP maps streams
    onto a few hardware queues and two streams that share one run one after the other: pick_attention_stream()
    tries candidates and keeps the fastest."""

    def __init__(self, model, temperature=1.0, attn_blocks=160, gran=kv.W_TOKEN, align_stream=None, attn_stream=None):
        self.model, self.temperature, self.attn_blocks, self.gran = model, temperature, attn_blocks, gran
        self.s_align = align_stream or torch.cuda.Stream()
        self.s_attn = attn_stream or torch.cuda.Stream()
        self._done = {}

    def fork(self):
        """Both streams wait for the work already queued on the current stream."""
        cur = torch.cuda.current_stream()
        self.s_align.wait_stream(cur)
        self.s_attn.wait_stream(cur)

    def join(self):
        """The current stream waits for everything submitted so far."""
        cur = torch.cuda.current_stream()
        cur.wait_stream(self.s_align)
        cur.wait_stream(self.s_attn)

    def submit(self, key, wjobs, ajobs, workspace, q, cache_k, cache_v, n_ctx, out, q8=False):
        """One agent: batched weights and alignment (job lists as for the batched calls) on the alignment stream,
        then its suffix attention on the attention stream.  `key` names the agent's buffers."""
        with torch.cuda.stream(self.s_align):
            if key in self._done:
                self.s_align.wait_event(self._done[key])
            kv.kvcomm_anchor_weights_batch(self.model, wjobs, self.temperature, self.gran, workspace=workspace)
            if q8:
                kv.kvcomm_align_kv_q8_batch(self.model, ajobs, self.gran)
            else:
                kv.kvcomm_align_kv_batch(self.model, ajobs, self.gran)
            aligned = torch.cuda.Event()
            aligned.record(self.s_align)
        with torch.cuda.stream(self.s_attn):
            self.s_attn.wait_event(aligned)
            if q is not None:
                if self.attn_blocks > 0:
                    kv.kvcomm_suffix_attn_confined(self.model, q, cache_k, cache_v, n_ctx, self.attn_blocks, out=out)
                else:
                    kv.kvcomm_suffix_attn(self.model, q, cache_k, cache_v, n_ctx, out=out)
            done = torch.cuda.Event()
            done.record(self.s_attn)
            self._done[key] = done

    def pick_attention_stream(self, run_steps, candidates=None, warm=2, timed=3):
        """run_steps(n) must submit n steps through this pipeline (fork ... join).  Tries every candidate stream
        for the attention and keeps the one with the shortest steps."""
        import time
        candidates = candidates or [self.s_attn] + [torch.cuda.Stream() for _ in range(2)]
        best = None
        for cand in candidates:
            self.s_attn = cand
            run_steps(warm)
            torch.cuda.synchronize()
            t = time.perf_counter()
            run_steps(timed)
            torch.cuda.synchronize()
            t = time.perf_counter() - t
            if best is None or t < best[0]:
                best = (t, cand)
        self.s_attn = best[1]
        return best[1]
