"""GPU parity: the HIP library (through its C ABI) against the float64 oracle, element by
element on small seeded inputs and on sampled outputs at the full sizes of the five
baseline configurations.  Integers bit-exact, floats to the tolerances in tests/parity.py.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_12872_amd as kv
from paper_2510_12872_amd import hotpath, workloads
from paper_2510_12872_amd.workloads import scaled

from parity import check_close, check_weights, oracle_attention, oracle_segment, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda"


def say(msg):
    print(msg, flush=True)


def run_segment(w, seg, gran=kv.W_TOKEN, in_place=False):
    model = hotpath.model_of(w)
    if in_place:
        out_k, out_v = seg.base_k, seg.base_v
    else:
        out_k, out_v = torch.empty_like(seg.base_k), torch.empty_like(seg.base_v)
    sc = hotpath.align_segment(model, seg, out_k, out_v, w.temperature, gran)
    torch.cuda.synchronize()
    return sc, out_k, out_v


def compare_segment(w, seg, sc, out_k, out_v, gran=kv.W_TOKEN, tokens=None, ref=None):
    """Compare weights / nearest / selected / K^ / V^ with the oracle (on `tokens` if given)."""
    ref = ref or oracle_segment(w, seg, tokens, gran)
    L, H, S, D = seg.base_k.shape
    A = len(seg.anchor_k)
    assert np.array_equal(sc.selected.cpu().numpy(), ref["selected"]), "selected"
    wg = sc.weights.cpu().numpy()            # [n, A]
    ng = sc.nearest.cpu().numpy()
    if tokens is not None:
        assert gran == kv.W_TOKEN
        wg, ng = wg[tokens], ng[tokens]
        idx = torch.as_tensor(tokens, device=out_k.device)
        out_k, out_v = out_k[:, :, idx], out_v[:, :, idx]
    assert np.array_equal(ng, ref["nearest"]), "nearest"
    check_weights(wg, ref["w"].T)
    check_close(to_np(out_k), ref["out_k"], w.dtype, "K^")
    check_close(to_np(out_v), ref["out_v"], w.dtype, "V^")


# ------------------------------------------------------------------------------ config 1
@pytest.mark.parametrize("gran", [kv.W_TOKEN, kv.W_LAYER_HEAD_TOKEN, kv.W_SEGMENT])
def test_tiny_config_all_granularities(gran):
    w = workloads.TINY
    say(f"tiny gran={gran}")
    seg = workloads.make_segment(w, 0, 0, DEV)
    sc, ok, ov = run_segment(w, seg, gran)
    compare_segment(w, seg, sc, ok, ov, gran)


def test_tiny_config_whole_hot_path():
    w = workloads.TINY
    say("tiny whole path")
    model = hotpath.model_of(w)
    agent = workloads.make_agent(w, 0, DEV)
    before_k = agent.cache_k.clone()
    out = hotpath.reuse_agent(w, model, agent)
    torch.cuda.synchronize()
    # prefix and suffix rows of the cache are untouched by the alignment
    p0, S = w.seg_offset(0), w.seg_len
    assert torch.equal(agent.cache_k[:, :, :p0], before_k[:, :, :p0])
    assert torch.equal(agent.cache_k[:, :, p0 + S:], before_k[:, :, p0 + S:])
    ref = oracle_segment(w, agent.segments[0])
    check_close(to_np(agent.cache_k[:, :, p0:p0 + S]), ref["out_k"], w.dtype, "cache K^")
    check_close(to_np(agent.cache_v[:, :, p0:p0 + S]), ref["out_v"], w.dtype, "cache V^")
    # attention over the oracle's own assembled cache (so each step is judged on its own) ...
    ck, cv = to_np(agent.cache_k), to_np(agent.cache_v)
    ck[:, :, p0:p0 + S], cv[:, :, p0:p0 + S] = ref["out_k"], ref["out_v"]
    want = oracle.suffix_attn(to_np(agent.q), ck, cv, w.n_ctx)
    check_close(to_np(out), want, w.dtype, "O")


# --------------------------------------------------------------------- small, ragged, edge cases
SMALL_BF16 = scaled(workloads.LLAMA8B_5AGENTS, name="small_bf16", n_layers=3, n_kv_heads=2, n_q_heads=8,
                    n_agents=1, prefix_len=37, seg_len=203, n_segments=2, n_anchors=5, tq=70)
SMALL_F32_D128 = scaled(workloads.TINY, name="small_f32_d128", head_dim=128, seg_len=77, prefix_len=5, tq=19,
                        n_anchors=3)
SMALL_BF16_D64 = scaled(SMALL_BF16, name="small_bf16_d64", head_dim=64, n_q_heads=2, seg_len=131)
SMALL_BF16_D256 = scaled(SMALL_BF16, name="small_bf16_d256", head_dim=256, n_layers=2, n_q_heads=4, seg_len=90, tq=45)
SMALL_F32_D256 = scaled(workloads.TINY, name="small_f32_d256", head_dim=256, seg_len=40, prefix_len=3, tq=9, n_anchors=2)


@pytest.mark.parametrize("w", [SMALL_BF16, SMALL_F32_D128, SMALL_BF16_D64, SMALL_BF16_D256, SMALL_F32_D256],
                         ids=lambda w: w.name)
def test_small_whole_hot_path(w):
    say(f"small whole path {w.name}")
    model = hotpath.model_of(w)
    agent = workloads.make_agent(w, 0, DEV)
    ck, cv = to_np(agent.cache_k), to_np(agent.cache_v)      # oracle's cache: generator rows only so far
    for j, seg in enumerate(agent.segments):
        p0, S = w.seg_offset(j), w.seg_len
        ref = oracle_segment(w, seg)
        ck[:, :, p0:p0 + S], cv[:, :, p0:p0 + S] = ref["out_k"], ref["out_v"]
        sc = hotpath.align_segment(model, seg, agent.cache_k[:, :, p0:p0 + S], agent.cache_v[:, :, p0:p0 + S],
                                   w.temperature)
        torch.cuda.synchronize()
        compare_segment(w, seg, sc, agent.cache_k[:, :, p0:p0 + S], agent.cache_v[:, :, p0:p0 + S], ref=ref)
    out, lse = kv.kvcomm_suffix_attn(model, agent.q, agent.cache_k, agent.cache_v, w.n_ctx, want_lse=True)
    torch.cuda.synchronize()
    want, want_lse = oracle.suffix_attn(to_np(agent.q), ck, cv, w.n_ctx, want_lse=True)
    check_close(to_np(out), want, w.dtype, "O")
    assert np.max(np.abs(lse.cpu().numpy() - want_lse)) < (2e-2 if w.dtype == torch.bfloat16 else 1e-4)


@pytest.mark.parametrize("n_anchors", [1, 2, 17, 64])
def test_anchor_counts(n_anchors):
    w = scaled(SMALL_BF16, n_anchors=n_anchors, seg_len=45, n_layers=2)
    say(f"anchor count {n_anchors}")
    seg = workloads.make_segment(w, 0, 0, DEV)
    sc, ok, ov = run_segment(w, seg)
    compare_segment(w, seg, sc, ok, ov)
    if n_anchors == 1:
        assert torch.all(sc.weights == 1.0)


def test_selection_of_shorter_anchors_and_none_selected():
    w = scaled(SMALL_BF16, n_anchors=4, seg_len=50, anchor_lens=(49, 50, 64, 10))
    say("selection")
    seg = workloads.make_segment(w, 0, 0, DEV)
    # poison what must never be read: tokens beyond an anchor's valid length
    for lst in (seg.anchor_k, seg.anchor_dk, seg.anchor_dv):
        lst[0][:, :, 49:] = float("nan")
        lst[3][:, :, 10:] = float("nan")
    sc, ok, ov = run_segment(w, seg)
    assert sc.selected.tolist() == [0, 1, 1, 0]
    assert torch.all(sc.weights[:, 0] == 0) and torch.all(sc.weights[:, 3] == 0)
    compare_segment(w, seg, sc, ok, ov)
    w0 = scaled(w, anchor_lens=(1, 2, 3, 4))
    seg = workloads.make_segment(w0, 0, 0, DEV)
    sc, ok, ov = run_segment(w0, seg)
    assert sc.selected.tolist() == [0, 0, 0, 0] and torch.all(sc.weights == 0) and torch.all(sc.nearest == -1)
    compare_segment(w0, seg, sc, ok, ov)   # pure re-positioning of the base cache


def test_duplicate_anchors_tie_and_identical_anchor():
    w = scaled(SMALL_BF16, n_anchors=4, seg_len=40)
    say("ties")
    seg = workloads.make_segment(w, 0, 0, DEV)
    seg.anchor_k[3] = seg.anchor_k[1].clone()          # exact duplicate: equal weights, lowest index nearest
    sc, ok, ov = run_segment(w, seg)
    assert torch.equal(sc.weights[:, 1], sc.weights[:, 3])
    assert not torch.any(sc.nearest == 3)
    compare_segment(w, seg, sc, ok, ov)
    seg.anchor_k[2] = seg.base_k.clone()               # identical to the segment: distance 0
    wc = scaled(w, temperature=1e-3)
    sc, ok, ov = run_segment(wc, seg)
    assert torch.all(sc.nearest == 2) and torch.all(sc.weights[:, 2] == 1.0)
    compare_segment(wc, seg, sc, ok, ov)


@pytest.mark.parametrize("delta", [0, 1, 8191, 131071])
def test_position_deltas(delta):
    w = scaled(SMALL_BF16, n_anchors=3, seg_len=33)
    say(f"delta {delta}")
    seg = workloads.make_segment(w, 0, 0, DEV)
    seg.delta_pos = delta
    sc, ok, ov = run_segment(w, seg)
    compare_segment(w, seg, sc, ok, ov)
    seg.anchor_delta_pos = [0, delta, 77]              # base frame, same frame, another frame
    sc, ok, ov = run_segment(w, seg)
    compare_segment(w, seg, sc, ok, ov)


def test_zero_deviation_zero_delta_is_bit_exact_identity_and_in_place():
    w = scaled(SMALL_BF16, n_anchors=3, seg_len=64)
    say("identity / in place")
    seg = workloads.make_segment(w, 0, 0, DEV)
    seg.delta_pos = 0
    for lst in (seg.anchor_dk, seg.anchor_dv):
        for t in lst:
            t.zero_()
    sc, ok, ov = run_segment(w, seg)
    assert torch.equal(ok, seg.base_k) and torch.equal(ov, seg.base_v)
    # in place gives the same bits as out of place
    seg = workloads.make_segment(w, 0, 0, DEV)
    _, ok, ov = run_segment(w, seg)
    _, ik, iv = run_segment(w, seg, in_place=True)
    assert torch.equal(ok, ik) and torch.equal(ov, iv)


def test_fp32_granularities_with_per_anchor_deltas():
    w = scaled(workloads.TINY, n_anchors=6, seg_len=70, anchor_delta_choices=(16, 64, 100))
    for gran in (kv.W_TOKEN, kv.W_LAYER_HEAD_TOKEN, kv.W_SEGMENT):
        say(f"fp32 per-anchor deltas gran={gran}")
        seg = workloads.make_segment(w, 0, 0, DEV)
        sc, ok, ov = run_segment(w, seg, gran)
        compare_segment(w, seg, sc, ok, ov, gran)


@pytest.mark.parametrize("n_ctx,tq,G", [(0, 1, 1), (0, 130, 4), (5, 1, 8), (1000, 3, 2), (129, 257, 4)])
def test_attention_shapes(n_ctx, tq, G):
    say(f"attn n_ctx={n_ctx} tq={tq} G={G}")
    for dtype in (torch.bfloat16, torch.float32):
        w = scaled(SMALL_BF16, dtype=dtype, n_kv_heads=2, n_q_heads=2 * G, prefix_len=n_ctx, n_segments=0, tq=tq,
                   n_layers=2)
        model = hotpath.model_of(w)
        agent = workloads.make_agent(w, 1, DEV)
        out = kv.kvcomm_suffix_attn(model, agent.q, agent.cache_k, agent.cache_v, w.n_ctx)
        torch.cuda.synchronize()
        want = oracle.suffix_attn(to_np(agent.q), to_np(agent.cache_k), to_np(agent.cache_v), w.n_ctx)
        check_close(to_np(out), want, dtype, f"O {dtype}")


def test_attention_large_scores_and_custom_scale():
    w = scaled(SMALL_BF16, n_segments=0, prefix_len=300, tq=64)
    say("attn large scores")
    model = hotpath.model_of(w)
    agent = workloads.make_agent(w, 2, DEV)
    agent.q.mul_(6.0)   # scores of several tens: the online softmax must not overflow
    out = kv.kvcomm_suffix_attn(model, agent.q, agent.cache_k, agent.cache_v, w.n_ctx, softmax_scale=0.2)
    torch.cuda.synchronize()
    want = oracle.suffix_attn(to_np(agent.q), to_np(agent.cache_k), to_np(agent.cache_v), w.n_ctx, scale=0.2)
    check_close(to_np(out), want, w.dtype, "O")


@pytest.mark.parametrize("n_ctx,tq", [(0, 512), (40, 512), (0, 300)])
def test_attention_short_context_full_blocks(n_ctx, tq):
    """Blocks of eight wavefronts whose row tile sees three or more key tiles with next to no context before it.

    The first two 32-key halves of a block are read before the main loop, and the first tile of the loop requests
    the fifth and sixth halves into the same two slots of the ring of key buffers: a barrier after the first
    scores keeps a fast wavefront's request from overwriting keys that a slow one has not read yet.  With so
    short a context every block reaches that reuse at once, on every (layer, head)."""
    w = scaled(SMALL_BF16, n_layers=3, n_kv_heads=2, n_q_heads=8, prefix_len=n_ctx, n_segments=0, tq=tq)
    say(f"attn short context n_ctx={n_ctx} tq={tq}")
    model = hotpath.model_of(w)
    agent = workloads.make_agent(w, 3, DEV)
    out = kv.kvcomm_suffix_attn(model, agent.q, agent.cache_k, agent.cache_v, w.n_ctx)
    torch.cuda.synchronize()
    want = oracle.suffix_attn(to_np(agent.q), to_np(agent.cache_k), to_np(agent.cache_v), w.n_ctx)
    check_close(to_np(out), want, w.dtype, "O")


@pytest.mark.parametrize("max_blocks", [8, 9, 13, 24, 47, 48, 1000])
def test_attention_confined_is_bit_identical(max_blocks):
    """The persistent form of the attention launch (at most max_blocks thread blocks, each walking a share of the
    work items of its XCD): same bits as the plain launch, for grids smaller than, equal to and larger than the
    number of items (48 here: 3 layers x 2 kv heads x 8 row tiles), including grids that leave some XCD with fewer
    blocks than others and blocks with nothing to do."""
    w = scaled(SMALL_BF16, n_layers=3, n_kv_heads=2, n_q_heads=8, prefix_len=100, n_segments=0, tq=500)
    say(f"attn confined max_blocks={max_blocks}")
    model = hotpath.model_of(w)
    agent = workloads.make_agent(w, 5, DEV)
    out, lse = kv.kvcomm_suffix_attn(model, agent.q, agent.cache_k, agent.cache_v, w.n_ctx, want_lse=True)
    out2, lse2 = kv.kvcomm_suffix_attn_confined(model, agent.q, agent.cache_k, agent.cache_v, w.n_ctx, max_blocks,
                                                want_lse=True)
    torch.cuda.synchronize()
    assert torch.equal(out, out2) and torch.equal(lse, lse2)
    if max_blocks == 13:
        want = oracle.suffix_attn(to_np(agent.q), to_np(agent.cache_k), to_np(agent.cache_v), w.n_ctx)
        check_close(to_np(out2), want, w.dtype, "O")


@pytest.mark.parametrize("w", [SMALL_BF16_D64, SMALL_BF16_D256, SMALL_F32_D128], ids=lambda w: w.name)
def test_attention_confined_other_head_dims_and_fp32(w):
    say(f"attn confined {w.name}")
    model = hotpath.model_of(w)
    agent = workloads.make_agent(w, 6, DEV)
    out = kv.kvcomm_suffix_attn(model, agent.q, agent.cache_k, agent.cache_v, w.n_ctx)
    out2 = kv.kvcomm_suffix_attn_confined(model, agent.q, agent.cache_k, agent.cache_v, w.n_ctx, 8)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)


def test_two_stream_pipeline_equals_sequential_steps():
    """hotpath.TwoStreamPipeline (weights + alignment of the next agent beside the confined attention of the current
    one; two buffer sets; several steps, the inputs of every step different) against the same calls on one stream:
    bit-identical outputs for every agent of every step, i.e. the events order every read behind its write."""
    w = scaled(SMALL_BF16, n_layers=3, n_agents=2, seg_len=128, n_segments=2, prefix_len=40, tq=300)
    say("two-stream pipeline")
    model = hotpath.model_of(w)
    agents = [workloads.make_agent(w, a, DEV) for a in range(2)]
    scr = [hotpath.AgentScratch(model, [w.seg_len] * w.n_segments, [w.n_anchors] * w.n_segments, kv.W_TOKEN, DEV)
           for _ in agents]

    def jobs(ai):
        ag, sc = agents[ai], scr[ai]
        wj = [dict(seg_base_k=s.base_k, anchor_base_k=s.anchor_k, anchor_len=s.anchor_len, weights_out=sc.weights[j],
                   nearest_out=sc.nearest[j], selected_out=sc.selected[j]) for j, s in enumerate(ag.segments)]
        aj = [dict(base_k=s.base_k, base_v=s.base_v, anchor_dk=s.anchor_dk, anchor_dv=s.anchor_dv,
                   anchor_len=s.anchor_len, weights=sc.weights[j], delta_pos=s.delta_pos,
                   anchor_delta_pos=s.anchor_delta_pos,
                   out_k=ag.cache_k[:, :, w.seg_offset(j):w.seg_offset(j) + w.seg_len],
                   out_v=ag.cache_v[:, :, w.seg_offset(j):w.seg_offset(j) + w.seg_len])
              for j, s in enumerate(ag.segments)]
        return wj, aj

    J = [jobs(0), jobs(1)]
    n_steps = 4
    base0 = [[s.base_k.clone() for s in ag.segments] for ag in agents]

    def set_inputs(step):   # every step works on different base keys, so a stale read would show
        for ai, ag in enumerate(agents):
            for j, s in enumerate(ag.segments):
                s.base_k.copy_(base0[ai][j] * (1.0 + 0.25 * step))

    # sequential reference: one stream, synchronised step by step
    want = []
    for step in range(n_steps):
        set_inputs(step)
        for ai, ag in enumerate(agents):
            kv.kvcomm_anchor_weights_batch(model, J[ai][0], w.temperature, kv.W_TOKEN, workspace=scr[ai].workspace)
            kv.kvcomm_align_kv_batch(model, J[ai][1], kv.W_TOKEN)
            want.append(kv.kvcomm_suffix_attn(model, ag.q, ag.cache_k, ag.cache_v, w.n_ctx).clone())
        torch.cuda.synchronize()
    for blocks in (8, 11, 0):
        pipe = hotpath.TwoStreamPipeline(model, w.temperature, attn_blocks=blocks)
        outs = [torch.empty_like(agents[0].q) for _ in range(n_steps * 2)]
        for step in range(n_steps):
            set_inputs(step)          # on the current stream; fork() puts the pipeline behind it
            pipe.fork()
            for ai, ag in enumerate(agents):
                pipe.submit(ai, J[ai][0], J[ai][1], scr[ai].workspace, ag.q, ag.cache_k, ag.cache_v, w.n_ctx,
                            outs[2 * step + ai])
            pipe.join()               # the next step's inputs are written behind this step's reads
        torch.cuda.synchronize()
        for i, (got, ref) in enumerate(zip(outs, want)):
            assert torch.equal(got, ref), f"attn_blocks {blocks}: step {i // 2} agent {i % 2}"


# ------------------------------------------------- full-size configurations, sampled outputs
def sample_tokens(S, seed, n_min=64):
    """At least n_min tokens of a segment: both ends, every multiple of 16 in the first and the last 128 tokens
    and the middle one with its two neighbours (the kernels' blocks take 16 or 32 tokens, so these are the first
    and last rows of blocks at the start, in the middle and in the ragged end of the grid), the rest random."""
    edges = {0, 1, S - 2, S - 1}
    for m in list(range(16, min(S, 129), 16)) + list(range(max(S - 128, 16), S, 16)) + [S // 2]:
        edges.update((m - 1, m, m + 1))
    tokens = {t for t in edges if 0 <= t < S}
    g = np.random.default_rng(seed)
    while len(tokens) < min(n_min, S):
        tokens.add(int(g.integers(0, S)))
    return sorted(tokens)


def attention_pairs(w, seed):
    """(layer, query head) pairs: every position g of the grouped-query group, on the first and the last kv head
    in turn, layers spread over the depth; plus the very first and the very last pair."""
    G = w.n_q_heads // w.n_kv_heads
    g = np.random.default_rng(1000 + seed)
    pairs = [(0, 0), (w.n_layers - 1, w.n_q_heads - 1)]
    for i in range(G):
        hk = 0 if i % 2 == 0 else w.n_kv_heads - 1
        pairs.append((int(g.integers(w.n_layers)), hk * G + i))
    for i in range(G):                                   # the other kv head for each g
        hk = w.n_kv_heads - 1 if i % 2 == 0 else 0
        pairs.append((int(g.integers(w.n_layers)), hk * G + i))
    return sorted(set(pairs))


def oracle_token_weights(w, seg, layers_per_chunk=8):
    """The oracle's per-token weights of ALL tokens of a full-size segment.

    The oracle's distance is the root of a sum of squares over (layer, head, channel).  To stay within host
    memory it is called on chunks of layers and the squares of its values are added: the root of that sum is
    its value on all layers (up to the order of the additions)."""
    L = seg.base_k.shape[0]
    sq, sel = None, None
    for l0 in range(0, L, layers_per_chunk):
        l1 = min(l0 + layers_per_chunk, L)
        d, sel = oracle.distances(to_np(seg.base_k[l0:l1]), [to_np(a[l0:l1]) for a in seg.anchor_k])
        sq = d * d if sq is None else sq + d * d
    return oracle.weights(np.sqrt(sq), sel, w.temperature)


def check_agent_sampled(w, agent_id, seg_ids=None, chain=True):
    """Full-size parity of one agent.

    Every segment in seg_ids (default: all): weights / nearest / selected / K^ / V^ on sampled tokens (all
    layers and heads).
    chain=True: the oracle also computes the weights of ALL tokens and aligns the sampled kv heads
    itself, so the attention check runs end to end with no oracle input taken from the GPU path.
    chain=False: attention is checked on a cache whose segment slots hold generator values, then the
    aligned cache is checked for sanity.
    """
    model = hotpath.model_of(w)
    G = w.n_q_heads // w.n_kv_heads
    seg_ids = range(w.n_segments) if seg_ids is None else seg_ids
    agent = workloads.make_agent(w, agent_id, DEV, with_segments=False)
    pairs = attention_pairs(w, agent_id)
    ocache = {}
    if w.tq and not chain:
        say(f"  {w.name} agent {agent_id} attention on generator-filled cache, {len(pairs)} (layer, head) pairs")
        gen = torch.Generator(device=DEV)
        gen.manual_seed(777 + agent_id)
        for c in (agent.cache_k, agent.cache_v):
            c[:, :, w.prefix_len:w.n_ctx] = torch.randn(c[:, :, w.prefix_len:w.n_ctx].shape, generator=gen,
                                                        device=DEV).to(w.dtype)
        out = kv.kvcomm_suffix_attn(model, agent.q, agent.cache_k, agent.cache_v, w.n_ctx)
        torch.cuda.synchronize()
        for (l, hq), (want, _) in oracle_attention(w, agent, pairs).items():
            check_close(to_np(out[l, hq]), want, w.dtype, f"O[{l},{hq}]")
    if w.tq and chain:
        for (l, hq) in pairs:
            hk = hq // G
            if (l, hk) not in ocache:
                ocache[(l, hk)] = (to_np(agent.cache_k[l, hk]), to_np(agent.cache_v[l, hk]))   # generator rows
    guard_k = agent.cache_k[:, :, : w.prefix_len].clone()
    for j in range(w.n_segments):
        say(f"  {w.name} agent {agent_id} segment {j}")
        seg = workloads.make_segment(w, agent_id, j, DEV)
        p0, S = w.seg_offset(j), w.seg_len
        ok, ov = agent.cache_k[:, :, p0:p0 + S], agent.cache_v[:, :, p0:p0 + S]
        sc = hotpath.align_segment(model, seg, ok, ov, w.temperature)
        torch.cuda.synchronize()
        if j in seg_ids:
            compare_segment(w, seg, sc, ok, ov, tokens=sample_tokens(S, 10 * agent_id + j))
        # properties that hold at any size
        ws = sc.weights.sum(1)
        assert torch.allclose(ws, torch.ones_like(ws), atol=1e-5)
        assert torch.isfinite(ok.float()).all() and torch.isfinite(ov.float()).all()
        if ocache:
            wts, nearest = oracle_token_weights(w, seg)
            assert np.array_equal(sc.nearest.cpu().numpy(), nearest)
            check_weights(sc.weights.cpu().numpy(), wts.T)
            for (l, hk), (ck, cv) in ocache.items():
                cut = lambda t: to_np(t[l:l + 1, hk:hk + 1])
                rk, rv = oracle.align(cut(seg.base_k), cut(seg.base_v), [cut(a) for a in seg.anchor_dk],
                                      [cut(a) for a in seg.anchor_dv], wts, seg.delta_pos, w.rope_theta,
                                      seg.anchor_delta_pos)
                ck[p0:p0 + S], cv[p0:p0 + S] = rk[0, 0], rv[0, 0]
                # every token of these (layer, kv head) rows of the aligned cache, not only the sampled ones
                check_close(to_np(ok[l, hk]), rk[0, 0], w.dtype, f"K^[{l},{hk}] seg {j}")
                check_close(to_np(ov[l, hk]), rv[0, 0], w.dtype, f"V^[{l},{hk}] seg {j}")
        del seg
    assert torch.equal(agent.cache_k[:, :, : w.prefix_len], guard_k)
    if not w.tq:
        return
    say(f"  {w.name} agent {agent_id} attention")
    out = kv.kvcomm_suffix_attn(model, agent.q, agent.cache_k, agent.cache_v, w.n_ctx)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    for (l, hq) in pairs if chain else []:
        ck, cv = ocache[(l, hq // G)]
        want = oracle.suffix_attn(to_np(agent.q[l:l + 1, hq:hq + 1]), ck[None, None], cv[None, None], w.n_ctx)
        check_close(to_np(out[l, hq]), want[0, 0], w.dtype, f"O[{l},{hq}]")


def test_sampled_tokens_and_pairs_cover_the_edges():
    for S in (512, 1024, 2048):
        t = sample_tokens(S, 0)
        assert len(t) >= 64 and t[0] == 0 and t[-1] == S - 1
        assert {15, 16, 17, 31, 32, 33, S - 33, S - 32, S - 31, S - 17, S - 16, S - 15} <= set(t)
    for w in (workloads.LLAMA8B_5AGENTS, workloads.LONG_CONTEXT, workloads.LLAMA70B):
        G = w.n_q_heads // w.n_kv_heads
        pairs = attention_pairs(w, 0)
        for hk in (0, w.n_kv_heads - 1):
            assert {hq % G for _, hq in pairs if hq // G == hk} == set(range(G))


def test_config2_llama8b_5agents_sampled():
    check_agent_sampled(workloads.LLAMA8B_5AGENTS, 0)


def test_config2_llama8b_5agents_last_agent_sampled():
    check_agent_sampled(workloads.LLAMA8B_5AGENTS, 4, chain=False)


@pytest.mark.parametrize("w", workloads.POOL_SCALING, ids=lambda w: w.name)
def test_config3_pool_scaling_sampled(w):
    check_agent_sampled(w, 0)


def test_config4_long_context_sampled():
    check_agent_sampled(workloads.LONG_CONTEXT, 5)


def test_config4_long_context_second_agent_sampled():
    check_agent_sampled(workloads.LONG_CONTEXT, 0, chain=False)


def test_config5_llama70b_sampled_and_chained():
    """Every segment on sampled tokens, and the attention of the sampled (layer, head) pairs on a cache the
    oracle aligned itself from its own all-token weights (distances summed over chunks of layers)."""
    check_agent_sampled(workloads.LLAMA70B, 2)


def test_config5_llama70b_second_agent_sampled():
    check_agent_sampled(workloads.LLAMA70B, 0, chain=False)


def test_config2_batched_launch_as_benchmarked():
    """Config 2 in the launch configuration the benchmark times: the four segments of an agent in one
    batched launch per stage, then attention.  Oracle on sampled tokens of every segment (tokens are
    independent under per-token weights) and on sampled (layer, query head) pairs of the attention, whose
    reference cache is assembled by the oracle itself for those kv heads."""
    w = workloads.LLAMA8B_5AGENTS
    agent_id = 1
    say(f"{w.name} agent {agent_id}, batched")
    model = hotpath.model_of(w)
    G = w.n_q_heads // w.n_kv_heads
    agent = workloads.make_agent(w, agent_id, DEV)
    pairs = attention_pairs(w, agent_id)
    ocache = {}
    for l, hq in pairs:
        ocache.setdefault((l, hq // G), (to_np(agent.cache_k[l, hq // G]), to_np(agent.cache_v[l, hq // G])))
    sc = hotpath.align_agent_batched(w, model, agent)
    out = kv.kvcomm_suffix_attn(model, agent.q, agent.cache_k, agent.cache_v, w.n_ctx)
    torch.cuda.synchronize()
    for j, seg in enumerate(agent.segments):
        p0, S = w.seg_offset(j), w.seg_len
        tokens = sample_tokens(S, 100 + j)
        ref = oracle_segment(w, seg, tokens)
        idx = torch.as_tensor(tokens, device=DEV)
        assert np.array_equal(sc.selected[j].cpu().numpy(), ref["selected"])
        assert np.array_equal(sc.nearest[j].cpu().numpy()[tokens], ref["nearest"])
        check_weights(sc.weights[j].cpu().numpy()[tokens], ref["w"].T)
        check_close(to_np(agent.cache_k[:, :, p0:p0 + S][:, :, idx]), ref["out_k"], w.dtype, f"K^ seg {j}")
        check_close(to_np(agent.cache_v[:, :, p0:p0 + S][:, :, idx]), ref["out_v"], w.dtype, f"V^ seg {j}")
        # the oracle's own cache for the sampled kv heads: all tokens of the segment
        dist, sel = oracle.distances(to_np(seg.base_k), [to_np(a) for a in seg.anchor_k])
        wts, _ = oracle.weights(dist, sel, w.temperature)
        for (l, hk), (ck, cv) in ocache.items():
            cut = lambda t: to_np(t[l:l + 1, hk:hk + 1])
            rk, rv = oracle.align(cut(seg.base_k), cut(seg.base_v), [cut(a) for a in seg.anchor_dk],
                                  [cut(a) for a in seg.anchor_dv], wts, seg.delta_pos, w.rope_theta)
            ck[p0:p0 + S], cv[p0:p0 + S] = rk[0, 0], rv[0, 0]
    for (l, hq) in pairs:
        ck, cv = ocache[(l, hq // G)]
        want = oracle.suffix_attn(to_np(agent.q[l:l + 1, hq:hq + 1]), ck[None, None], cv[None, None], w.n_ctx)
        check_close(to_np(out[l, hq]), want[0, 0], w.dtype, f"O[{l},{hq}]")


@pytest.mark.parametrize("n_anchors,lens", [(5, None), (16, None), (17, None), (4, (1, 2, 3, 4)), (18, (60,) * 9 + (3,) * 9)])
def test_layer_head_token_weights_fused_and_two_stage(n_anchors, lens):
    """One softmax per (layer, head, token): the distance kernel finishes the softmax itself for pools of up to 16
    selected anchors and falls back to the two-stage form otherwise (larger pools, nothing selected)."""
    w = scaled(SMALL_BF16, n_anchors=n_anchors, seg_len=45, n_layers=2, anchor_lens=lens)
    say(f"layer-head-token weights A={n_anchors} lens={lens}")
    seg = workloads.make_segment(w, 0, 0, DEV)
    sc, ok, ov = run_segment(w, seg, kv.W_LAYER_HEAD_TOKEN)
    compare_segment(w, seg, sc, ok, ov, kv.W_LAYER_HEAD_TOKEN)
