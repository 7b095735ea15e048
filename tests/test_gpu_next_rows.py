"""GPU parity of the rows beyond the reuse step proper: weighting variants (nearest, cosine),
anchor prediction (Eq. "pred") and offset capture (fallback branch of Algorithm 1), through
the C ABI against the float64 oracle.  Integers bit-exact, floats to tests/parity.py's rules.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_12872_amd as kv
from paper_2510_12872_amd import hotpath, workloads
from paper_2510_12872_amd.workloads import scaled

from parity import check_close, check_weights, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda"

SMALL_BF16 = scaled(workloads.LLAMA8B_5AGENTS, name="small_bf16", n_layers=3, n_kv_heads=2, n_q_heads=8,
                    n_agents=1, prefix_len=37, seg_len=203, n_segments=1, n_anchors=5, tq=0)
SMALL_F32 = scaled(workloads.TINY, name="small_f32", seg_len=77, prefix_len=5, tq=0, n_anchors=3)
RAGGED = scaled(SMALL_BF16, name="ragged", n_anchors=11, seg_len=50,
                anchor_lens=(49, 50, 64, 10, 50, 50, 50, 60, 50, 50, 50))


def say(msg):
    print(msg, flush=True)


def oracle_inputs(seg):
    S = seg.base_k.shape[2]
    anc = [to_np(a) if n >= S else np.zeros(seg.base_k.shape[:2] + (0, seg.base_k.shape[3]))
           for a, n in zip(seg.anchor_k, seg.anchor_len)]
    return to_np(seg.base_k), anc


# ------------------------------------------------------------------------- weighting variants
@pytest.mark.parametrize("w", [SMALL_BF16, SMALL_F32, RAGGED], ids=lambda w: w.name)
@pytest.mark.parametrize("gran", [kv.W_TOKEN, kv.W_LAYER_HEAD_TOKEN, kv.W_SEGMENT])
def test_nearest_and_cosine_rules(w, gran):
    say(f"rules {w.name} gran={gran}")
    model = hotpath.model_of(w)
    seg = workloads.make_segment(w, 0, 0, DEV)
    if w is RAGGED:   # what must never be read
        seg.anchor_k[0][:, :, 49:] = float("nan")
        seg.anchor_k[3][:, :, 10:] = float("nan")
    bk, anc = oracle_inputs(seg)
    dist, sel = oracle.distances(bk, anc, gran)
    # default rule through the new entry point == the original entry point, bit for bit
    w0, n0, s0 = kv.kvcomm_anchor_weights(model, seg.base_k, seg.anchor_k, seg.anchor_len, 0.7, gran)
    w1, n1, s1 = kv.kvcomm_anchor_weights_rule(model, kv.RULE_L2_SOFTMAX, seg.base_k, seg.anchor_k, seg.anchor_len,
                                               0.7, gran)
    torch.cuda.synchronize()
    assert torch.equal(w0, w1) and torch.equal(n0, n1) and torch.equal(s0, s1)
    want, near = oracle.weights(dist, sel, 0.7)
    check_weights(w1.cpu().numpy(), want.T)
    assert np.array_equal(n1.cpu().numpy(), near)
    # nearest
    wn, nn, sn = kv.kvcomm_anchor_weights_rule(model, kv.RULE_NEAREST, seg.base_k, seg.anchor_k, seg.anchor_len,
                                               1.0, gran)
    torch.cuda.synchronize()
    want, near = oracle.weights_nearest(dist, sel)
    assert np.array_equal(sn.cpu().numpy(), sel)
    assert np.array_equal(nn.cpu().numpy(), near)
    assert np.array_equal(wn.cpu().numpy(), want.T.astype(np.float32))      # one-hot: exact
    # cosine
    for tau in (1.0, 0.05):
        wc, nc, sc = kv.kvcomm_anchor_weights_rule(model, kv.RULE_COSINE_SOFTMAX, seg.base_k, seg.anchor_k,
                                                   seg.anchor_len, tau, gran)
        torch.cuda.synchronize()
        sim, sel_c = oracle.cosine(bk, anc, gran)
        want, best = oracle.weights_from_sim(sim, sel_c, tau)
        assert np.array_equal(sc.cpu().numpy(), sel_c)
        assert np.array_equal(nc.cpu().numpy(), best)
        check_weights(wc.cpu().numpy(), want.T, "cosine weights")


def test_rules_with_duplicate_and_identical_anchors():
    w = scaled(SMALL_BF16, n_anchors=4, seg_len=33)
    say("rules ties")
    model = hotpath.model_of(w)
    seg = workloads.make_segment(w, 0, 0, DEV)
    seg.anchor_k[2] = seg.anchor_k[1].clone()          # exact tie between 1 and 2
    seg.anchor_k[3] = seg.base_k.clone()               # identical to the sample
    wn, nn, _ = kv.kvcomm_anchor_weights_rule(model, kv.RULE_NEAREST, seg.base_k, seg.anchor_k, seg.anchor_len)
    wc, nc, _ = kv.kvcomm_anchor_weights_rule(model, kv.RULE_COSINE_SOFTMAX, seg.base_k, seg.anchor_k, seg.anchor_len,
                                              0.01)
    torch.cuda.synchronize()
    assert torch.all(nn == 3) and torch.all(wn[:, 3] == 1) and torch.all(wn[:, :3] == 0)
    assert torch.all(nc == 3) and torch.all(wc[:, 3] > 0.999)
    assert torch.equal(wc[:, 1], wc[:, 2])
    seg.anchor_k[3] = seg.anchor_k[0].clone()          # ties 0 == 3 and 1 == 2: lowest index wins
    wn, nn, _ = kv.kvcomm_anchor_weights_rule(model, kv.RULE_NEAREST, seg.base_k, seg.anchor_k, seg.anchor_len)
    torch.cuda.synchronize()
    bk, anc = oracle_inputs(seg)
    dist, sel = oracle.distances(bk, anc)
    _, near = oracle.weights_nearest(dist, sel)
    assert np.array_equal(nn.cpu().numpy(), near) and set(near.tolist()) <= {0, 1}
    # the same ties under the cosine rule: equal weights, lowest index is the most similar anchor
    wc, nc, _ = kv.kvcomm_anchor_weights_rule(model, kv.RULE_COSINE_SOFTMAX, seg.base_k, seg.anchor_k, seg.anchor_len,
                                              0.2)
    torch.cuda.synchronize()
    sim, sel_c = oracle.cosine(bk, anc)
    want, best = oracle.weights_from_sim(sim, sel_c, 0.2)
    assert np.array_equal(nc.cpu().numpy(), best) and set(best.tolist()) <= {0, 1}
    assert torch.equal(wc[:, 0], wc[:, 3]) and torch.equal(wc[:, 1], wc[:, 2])
    check_weights(wc.cpu().numpy(), want.T, "cosine weights with ties")


def test_nearest_rule_feeds_align():
    """Nearest-anchor approximation end to end: K^ = R K + R dK_nearest, V^ = V + dV_nearest."""
    w = scaled(SMALL_BF16, n_anchors=6, seg_len=70)
    say("nearest -> align")
    model = hotpath.model_of(w)
    seg = workloads.make_segment(w, 0, 0, DEV)
    wn, nn, _ = kv.kvcomm_anchor_weights_rule(model, kv.RULE_NEAREST, seg.base_k, seg.anchor_k, seg.anchor_len)
    ok, ov = torch.empty_like(seg.base_k), torch.empty_like(seg.base_v)
    kv.kvcomm_align_kv(model, seg.base_k, seg.base_v, seg.anchor_dk, seg.anchor_dv, wn, seg.delta_pos, ok, ov,
                       seg.anchor_len)
    torch.cuda.synchronize()
    bk, anc = oracle_inputs(seg)
    dist, sel = oracle.distances(bk, anc)
    wo, _ = oracle.weights_nearest(dist, sel)
    rk, rv = oracle.align(bk, to_np(seg.base_v), [to_np(a) for a in seg.anchor_dk], [to_np(a) for a in seg.anchor_dv],
                          wo, seg.delta_pos, w.rope_theta)
    check_close(to_np(ok), rk, w.dtype, "K^ nearest")
    check_close(to_np(ov), rv, w.dtype, "V^ nearest")


def test_rule_full_size_sampled_tokens():
    """Config-2 segment at full size, cosine and nearest, oracle on sampled tokens (tokens are independent)."""
    w = scaled(workloads.LLAMA8B_5AGENTS, n_agents=1, n_segments=1)
    say("rules full size")
    model = hotpath.model_of(w)
    seg = workloads.make_segment(w, 0, 0, DEV)
    tokens = [0, 1, 255, 256, 300, 511]
    idx = torch.as_tensor(tokens, device=DEV)
    bk = to_np(seg.base_k[:, :, idx])
    anc = [to_np(a[:, :, idx]) for a in seg.anchor_k]
    wc, nc, _ = kv.kvcomm_anchor_weights_rule(model, kv.RULE_COSINE_SOFTMAX, seg.base_k, seg.anchor_k, seg.anchor_len)
    wn, nn, _ = kv.kvcomm_anchor_weights_rule(model, kv.RULE_NEAREST, seg.base_k, seg.anchor_k, seg.anchor_len)
    torch.cuda.synchronize()
    sim, sel = oracle.cosine(bk, anc)
    want, best = oracle.weights_from_sim(sim, sel, 1.0)
    check_weights(wc.cpu().numpy()[tokens], want.T, "cosine weights")
    assert np.array_equal(nc.cpu().numpy()[tokens], best)
    dist, sel = oracle.distances(bk, anc)
    want, near = oracle.weights_nearest(dist, sel)
    assert np.array_equal(nn.cpu().numpy()[tokens], near)
    assert np.array_equal(wn.cpu().numpy()[tokens], want.T.astype(np.float32))


# ------------------------------------------------------------------------- anchor prediction
@pytest.mark.parametrize("n_slots", [1, 7, 256, 1000, 300001])
def test_predict_on_seeded_weights(n_slots):
    say(f"predict n={n_slots}")
    g = torch.Generator().manual_seed(n_slots)
    A = 6
    wts = torch.softmax(torch.randn((n_slots, A), generator=g) * 2.0, dim=1).to(torch.float32)
    lens = [40, 50, 64, 50, 10, 50]
    wts[:, [0, 4]] = 0.0                                   # unselected anchors carry no weight
    wts = (wts / wts.sum(1, keepdim=True)).contiguous()
    sel = np.array([int(x >= 50) for x in lens], dtype=np.intc)
    new_o, ent_o, mean_o = oracle.predict(wts.numpy().T, sel, lens, 50, 0.0)
    res, ent = kv.kvcomm_anchor_predict(wts.to(DEV), lens, 50, 0.3, want_entropy=True)
    torch.cuda.synchronize()
    np.testing.assert_allclose(ent.cpu().numpy(), ent_o, atol=1e-5)
    assert abs(float(res[1]) - mean_o) <= 1e-5
    # decisions for thresholds well on either side of the mean entropy
    for gamma in (0.0, 0.5 * mean_o / np.log(4), 1.5 * mean_o / np.log(4), 10.0):
        gamma = float(np.float32(gamma))
        want = oracle.predict(wts.numpy().T, sel, lens, 50, gamma)[0]
        got = kv.kvcomm_anchor_predict(wts.to(DEV), lens, 50, gamma)
        torch.cuda.synchronize()
        assert int(got[0]) == want, gamma
    # longer than every anchor / no candidate: new anchor whatever the weights
    assert int(kv.kvcomm_anchor_predict(wts.to(DEV), lens, 65, 10.0)[0]) == 1 == oracle.predict(
        wts.numpy().T, np.zeros(A, dtype=np.intc), lens, 65, 10.0)[0]


def test_predict_closed_forms_and_chain():
    say("predict closed forms")
    A = 4
    uni = torch.full((3, A), 0.25, device=DEV)
    res, ent = kv.kvcomm_anchor_predict(uni, [8] * A, 8, 0.99, want_entropy=True)
    assert int(res[0]) == 1 and abs(float(res[1]) - np.log(4)) < 1e-6
    assert int(kv.kvcomm_anchor_predict(uni, [8] * A, 8, 1.01)[0]) == 0
    hot = torch.zeros((3, A), device=DEV)
    hot[:, 2] = 1.0
    res = kv.kvcomm_anchor_predict(hot, [8] * A, 8, 0.3)
    assert int(res[0]) == 0 and float(res[1]) == 0.0
    # chained with the device weights: segment granularity = the paper's scalar case
    w = scaled(SMALL_BF16, n_anchors=5, seg_len=64)
    model = hotpath.model_of(w)
    seg = workloads.make_segment(w, 0, 0, DEV)
    for gran in (kv.W_SEGMENT, kv.W_TOKEN):
        wd, _, _ = kv.kvcomm_anchor_weights(model, seg.base_k, seg.anchor_k, seg.anchor_len, 1.0, gran)
        res = kv.kvcomm_anchor_predict(wd, seg.anchor_len, w.seg_len, 0.3)
        torch.cuda.synchronize()
        bk, anc = oracle_inputs(seg)
        dist, sel = oracle.distances(bk, anc, gran)
        wo, _ = oracle.weights(dist, sel, 1.0)
        new, _, mean = oracle.predict(wo, sel, seg.anchor_len, w.seg_len, float(np.float32(0.3)))
        assert abs(float(res[1]) - mean) < 1e-4
        if abs(mean - 0.3 * np.log(5)) > 1e-3:
            assert int(res[0]) == new


# ------------------------------------------------------------------------- offset capture
@pytest.mark.parametrize("w", [SMALL_BF16, SMALL_F32, scaled(SMALL_BF16, name="bf16_d64", head_dim=64, n_q_heads=2)],
                         ids=lambda w: w.name)
@pytest.mark.parametrize("delta", [0, 300, 131071])
def test_capture_offsets(w, delta):
    say(f"capture {w.name} delta={delta}")
    model = hotpath.model_of(w)
    seg = workloads.make_segment(w, 0, 0, DEV)
    # "real" cache of a dense prefill: an independent N(0,1) draw (any tensor exercises the arithmetic);
    # the offsets then stay below 8 in magnitude, where half a bf16 ulp is within the 2e-2 bound
    g = torch.Generator(device=DEV).manual_seed(1234 + delta)
    shape = seg.base_k.shape
    real_k = torch.randn(shape, generator=g, device=DEV).to(w.dtype)
    real_v = torch.randn(shape, generator=g, device=DEV).to(w.dtype)
    # real tensors as strided views into a longer cache, as in the agent's cache
    cache_k = torch.zeros(shape[:2] + (shape[2] + 24, shape[3]), dtype=w.dtype, device=DEV)
    cache_v = torch.zeros_like(cache_k)
    cache_k[:, :, 8:8 + shape[2]] = real_k
    cache_v[:, :, 8:8 + shape[2]] = real_v
    dk, dv = kv.kvcomm_capture_offsets(model, seg.base_k, seg.base_v, cache_k[:, :, 8:8 + shape[2]],
                                       cache_v[:, :, 8:8 + shape[2]], delta)
    torch.cuda.synchronize()
    want_k, want_v = oracle.capture(to_np(seg.base_k), to_np(seg.base_v), to_np(real_k), to_np(real_v), delta,
                                    w.rope_theta)
    check_close(to_np(dk), want_k, w.dtype, "dK")
    check_close(to_np(dv), want_v, w.dtype, "dV")
    if delta == 0 and w.dtype == torch.float32:
        assert torch.equal(dk, real_k - seg.base_k) and torch.equal(dv, real_v - seg.base_v)


def test_capture_then_align_reproduces_real_cache_fp32():
    """A captured anchor of weight 1 gives back the real cache (round trip through both kernels)."""
    w = scaled(SMALL_F32, seg_len=61)
    say("capture round trip")
    model = hotpath.model_of(w)
    seg = workloads.make_segment(w, 0, 0, DEV)
    g = torch.Generator(device=DEV).manual_seed(5)
    real_k = torch.randn(seg.base_k.shape, generator=g, device=DEV)
    real_v = torch.randn(seg.base_k.shape, generator=g, device=DEV)
    dk, dv = kv.kvcomm_capture_offsets(model, seg.base_k, seg.base_v, real_k, real_v, 777)
    ones = torch.ones((w.seg_len, 1), device=DEV)
    ok, ov = torch.empty_like(real_k), torch.empty_like(real_v)
    kv.kvcomm_align_kv(model, seg.base_k, seg.base_v, [dk], [dv], ones, 777, ok, ov)
    torch.cuda.synchronize()
    assert float((ok - real_k).abs().max()) < 1e-5 and float((ov - real_v).abs().max()) < 1e-6


# ------------------------------------------------------------------------- batched launches
def test_batched_agent_equals_per_segment_calls():
    """All segments of an agent in one launch per step: K^/V^ bit-identical to per-segment calls
    (same arithmetic in the same order); weights equal up to the cut of the double partial sums."""
    w = scaled(workloads.LLAMA8B_5AGENTS, name="batch", n_layers=3, n_kv_heads=2, n_q_heads=8, n_agents=1,
               prefix_len=16, seg_len=97, n_segments=4, n_anchors=5, tq=8, anchor_delta_choices=(16, 64, 100))
    say("batched agent")
    model = hotpath.model_of(w)
    agent = workloads.make_agent(w, 0, DEV)
    agent.segments[2].anchor_len[1] = 10          # one unselected anchor in one pool
    ref_k, ref_v = agent.cache_k.clone(), agent.cache_v.clone()
    singles = []
    for j, seg in enumerate(agent.segments):
        p0 = w.seg_offset(j)
        singles.append(hotpath.align_segment(model, seg, ref_k[:, :, p0:p0 + w.seg_len], ref_v[:, :, p0:p0 + w.seg_len]))
    sc = hotpath.align_agent_batched(w, model, agent)
    torch.cuda.synchronize()
    for j in range(w.n_segments):
        assert torch.equal(sc.selected[j], singles[j].selected)
        assert torch.equal(sc.nearest[j], singles[j].nearest)
        assert float((sc.weights[j] - singles[j].weights).abs().max()) < 1e-6
    # same weights in -> bit-identical caches: rerun the batched align with the single-call weights
    jobs = []
    for j, seg in enumerate(agent.segments):
        p0 = w.seg_offset(j)
        jobs.append(dict(base_k=seg.base_k, base_v=seg.base_v, anchor_dk=seg.anchor_dk, anchor_dv=seg.anchor_dv,
                         anchor_len=seg.anchor_len, weights=singles[j].weights, delta_pos=seg.delta_pos,
                         anchor_delta_pos=seg.anchor_delta_pos, out_k=agent.cache_k[:, :, p0:p0 + w.seg_len],
                         out_v=agent.cache_v[:, :, p0:p0 + w.seg_len]))
    kv.kvcomm_align_kv_batch(model, jobs)
    torch.cuda.synchronize()
    assert torch.equal(agent.cache_k, ref_k) and torch.equal(agent.cache_v, ref_v)
    # and against the oracle for one of the segments
    seg = agent.segments[2]
    bk, anc = oracle_inputs(seg)
    ref = oracle.reuse_step(bk, to_np(seg.base_v), anc,
                            [to_np(a) if n >= w.seg_len else np.zeros(bk.shape[:2] + (0, bk.shape[3]))
                             for a, n in zip(seg.anchor_dk, seg.anchor_len)],
                            [to_np(a) if n >= w.seg_len else np.zeros(bk.shape[:2] + (0, bk.shape[3]))
                             for a, n in zip(seg.anchor_dv, seg.anchor_len)],
                            seg.delta_pos, w.rope_theta, anc_delta=seg.anchor_delta_pos)
    p0 = w.seg_offset(2)
    check_weights(sc.weights[2].cpu().numpy(), ref["w"].T)
    check_close(to_np(agent.cache_k[:, :, p0:p0 + w.seg_len]), ref["out_k"], w.dtype, "K^ batched")
    check_close(to_np(agent.cache_v[:, :, p0:p0 + w.seg_len]), ref["out_v"], w.dtype, "V^ batched")


def test_batched_mixed_lengths_and_prefix_segment_update():
    """Jobs of different lengths and pool sizes; a prefix-segment job (Eq. "pf_update") that uses the
    placeholder's per-segment weights with its own tensors."""
    # all pools are padded to one capacity (77 tokens): the anchors of a launch share one layout
    w = scaled(SMALL_F32, n_anchors=3, seg_len=40, anchor_lens=(77, 77, 77))
    say("batched mixed")
    model = hotpath.model_of(w)
    ph = workloads.make_segment(w, 0, 0, DEV)                                   # placeholder
    pf = workloads.make_segment(scaled(w, seg_len=23, seed=5), 0, 1, DEV)       # following prefix segment, other length
    other = workloads.make_segment(scaled(w, seg_len=77, n_anchors=6, seed=9, anchor_lens=(77,) * 6), 0, 2, DEV)
    outs = kv.kvcomm_anchor_weights_batch(model, [dict(seg_base_k=ph.base_k, anchor_base_k=ph.anchor_k),
                                                   dict(seg_base_k=other.base_k, anchor_base_k=other.anchor_k)],
                                          gran=kv.W_SEGMENT)
    w_ph, w_other = outs[0][0], outs[1][0]
    mk = lambda s: (torch.empty_like(s.base_k), torch.empty_like(s.base_v))
    o_ph, o_pf, o_other = mk(ph), mk(pf), mk(other)
    kv.kvcomm_align_kv_batch(model, [
        dict(base_k=ph.base_k, base_v=ph.base_v, anchor_dk=ph.anchor_dk, anchor_dv=ph.anchor_dv, weights=w_ph,
             delta_pos=64, out_k=o_ph[0], out_v=o_ph[1]),
        dict(base_k=pf.base_k, base_v=pf.base_v, anchor_dk=pf.anchor_dk, anchor_dv=pf.anchor_dv, weights=w_ph,
             delta_pos=104, out_k=o_pf[0], out_v=o_pf[1]),
        dict(base_k=other.base_k, base_v=other.base_v, anchor_dk=other.anchor_dk, anchor_dv=other.anchor_dv,
             weights=w_other, delta_pos=0, out_k=o_other[0], out_v=o_other[1])], gran=kv.W_SEGMENT)
    torch.cuda.synchronize()
    f = to_np
    d_ph, s_ph = oracle.distances(f(ph.base_k), [f(a) for a in ph.anchor_k], oracle.GRAN_SEGMENT)
    wo_ph, _ = oracle.weights(d_ph, s_ph, 1.0)
    d_o, s_o = oracle.distances(f(other.base_k), [f(a) for a in other.anchor_k], oracle.GRAN_SEGMENT)
    wo_o, _ = oracle.weights(d_o, s_o, 1.0)
    check_weights(w_ph.cpu().numpy(), wo_ph.T)
    check_weights(w_other.cpu().numpy(), wo_o.T)
    for seg, out, wo, delta in ((ph, o_ph, wo_ph, 64), (pf, o_pf, wo_ph, 104), (other, o_other, wo_o, 0)):
        rk, rv = oracle.align(f(seg.base_k), f(seg.base_v), [f(a) for a in seg.anchor_dk], [f(a) for a in seg.anchor_dv],
                              wo, delta, w.rope_theta, gran=oracle.GRAN_SEGMENT)
        check_close(f(out[0]), rk, w.dtype, "K^")
        check_close(f(out[1]), rv, w.dtype, "V^")


# ------------------------------------------------------------------------- compressed deviations
def test_e4m3_hardware_decode_is_the_ocp_format():
    """All 256 codes through the kernel's unpacking (one anchor of weight 1 and scale 1, zero base, no
    rotation, fp32 output) against the oracle's decoder: pins the conversion instruction's format."""
    say("e4m3 decode")
    w = scaled(SMALL_F32, n_layers=1, n_kv_heads=1, n_q_heads=1, head_dim=64, seg_len=4, n_anchors=1)
    model = hotpath.model_of(w)
    codes = torch.arange(256, dtype=torch.uint8, device=DEV).reshape(1, 1, 4, 64)
    zero = torch.zeros((1, 1, 4, 64), dtype=torch.float32, device=DEV)
    ones = torch.ones((4, 1), dtype=torch.float32, device=DEV)
    ok, ov = torch.empty_like(zero), torch.empty_like(zero)
    kv.kvcomm_align_kv_q8(model, zero, zero, [codes], [codes], [1.0], [2.0], ones, 0, ok, ov)
    torch.cuda.synchronize()
    want = np.array([oracle.e4m3_decode(c) for c in range(256)])
    fin = ~np.isnan(want)
    assert np.array_equal(ok.cpu().numpy().reshape(-1)[fin], want[fin].astype(np.float32))
    assert np.array_equal(ov.cpu().numpy().reshape(-1)[fin], (2 * want[fin]).astype(np.float32))
    assert np.isnan(ok.cpu().numpy().reshape(-1)[~fin]).all()


@pytest.mark.parametrize("w", [SMALL_BF16, SMALL_F32, scaled(SMALL_BF16, name="bf16_d64", head_dim=64, n_q_heads=2)],
                         ids=lambda w: w.name)
def test_quantize_deltas_bit_exact(w):
    say(f"quantize {w.name}")
    model = hotpath.model_of(w)
    seg = workloads.make_segment(w, 0, 0, DEV)
    x = seg.anchor_dk[0].clone()
    x[0, 0, 0, :8] = torch.tensor([0.0, -0.0, 1e-9, 0.44, 10.0, -10.0, 2.0 ** -16, -2.0 ** -19], dtype=w.dtype)
    # ties of the E4M3 grid that the model dtype can hold exactly (scale 2^-10): 1.0625, 1.1875, 2^-10, 3 * 2^-10
    x[0, 0, 1, :4] = torch.tensor([1.0625, 1.1875, 2.0 ** -10, 3 * 2.0 ** -10], dtype=w.dtype) * 2.0 ** -10
    for scale in (2.0 ** -10, 2.0 ** -7):
        q = kv.kvcomm_quantize_deltas(model, x, scale)
        torch.cuda.synchronize()
        want = oracle.quantize(to_np(x), scale)
        got = q.cpu().numpy()
        # +0 and -0 are both zero: compare values, and codes wherever the value is not zero
        same = got == want
        zero_both = ((got & 0x7f) == 0) & ((want & 0x7f) == 0)
        assert np.all(same | zero_both)
    with pytest.raises(kv.KVCommError):
        kv.kvcomm_quantize_deltas(model, x, 0.003)           # not a power of two


@pytest.mark.parametrize("w", [SMALL_BF16, SMALL_F32], ids=lambda w: w.name)
@pytest.mark.parametrize("gran", [kv.W_TOKEN, kv.W_LAYER_HEAD_TOKEN, kv.W_SEGMENT])
def test_align_with_compressed_deviations(w, gran):
    say(f"align q8 {w.name} gran={gran}")
    w = scaled(w, anchor_delta_choices=(16, 64, 100), n_anchors=6)
    model = hotpath.model_of(w)
    seg = workloads.make_segment(w, 0, 0, DEV)
    scales_k = [2.0 ** -10, 2.0 ** -9, 2.0 ** -10, 2.0 ** -11, 2.0 ** -10, 2.0 ** -8]
    scales_v = [2.0 ** -10] * 6
    qk = [kv.kvcomm_quantize_deltas(model, a, s) for a, s in zip(seg.anchor_dk, scales_k)]
    qv = [kv.kvcomm_quantize_deltas(model, a, s) for a, s in zip(seg.anchor_dv, scales_v)]
    wts, _, _ = kv.kvcomm_anchor_weights(model, seg.base_k, seg.anchor_k, seg.anchor_len, 1.0, gran)
    ok, ov = torch.empty_like(seg.base_k), torch.empty_like(seg.base_v)
    kv.kvcomm_align_kv_q8(model, seg.base_k, seg.base_v, qk, qv, scales_k, scales_v, wts, seg.delta_pos, ok, ov,
                          seg.anchor_len, seg.anchor_delta_pos, gran)
    torch.cuda.synchronize()
    # the oracle sees what is stored: the decoded codes (its own quantiser of the same inputs gives the same codes)
    dk = [oracle.dequantize(oracle.quantize(to_np(a), s), s) for a, s in zip(seg.anchor_dk, scales_k)]
    dv = [oracle.dequantize(oracle.quantize(to_np(a), s), s) for a, s in zip(seg.anchor_dv, scales_v)]
    bk, anc = oracle_inputs(seg)
    dist, sel = oracle.distances(bk, anc, gran)
    wo, _ = oracle.weights(dist, sel, 1.0)
    rk, rv = oracle.align(bk, to_np(seg.base_v), dk, dv, wo, seg.delta_pos, w.rope_theta,
                          anc_delta=seg.anchor_delta_pos, gran=gran)
    check_close(to_np(ok), rk, w.dtype, "K^ q8")
    check_close(to_np(ov), rv, w.dtype, "V^ q8")
    # and the compression error itself stays within the format's bound: |dec - x| <= 2^-4 |x| (+ tiny absolute floor)
    x = to_np(seg.anchor_dk[5])
    assert np.all(np.abs(dk[5] - x) <= np.abs(x) * 2.0 ** -4 + scales_k[5] * 2.0 ** -10)


def test_compressed_align_full_size_rate_inputs():
    """Config-2 segment at full size through the compressed path, oracle on sampled tokens."""
    w = scaled(workloads.LLAMA8B_5AGENTS, n_agents=1, n_segments=1)
    say("align q8 full size")
    model = hotpath.model_of(w)
    seg = workloads.make_segment(w, 0, 0, DEV)
    s = 2.0 ** -10
    qk = [kv.kvcomm_quantize_deltas(model, a, s) for a in seg.anchor_dk]
    qv = [kv.kvcomm_quantize_deltas(model, a, s) for a in seg.anchor_dv]
    wts, _, _ = kv.kvcomm_anchor_weights(model, seg.base_k, seg.anchor_k, seg.anchor_len)
    ok, ov = torch.empty_like(seg.base_k), torch.empty_like(seg.base_v)
    kv.kvcomm_align_kv_q8(model, seg.base_k, seg.base_v, qk, qv, [s] * 8, [s] * 8, wts, seg.delta_pos, ok, ov)
    torch.cuda.synchronize()
    tokens = [0, 31, 32, 255, 300, 511]
    idx = torch.as_tensor(tokens, device=DEV)
    f = lambda t: to_np(t[:, :, idx])
    dk = [oracle.dequantize(oracle.quantize(f(a), s), s) for a in seg.anchor_dk]
    dv = [oracle.dequantize(oracle.quantize(f(a), s), s) for a in seg.anchor_dv]
    dist, sel = oracle.distances(f(seg.base_k), [f(a) for a in seg.anchor_k])
    wo, _ = oracle.weights(dist, sel, 1.0)
    rk, rv = oracle.align(f(seg.base_k), f(seg.base_v), dk, dv, wo, seg.delta_pos, w.rope_theta)
    check_close(f(ok), rk, w.dtype, "K^ q8 full")
    check_close(f(ov), rv, w.dtype, "V^ q8 full")


def test_quantize_nan_infinity_and_saturation():
    """NaN -> the format's NaN code 0x7f; +-infinity, +-448 * scale and anything beyond saturate at +-448
    (codes 0x7e / 0xfe); the largest value that still rounds below the bound keeps its own code."""
    say("quantize NaN / inf / saturation")
    for w in (SMALL_F32, SMALL_BF16):
        model = hotpath.model_of(w)
        scale = 2.0 ** -10
        x = torch.zeros((w.n_layers, w.n_kv_heads, 9, w.head_dim), dtype=w.dtype, device=DEV)
        special = [float("nan"), -float("nan"), float("inf"), -float("inf"), 448.0 * scale, -448.0 * scale,
                   480.0 * scale, -1e30, 416.0 * scale, 432.0 * scale, 1e-30, 464.0 * scale]
        x[0, 0, 3, :len(special)] = torch.tensor(special, dtype=torch.float32).to(w.dtype)
        x[-1, -1, 8, -len(special):] = torch.tensor(special, dtype=torch.float32).to(w.dtype)
        q = kv.kvcomm_quantize_deltas(model, x, scale)
        torch.cuda.synchronize()
        got, want = q.cpu().numpy(), oracle.quantize(to_np(x), scale)
        assert np.array_equal(got[0, 0, 3, :len(special)], want[0, 0, 3, :len(special)]), (got[0, 0, 3, :12], want[0, 0, 3, :12])
        assert np.array_equal(got[-1, -1, 8, -len(special):], want[-1, -1, 8, -len(special):])
        assert list(got[0, 0, 3, :8]) == [0x7f, 0x7f, 0x7e, 0xfe, 0x7e, 0xfe, 0x7e, 0xfe]
        zero_both = ((got & 0x7f) == 0) & ((want & 0x7f) == 0)
        assert np.all((got == want) | zero_both)


def test_compressed_batch_equals_single_calls_and_oracle():
    """kvcomm_align_kv_q8_batch over segments of mixed length, pool size and recording offsets, written into
    one agent cache: bit-identical to per-segment kvcomm_align_kv_q8 calls, and equal to the oracle's update
    on the stored (decoded) values."""
    say("align q8 batch")
    base = scaled(SMALL_BF16, n_layers=3, n_kv_heads=2, n_q_heads=4, anchor_delta_choices=(16, 64, 100))
    shapes = [(70, 5), (203, 3), (33, 8)]
    model = hotpath.model_of(base)
    total = sum(s for s, _ in shapes)
    cache_k = torch.zeros((base.n_layers, base.n_kv_heads, 16 + total, base.head_dim), dtype=base.dtype, device=DEV)
    cache_v = torch.zeros_like(cache_k)
    ref_k, ref_v = torch.zeros_like(cache_k), torch.zeros_like(cache_k)
    jobs, p0, per_seg = [], 16, []
    for j, (S, A) in enumerate(shapes):
        w = scaled(base, seg_len=S, n_anchors=A, anchor_lens=(203,) * A, seed=40 + j)   # one capacity: one layout
        seg = workloads.make_segment(w, 0, j, DEV)
        sk = [2.0 ** -(9 + (a % 3)) for a in range(A)]
        sv = [2.0 ** -10] * A
        qk = [kv.kvcomm_quantize_deltas(model, a, s) for a, s in zip(seg.anchor_dk, sk)]
        qv = [kv.kvcomm_quantize_deltas(model, a, s) for a, s in zip(seg.anchor_dv, sv)]
        wts, _, _ = kv.kvcomm_anchor_weights(model, seg.base_k, seg.anchor_k, seg.anchor_len)
        jobs.append(dict(base_k=seg.base_k, base_v=seg.base_v, anchor_dk8=qk, anchor_dv8=qv, scale_k=sk, scale_v=sv,
                         weights=wts, delta_pos=seg.delta_pos, anchor_delta_pos=seg.anchor_delta_pos,
                         anchor_len=seg.anchor_len, out_k=cache_k[:, :, p0:p0 + S], out_v=cache_v[:, :, p0:p0 + S]))
        kv.kvcomm_align_kv_q8(model, seg.base_k, seg.base_v, qk, qv, sk, sv, wts, seg.delta_pos,
                              ref_k[:, :, p0:p0 + S], ref_v[:, :, p0:p0 + S], seg.anchor_len, seg.anchor_delta_pos)
        per_seg.append((w, seg, sk, sv, p0))
        p0 += S
    kv.kvcomm_align_kv_q8_batch(model, jobs)
    torch.cuda.synchronize()
    assert torch.equal(cache_k, ref_k) and torch.equal(cache_v, ref_v)
    for w, seg, sk, sv, p0 in per_seg:
        S = w.seg_len
        dk = [oracle.dequantize(oracle.quantize(to_np(a), s), s) for a, s in zip(seg.anchor_dk, sk)]
        dv = [oracle.dequantize(oracle.quantize(to_np(a), s), s) for a, s in zip(seg.anchor_dv, sv)]
        bk, anc = oracle_inputs(seg)
        dist, sel = oracle.distances(bk, anc, 0)
        wo, _ = oracle.weights(dist, sel, 1.0)
        rk, rv = oracle.align(bk, to_np(seg.base_v), dk, dv, wo, seg.delta_pos, w.rope_theta, anc_delta=seg.anchor_delta_pos)
        check_close(to_np(cache_k[:, :, p0:p0 + S]), rk, w.dtype, "K^ q8 batch")
        check_close(to_np(cache_v[:, :, p0:p0 + S]), rv, w.dtype, "V^ q8 batch")
    assert float(cache_k[:, :, :16].abs().max()) == 0.0      # rows outside the segments' slots untouched
    # a job whose output overlaps another job's is refused
    jobs[1]["out_k"] = jobs[0]["out_k"]
    with pytest.raises(kv.KVCommError):
        kv.kvcomm_align_kv_q8_batch(model, jobs)


def test_align_refuses_partial_overlap_on_device_tensors():
    """The aliasing rule of the boundary on real tensors: in place is fine, a shifted view of the base is not."""
    say("align aliasing")
    w = SMALL_BF16
    model = hotpath.model_of(w)
    seg = workloads.make_segment(w, 0, 0, DEV)
    wts, _, _ = kv.kvcomm_anchor_weights(model, seg.base_k, seg.anchor_k, seg.anchor_len)
    big_k = torch.zeros((w.n_layers, w.n_kv_heads, w.seg_len + 8, w.head_dim), dtype=w.dtype, device=DEV)
    big_v = torch.zeros_like(big_k)
    big_k[:, :, :w.seg_len], big_v[:, :, :w.seg_len] = seg.base_k, seg.base_v
    args = (seg.anchor_dk, seg.anchor_dv, wts, seg.delta_pos)
    want_k, want_v = torch.empty_like(seg.base_k), torch.empty_like(seg.base_v)
    kv.kvcomm_align_kv(model, seg.base_k, seg.base_v, *args, want_k, want_v)
    bk, bv = big_k[:, :, :w.seg_len], big_v[:, :, :w.seg_len]
    with pytest.raises(kv.KVCommError) as e:
        kv.kvcomm_align_kv(model, bk, bv, *args, big_k[:, :, 8:], bv)        # out_k = base_k shifted by 8 tokens
    assert e.value.status == -1
    with pytest.raises(kv.KVCommError):
        kv.kvcomm_align_kv(model, bk, bv, *args, bv, bk)                     # outputs swapped onto the other base
    kv.kvcomm_align_kv(model, bk, bv, *args, bk, bv)                         # in place
    torch.cuda.synchronize()
    assert torch.equal(bk, want_k) and torch.equal(bv, want_v)


def test_whole_step_under_hip_graph_capture_and_replay():
    """The library only enqueues kernels (no allocation, copy or memset), so a caller can record a whole
    reuse step of an agent into a HIP graph.  Every replay, with eager work and synchronisations between
    the replays and inputs changed in place, must reproduce the eager result bit for bit."""
    w = scaled(workloads.LLAMA8B_5AGENTS, name="graph", n_layers=4, n_kv_heads=2, n_q_heads=8, n_agents=1,
               prefix_len=64, seg_len=200, n_segments=3, n_anchors=6, tq=40, anchor_delta_choices=(64, 264))
    say("graph capture")
    model = hotpath.model_of(w)
    agent = workloads.make_agent(w, 0, DEV)
    sc = hotpath.AgentScratch(model, [w.seg_len] * w.n_segments, [w.n_anchors] * w.n_segments, kv.W_TOKEN, DEV)
    out = torch.empty_like(agent.q)
    lse = torch.empty(agent.q.shape[:3], dtype=torch.float32, device=DEV)

    def step():
        hotpath.align_agent_batched(w, model, agent, kv.W_TOKEN, sc)
        kv.kvcomm_suffix_attn(model, agent.q, agent.cache_k, agent.cache_v, w.n_ctx, out=out, lse_out=lse)

    def eager_reference():
        step()
        torch.cuda.synchronize()
        return agent.cache_k.clone(), agent.cache_v.clone(), out.clone(), lse.clone(), [x.clone() for x in sc.weights]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    torch.cuda.synchronize()

    g = torch.Generator(device=DEV)
    g.manual_seed(7)
    for replay in range(3):
        # new inputs in the same buffers: the graph holds addresses, not values
        seg = agent.segments[replay % w.n_segments]
        seg.base_k.copy_(torch.randn(seg.base_k.shape, generator=g, device=DEV).to(seg.base_k.dtype))
        agent.q.copy_(torch.randn(agent.q.shape, generator=g, device=DEV).to(agent.q.dtype))
        want = eager_reference()
        for t in (agent.cache_k[:, :, w.prefix_len:w.n_ctx], agent.cache_v[:, :, w.prefix_len:w.n_ctx], out, lse):
            t.zero_()                            # eager work between the replays; stale results cannot pass
        for x in sc.weights:
            x.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (agent.cache_k, agent.cache_v, out, lse, sc.weights)
        assert torch.equal(got[0], want[0]) and torch.equal(got[1], want[1]), f"replay {replay}: caches differ"
        assert torch.equal(got[2], want[2]) and torch.equal(got[3], want[3]), f"replay {replay}: attention differs"
        for a, b in zip(got[4], want[4]):
            assert torch.equal(a, b), f"replay {replay}: weights differ"
    # and the last replay against the oracle, end to end, on one (layer, head) sample of the attention output
    q, k, v = (to_np(t) for t in (agent.q, agent.cache_k, agent.cache_v))
    check_close(to_np(out[:1]), oracle.suffix_attn(q[:1], k[:1], v[:1], w.n_ctx), w.dtype, "graph replay attention")


def test_batched_agent_is_cut_into_launches_by_segment_and_anchor_limits():
    """Eleven segments (more than one launch holds) and, separately, pools whose anchors add up to more
    than one launch holds: the helper cuts the agent into several launches; result as per-segment calls."""
    for name, n_segments, n_anchors in (("many segments", 11, 3), ("many anchors", 3, 30)):
        w = scaled(workloads.LLAMA8B_5AGENTS, name="cut", n_layers=2, n_kv_heads=2, n_q_heads=4, n_agents=1,
                   prefix_len=8, seg_len=40, n_segments=n_segments, n_anchors=n_anchors, tq=4)
        say(f"batched agent, {name}")
        model = hotpath.model_of(w)
        agent = workloads.make_agent(w, 0, DEV)
        ref_k, ref_v = agent.cache_k.clone(), agent.cache_v.clone()
        singles = []
        for j, seg in enumerate(agent.segments):
            p0 = w.seg_offset(j)
            singles.append(hotpath.align_segment(model, seg, ref_k[:, :, p0:p0 + w.seg_len], ref_v[:, :, p0:p0 + w.seg_len]))
        sc = hotpath.align_agent_batched(w, model, agent)
        torch.cuda.synchronize()
        for j in range(w.n_segments):
            assert torch.equal(sc.nearest[j], singles[j].nearest)
            assert float((sc.weights[j] - singles[j].weights).abs().max()) < 1e-6
        err_k = float((agent.cache_k.float() - ref_k.float()).abs().max())
        err_v = float((agent.cache_v.float() - ref_v.float()).abs().max())
        assert err_k < 2e-2 and err_v < 2e-2, (err_k, err_v)   # same path up to the last bit of the weights
