"""GPU parity on seeded random shapes: the whole hot path (anchor weights, align, suffix attention; single-segment
and batched calls alike) against the float64 oracle, over head dimensions, dtypes, head groupings, ragged segment,
prefix and suffix lengths, shorter and longer anchors and per-anchor recording offsets.  Same comparison rules
as the other parity tests."""
import random

import numpy as np
import pytest
import torch

import oracle
import paper_2510_12872_amd as kv
from paper_2510_12872_amd import hotpath, workloads

from parity import check_close, check_weights, oracle_segment, to_np

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_random_shapes_whole_hot_path(seed):
    rng = random.Random(seed)
    for case in range(40):
        D = rng.choice([64, 128, 128, 128, 256])
        dtype = rng.choice([torch.bfloat16, torch.bfloat16, torch.float32])
        Hkv = rng.choice([1, 2, 4])
        G = rng.choice([1, 2, 4, 8])
        S = rng.choice([1, 2, 7, 16, 31, 32, 33, 64, 100, 129, 255])
        A = rng.choice([1, 2, 3, 5, 8, 12, 17])
        nseg = rng.choice([1, 2, 3])
        lens = tuple(rng.choice([S, S, S, S + rng.randint(1, 20), max(1, S - rng.randint(1, 5))]) for _ in range(A))
        w = workloads.Workload(name=f"rand{seed}_{case}", n_layers=rng.choice([1, 2, 3]), n_kv_heads=Hkv, n_q_heads=Hkv * G,
                               head_dim=D, dtype=dtype, rope_theta=rng.choice([1e4, 5e5]), n_agents=1,
                               prefix_len=rng.choice([0, 1, 5, 63, 64, 200]), seg_len=S, n_segments=nseg, n_anchors=A,
                               tq=rng.choice([1, 2, 17, 32, 63, 64, 65, 130, 257]), sigma_delta=0.05,
                               temperature=rng.choice([1.0, 0.5, 2.0]), seed=1000 * seed + case,
                               anchor_delta_choices=rng.choice([None, (16, 64, 100), (0, 2048)]), anchor_lens=lens)
        batched = rng.random() < 0.5
        print(f"seed {seed} case {case}: D{D} {str(dtype)[6:]} Hkv{Hkv} G{G} L{w.n_layers} S{S} A{A} nseg{nseg} "
              f"prefix{w.prefix_len} tq{w.tq} lens{lens} batched={batched}", flush=True)
        model = hotpath.model_of(w)
        agent = workloads.make_agent(w, 0, "cuda")
        ck, cv = to_np(agent.cache_k), to_np(agent.cache_v)
        refs = []
        for j, seg in enumerate(agent.segments):
            p0 = w.seg_offset(j)
            ref = oracle_segment(w, seg)
            refs.append(ref)
            ck[:, :, p0:p0 + S], cv[:, :, p0:p0 + S] = ref["out_k"], ref["out_v"]
        if batched:
            sc = hotpath.align_agent_batched(w, model, agent)
            got = [(sc.weights[j], sc.nearest[j], sc.selected[j]) for j in range(nseg)]
        else:
            got = []
            for j, seg in enumerate(agent.segments):
                p0 = w.seg_offset(j)
                s1 = hotpath.align_segment(model, seg, agent.cache_k[:, :, p0:p0 + S], agent.cache_v[:, :, p0:p0 + S],
                                           w.temperature)
                got.append((s1.weights, s1.nearest, s1.selected))
        out, lse = kv.kvcomm_suffix_attn(model, agent.q, agent.cache_k, agent.cache_v, w.n_ctx, want_lse=True)
        torch.cuda.synchronize()
        for j, ref in enumerate(refs):
            p0 = w.seg_offset(j)
            wts, nearest, selected = got[j]
            assert np.array_equal(selected.cpu().numpy(), ref["selected"]), "selected"
            assert np.array_equal(nearest.cpu().numpy(), ref["nearest"]), "nearest"
            check_weights(wts.cpu().numpy(), ref["w"].T)
            check_close(to_np(agent.cache_k[:, :, p0:p0 + S]), ref["out_k"], dtype, "K^")
            check_close(to_np(agent.cache_v[:, :, p0:p0 + S]), ref["out_v"], dtype, "V^")
        want, want_lse = oracle.suffix_attn(to_np(agent.q), ck, cv, w.n_ctx, want_lse=True)
        check_close(to_np(out), want, dtype, "O")
        assert float(np.max(np.abs(lse.cpu().numpy() - want_lse))) < (2e-2 if dtype == torch.bfloat16 else 1e-4), "lse"


@pytest.mark.parametrize("seed", [10, 11])
def test_random_shapes_granularities_and_rules(seed):
    """Anchor weights for every granularity and weighting rule on seeded random shapes, and the aligned cache that
    the non-default granularities produce."""
    rng = random.Random(seed)
    for case in range(30):
        D = rng.choice([64, 128, 128, 256])
        dtype = rng.choice([torch.bfloat16, torch.float32])
        S = rng.choice([1, 3, 16, 31, 33, 64, 97, 130])
        A = rng.choice([1, 2, 4, 7, 9, 16, 20])
        lens = tuple(rng.choice([S, S, S, S + rng.randint(1, 9), max(1, S - 1)]) for _ in range(A))
        gran = rng.choice([kv.W_TOKEN, kv.W_LAYER_HEAD_TOKEN, kv.W_SEGMENT])
        tau = rng.choice([1.0, 0.3, 3.0])
        w = workloads.Workload(name=f"rules{seed}_{case}", n_layers=rng.choice([1, 2, 5]), n_kv_heads=rng.choice([1, 2, 3]),
                               n_q_heads=6, head_dim=D, dtype=dtype, rope_theta=5e5, n_agents=1, prefix_len=0, seg_len=S,
                               n_segments=1, n_anchors=A, tq=0, sigma_delta=0.05, temperature=tau, seed=2000 * seed + case,
                               anchor_delta_choices=rng.choice([None, (8, 40)]), anchor_lens=lens)
        print(f"seed {seed} case {case}: D{D} {str(dtype)[6:]} L{w.n_layers} H{w.n_kv_heads} S{S} A{A} gran{gran} tau{tau} "
              f"lens{lens}", flush=True)
        model = hotpath.model_of(w)
        seg = workloads.make_segment(w, 0, 0, "cuda")
        bk = to_np(seg.base_k)
        anc = [to_np(a) if n >= S else np.zeros(bk.shape[:2] + (0, bk.shape[3])) for a, n in zip(seg.anchor_k, seg.anchor_len)]
        dist, sel = oracle.distances(bk, anc, gran)
        w_l2, n_l2, s_l2 = kv.kvcomm_anchor_weights_rule(model, kv.RULE_L2_SOFTMAX, seg.base_k, seg.anchor_k, seg.anchor_len,
                                                         tau, gran)
        w_nn, n_nn, _ = kv.kvcomm_anchor_weights_rule(model, kv.RULE_NEAREST, seg.base_k, seg.anchor_k, seg.anchor_len, tau,
                                                      gran)
        w_cs, n_cs, s_cs = kv.kvcomm_anchor_weights_rule(model, kv.RULE_COSINE_SOFTMAX, seg.base_k, seg.anchor_k,
                                                         seg.anchor_len, tau, gran)
        ok, ov = torch.empty_like(seg.base_k), torch.empty_like(seg.base_v)
        kv.kvcomm_align_kv(model, seg.base_k, seg.base_v, seg.anchor_dk, seg.anchor_dv, w_l2, seg.delta_pos, ok, ov,
                           seg.anchor_len, seg.anchor_delta_pos, gran)
        torch.cuda.synchronize()
        want, near = oracle.weights(dist, sel, tau)
        assert np.array_equal(s_l2.cpu().numpy(), sel)
        assert np.array_equal(n_l2.cpu().numpy(), near)
        check_weights(w_l2.cpu().numpy(), want.T)
        want_nn, near_nn = oracle.weights_nearest(dist, sel)
        assert np.array_equal(n_nn.cpu().numpy(), near_nn)
        assert np.array_equal(w_nn.cpu().numpy(), want_nn.T.astype(np.float32))
        sim, sel_c = oracle.cosine(bk, anc, gran)
        want_cs, best = oracle.weights_from_sim(sim, sel_c, tau)
        assert np.array_equal(s_cs.cpu().numpy(), sel_c)
        assert np.array_equal(n_cs.cpu().numpy(), best)
        check_weights(w_cs.cpu().numpy(), want_cs.T, "cosine weights")
        ref = oracle_segment(w, seg, gran=gran)
        check_close(to_np(ok), ref["out_k"], dtype, "K^")
        check_close(to_np(ov), ref["out_v"], dtype, "V^")
