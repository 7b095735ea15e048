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
