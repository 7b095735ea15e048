#!/usr/bin/env python3
"""Benchmark of the KVComm reuse hot path on one MI355X.

A step is one pass of the whole hot path over the Llama-3-8B-shaped five-agent workload
(workloads.LLAMA8B_5AGENTS): for each of the 5 agents, 4 peer segments of 512 tokens are
matched against their 8-anchor pools (kvcomm_anchor_weights_batch, one launch per stage for the
four segments), re-positioned and offset-corrected into the agent's cache (kvcomm_align_kv_batch,
one launch), and the agent's 512 suffix queries then attend over the 3072-token cache
(kvcomm_suffix_attn).  All inputs are synthetic, seeded and
resident in HBM before the timed region starts.

Prints ONE JSON line.  `value` = aligned KV tokens per second of the whole step (alignment
and attention); per-kernel achieved rates and roofline fractions come from HIP events recorded
around every library call inside the same timed region.  The `cpu_baseline` object is the
float64 oracle timed on the host cores on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, GB/s
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, TFLOP/s
# HBM bytes per launch on this workload (read, written), from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# runs of this script, each scaled by the same counter's reading for a plain 1 GiB copy
# (profiles/bench_llama8b_5agents_hbm_traffic.md; tests/test_bench_constants.py holds the two together).
# Not measured live: counters need the profiler.
HBM_TRAFFIC_READ_WRITTEN = {"align_kv": (2416182477, 268435456),                           # align_kernel
                            "anchor_weights": (1208184422 + 8502272, 8390349 + 82022),     # dist_partial_kernel + finalize_kernel
                            "suffix_attn": (537208422, 136314880)}                         # attn_mfma_kernel
HBM_TRAFFIC_BYTES = {k: r + w for k, (r, w) in HBM_TRAFFIC_READ_WRITTEN.items()}
# Share of the kernel's cycles in which a SIMD's matrix pipe is busy (SQ_VALU_MFMA_BUSY_CYCLES per SIMD over
# GRBM_GUI_ACTIVE per XCD, profiles/suffix_attn_llama8b_5agents_mfma_counters.md); not measured live either.
SUFFIX_ATTN_MFMA_BUSY_FRAC = 0.599


def cpu_baseline(w):
    """Oracle (as it stands) over the WHOLE workload: every segment alignment and the suffix attention of every
    agent, all layers and heads, one agent's inputs on the host at a time (about half a minute for config 2)."""
    import torch

    import oracle
    from paper_2510_12872_amd import workloads

    f64 = lambda t: t.to(torch.float64).numpy()
    t_align = t_attn = 0.0
    for a in range(w.n_agents):
        for j in range(w.n_segments):
            seg = workloads.make_segment(w, a, j, "cpu")
            args = (f64(seg.base_k), f64(seg.base_v), [f64(x) for x in seg.anchor_k],
                    [f64(x) for x in seg.anchor_dk], [f64(x) for x in seg.anchor_dv])
            t0 = time.perf_counter()
            oracle.reuse_step(*args, seg.delta_pos, w.rope_theta, tau=w.temperature)
            t_align += time.perf_counter() - t0
            del seg, args
        # the attention reads a cache of the right shape; its segment slots hold generator values (the oracle's
        # own aligned rows would cost the same to attend over)
        ag = workloads.make_agent(workloads.scaled(w, n_segments=0, prefix_len=w.n_ctx), a, "cpu")
        q, k, v = f64(ag.q), f64(ag.cache_k), f64(ag.cache_v)
        t0 = time.perf_counter()
        oracle.suffix_attn(q, k, v, w.n_ctx)
        t_attn += time.perf_counter() - t0
        del ag, q, k, v
    try:
        affinity = len(os.sched_getaffinity(0))
    except AttributeError:
        affinity = None
    return {
        "value": w.aligned_tokens / (t_align + t_attn),
        "unit": "tokens/s",
        "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": (f"whole workload: {w.n_agents * w.n_segments} segment alignments ({t_align:.2f} s) + suffix attention "
                   f"of {w.n_agents} agents ({t_attn:.2f} s), all layers and heads"),
        "nproc": os.cpu_count(),
        "affinity_cores": affinity,
        "align_tokens_per_s": w.aligned_tokens / t_align,
        "attn_gflops": w.attn_flops() / t_attn / 1e9,
    }


def _stats(events):
    """Mean and median of HIP-event pairs, in ms."""
    ts = sorted(a.elapsed_time(b) for a, b in events)
    if not ts:
        return None, None
    mid = len(ts) // 2
    med = ts[mid] if len(ts) % 2 else 0.5 * (ts[mid - 1] + ts[mid])
    return sum(ts) / len(ts), med


def config_steps(torch, kv, dev, names=("pool_scaling_a4", "pool_scaling_a16", "pool_scaling_a32", "pool_scaling_a64",
                                        "long_context", "llama70b"), steps=4, warmup=2, streams=None):
    """Whole steps of the other baseline configurations, in the launch configuration of the timed region: per agent
    one batched weights call, one batched align call into the agent's cache and the suffix attention.  One agent's
    inputs are generated and every agent of the step runs on them (an agent's pass streams several GB, far beyond
    the 256 MB last-level cache, so nothing is reused between passes); config 5's four agents would not fit
    288 GB otherwise.  Per-call HIP events inside the steps give the kernel rates."""
    from paper_2510_12872_amd import hotpath, workloads

    res = {}
    for name in names:
        w = workloads.WORKLOADS[name]
        model = hotpath.model_of(w)
        ag = workloads.make_agent(w, 0, dev)
        out = torch.empty_like(ag.q) if w.tq else None
        sc = hotpath.AgentScratch(model, [w.seg_len] * w.n_segments, [w.n_anchors] * w.n_segments, kv.W_TOKEN, dev)
        wjobs = [dict(seg_base_k=seg.base_k, anchor_base_k=seg.anchor_k, anchor_len=seg.anchor_len,
                      weights_out=sc.weights[j], nearest_out=sc.nearest[j], selected_out=sc.selected[j])
                 for j, seg in enumerate(ag.segments)]
        ajobs = [dict(base_k=seg.base_k, base_v=seg.base_v, anchor_dk=seg.anchor_dk, anchor_dv=seg.anchor_dv,
                      anchor_len=seg.anchor_len, weights=sc.weights[j], delta_pos=seg.delta_pos,
                      anchor_delta_pos=seg.anchor_delta_pos,
                      out_k=ag.cache_k[:, :, w.seg_offset(j):w.seg_offset(j) + w.seg_len],
                      out_v=ag.cache_v[:, :, w.seg_offset(j):w.seg_offset(j) + w.seg_len])
                 for j, seg in enumerate(ag.segments)]
        ev = {"weights": [], "align": [], "attn": []}

        def timed(kind, record, fn):
            if not record:
                fn()
                return
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            ev[kind].append((e0, e1))

        def step(record):
            for _ in range(w.n_agents):
                timed("weights", record, lambda: kv.kvcomm_anchor_weights_batch(model, wjobs, w.temperature, kv.W_TOKEN,
                                                                                 workspace=sc.workspace))
                timed("align", record, lambda: kv.kvcomm_align_kv_batch(model, ajobs, kv.W_TOKEN))
                if w.tq:
                    timed("attn", record, lambda: kv.kvcomm_suffix_attn(model, ag.q, ag.cache_k, ag.cache_v, w.n_ctx, out=out))

        for _ in range(warmup):
            step(False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step(True)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / steps * 1e3
        one = workloads.scaled(w, n_agents=1)
        r = {"ms_per_step": ms, "aligned_tokens_per_step": w.aligned_tokens, "tokens_per_s": w.aligned_tokens / (ms * 1e-3),
             "shape": f"{w.n_agents} agent(s) x {w.n_segments} segment(s) of {w.seg_len}, A {w.n_anchors}, L {w.n_layers}, "
                      f"Hq {w.n_q_heads}, n_ctx {w.n_ctx}, tq {w.tq}"}
        for kind, nbytes, key in (("weights", one.distance_bytes(), "distance"), ("align", one.align_bytes(), "align")):
            mean, med = _stats(ev[kind])
            r[key] = {"avg_call_ms": mean, "median_call_ms": med, "GBps": nbytes / mean / 1e6,
                      "frac_of_hbm_peak": nbytes / mean / 1e6 / HBM_PEAK_GBS}
        if w.tq:
            mean, med = _stats(ev["attn"])
            r["attn"] = {"avg_call_ms": mean, "median_call_ms": med, "tflops": one.attn_flops() / mean / 1e9,
                         "frac_of_mfma_peak": one.attn_flops() / mean / 1e9 / MFMA_BF16_PEAK_TFLOPS}
        if w.tq and w.n_agents >= 2 and streams is not None:
            r["two_stream"] = two_stream_config_step(torch, kv, w, model, streams, [(ag, out, sc, wjobs, ajobs)], dev, ms)
        res[name] = r
        del ag, out, sc, wjobs, ajobs
        torch.cuda.empty_cache()
    return res


def two_stream_config_step(torch, kv, w, model, streams, sets, dev, sequential_ms, steps=3):
    """The same step of a configuration on two streams: weights + alignment of the next agent beside the attention
    of the current one, the attention confined to a share of the compute units (kvcomm_suffix_attn_confined).  Two
    sets of agent buffers alternate (the alignment overwrites the cache slots the attention reads).  The share is
    the best of a few candidates, each tried for one step."""
    from paper_2510_12872_amd import hotpath, workloads

    ag = workloads.make_agent(w, 1, dev)
    sc = hotpath.AgentScratch(model, [w.seg_len] * w.n_segments, [w.n_anchors] * w.n_segments, kv.W_TOKEN, dev)
    wjobs = [dict(seg_base_k=seg.base_k, anchor_base_k=seg.anchor_k, anchor_len=seg.anchor_len,
                  weights_out=sc.weights[j], nearest_out=sc.nearest[j], selected_out=sc.selected[j])
             for j, seg in enumerate(ag.segments)]
    ajobs = [dict(base_k=seg.base_k, base_v=seg.base_v, anchor_dk=seg.anchor_dk, anchor_dv=seg.anchor_dv,
                  anchor_len=seg.anchor_len, weights=sc.weights[j], delta_pos=seg.delta_pos,
                  anchor_delta_pos=seg.anchor_delta_pos,
                  out_k=ag.cache_k[:, :, w.seg_offset(j):w.seg_offset(j) + w.seg_len],
                  out_v=ag.cache_v[:, :, w.seg_offset(j):w.seg_offset(j) + w.seg_len])
             for j, seg in enumerate(ag.segments)]
    sets = sets + [(ag, torch.empty_like(ag.q), sc, wjobs, ajobs)]
    pipe = hotpath.TwoStreamPipeline(model, w.temperature, 160, align_stream=streams[0], attn_stream=streams[1])
    count = [0]

    def run(n_steps, blocks):
        pipe.attn_blocks = blocks
        pipe.fork()
        for _ in range(n_steps * w.n_agents):
            b = count[0] % 2
            count[0] += 1
            a, o, scr, wj, aj = sets[b]
            pipe.submit(b, wj, aj, scr.workspace, a.q, a.cache_k, a.cache_v, w.n_ctx, o)
        pipe.join()

    def timed(n_steps, blocks):
        torch.cuda.synchronize()
        t = time.perf_counter()
        run(n_steps, blocks)
        torch.cuda.synchronize()
        return (time.perf_counter() - t) / n_steps * 1e3

    run(1, 160)
    trials = {blocks: timed(1, blocks) for blocks in (160, 152, 144, 136)}
    best = min(trials, key=trials.get)
    ms = timed(steps, best)
    return {"ms_per_step": ms, "tokens_per_s": w.aligned_tokens / (ms * 1e-3), "attn_blocks": best,
            "gain_over_sequential": sequential_ms / ms - 1.0,
            "trial_ms_per_step": {str(k): v for k, v in trials.items()}}


def compressed_step(torch, kv, w, model, agents, outs, scratches, wjobs, steps=5, warmup=2, pipe=None):
    """The timed region's step with every anchor's deviations stored as E4M3 (one byte per element, scale 2^-10):
    batched weights, batched compressed update, attention."""
    scale = 2.0 ** -10
    qjobs = []
    for ag, sc in zip(agents, scratches):
        jobs = []
        for j, seg in enumerate(ag.segments):
            jobs.append(dict(base_k=seg.base_k, base_v=seg.base_v,
                             anchor_dk8=[kv.kvcomm_quantize_deltas(model, a, scale) for a in seg.anchor_dk],
                             anchor_dv8=[kv.kvcomm_quantize_deltas(model, a, scale) for a in seg.anchor_dv],
                             scale_k=[scale] * w.n_anchors, scale_v=[scale] * w.n_anchors, anchor_len=seg.anchor_len,
                             weights=sc.weights[j], delta_pos=seg.delta_pos, anchor_delta_pos=seg.anchor_delta_pos,
                             out_k=ag.cache_k[:, :, w.seg_offset(j):w.seg_offset(j) + w.seg_len],
                             out_v=ag.cache_v[:, :, w.seg_offset(j):w.seg_offset(j) + w.seg_len]))
        qjobs.append(jobs)
    ev = []

    def step(record):
        for ai, ag in enumerate(agents):
            kv.kvcomm_anchor_weights_batch(model, wjobs[ai], w.temperature, kv.W_TOKEN, workspace=scratches[ai].workspace)
            if record:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
            kv.kvcomm_align_kv_q8_batch(model, qjobs[ai], kv.W_TOKEN)
            if record:
                e1.record()
                ev.append((e0, e1))
            kv.kvcomm_suffix_attn(model, ag.q, ag.cache_k, ag.cache_v, w.n_ctx, out=outs[ai])

    for _ in range(warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step(True)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    mean, med = _stats(ev)
    rows = w.n_layers * w.n_kv_heads * w.n_segments * w.seg_len          # per launch: the segments of one agent
    nbytes = rows * w.head_dim * (4 * 2 + 2 * w.n_anchors)
    two_stream = None
    if pipe is not None:     # the same step on two streams (see hotpath.TwoStreamPipeline)
        def run(n):
            pipe.fork()
            for _ in range(n):
                for ai, ag in enumerate(agents):
                    pipe.submit(ai, wjobs[ai], qjobs[ai], scratches[ai].workspace, ag.q, ag.cache_k, ag.cache_v, w.n_ctx,
                                outs[ai], q8=True)
            pipe.join()
        run(3)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        run(10)
        torch.cuda.synchronize()
        two_stream = (time.perf_counter() - t1) / 10 * 1e3
    return {"ms_per_step": ms, "tokens_per_s": w.aligned_tokens / (ms * 1e-3),
            "two_stream_ms_per_step": two_stream,
            "align_kv_q8_batch": {"avg_call_ms": mean, "median_call_ms": med, "algorithmic_bytes": nbytes,
                                  "GBps": nbytes / mean / 1e6, "frac_of_hbm_peak": nbytes / mean / 1e6 / HBM_PEAK_GBS},
            "note": "deviations stored as E4M3 x 2^-10 (lossy); same weights and attention calls as the timed region"}


def mfma_calibration(torch, kv, w, model, dev):
    """Matrix-core rate of a library GEMM and of the attention kernel, on N(0,1) inputs and on zeros.

    The instruction streams are identical in both cases; only the operand bits differ, so the ratio shows what
    the chip's power management costs on the benchmark's value distribution."""
    from paper_2510_12872_amd import workloads

    def time_ms(fn, warm, n):
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    res = {}
    n = 8192
    g = torch.Generator(device=dev)
    g.manual_seed(0)
    a = torch.randn(n, n, generator=g, device=dev).to(torch.bfloat16)
    b = torch.randn(n, n, generator=g, device=dev).to(torch.bfloat16)
    for kind in ("normal", "zeros"):
        if kind == "zeros":
            a.zero_()
            b.zero_()
        ms = time_ms(lambda: torch.matmul(a, b.t()), 40, 60)
        res[f"library_gemm_8192_{kind}_tflops"] = 2.0 * n ** 3 / ms / 1e9
    del a, b
    ag = workloads.make_agent(w, 0, dev, with_segments=False)
    ag.cache_k[:, :, w.prefix_len:w.n_ctx] = torch.randn(ag.cache_k[:, :, w.prefix_len:w.n_ctx].shape, generator=g,
                                                         device=dev).to(ag.cache_k.dtype)
    ag.cache_v[:, :, w.prefix_len:w.n_ctx] = torch.randn(ag.cache_v[:, :, w.prefix_len:w.n_ctx].shape, generator=g,
                                                         device=dev).to(ag.cache_v.dtype)
    out = torch.empty_like(ag.q)
    flops = workloads.scaled(w, n_agents=1).attn_flops()
    # torch's own fused attention on the same tensors (grouped heads, every query sees the whole cache: a little
    # more work than the causal suffix attention) as a second reference for what this machine sustains
    import torch.nn.functional as F
    sdpa_flops = 4.0 * w.head_dim * w.n_q_heads * w.n_layers * w.tq * (w.n_ctx + w.tq)
    try:
        ms = time_ms(lambda: F.scaled_dot_product_attention(ag.q, ag.cache_k, ag.cache_v, enable_gqa=True), 20, 30)
        res["torch_sdpa_full_mask_normal_tflops"] = sdpa_flops / ms / 1e9
    except Exception as exc:  # an older torch without grouped heads: the reference is optional
        res["torch_sdpa_full_mask_normal_tflops"] = f"unavailable ({type(exc).__name__})"
    for kind in ("normal", "zeros"):
        if kind == "zeros":
            ag.q.zero_()
            ag.cache_k.zero_()
            ag.cache_v.zero_()
        ms = time_ms(lambda: kv.kvcomm_suffix_attn(model, ag.q, ag.cache_k, ag.cache_v, w.n_ctx, out=out), 80, 60)
        res[f"suffix_attn_{kind}_tflops"] = flops / ms / 1e9
    return res


def next_rows(torch, kv, w, model, dev):
    """Each entry point beyond the reuse step proper, timed alone on one 512-token segment of the workload:
    30 launches over three rotating input sets (nothing stays in the last-level cache), HIP events."""
    from paper_2510_12872_amd import workloads

    segs = [workloads.make_segment(w, 0, j, dev) for j in range(3)]
    A, S = w.n_anchors, w.seg_len
    rows = w.n_layers * w.n_kv_heads * S
    rb = w.head_dim * 2                                           # bytes per bf16 row
    scale = 2.0 ** -10
    outs = [(torch.empty_like(sg.base_k), torch.empty_like(sg.base_v)) for sg in segs]
    out2 = [(torch.empty_like(sg.base_k), torch.empty_like(sg.base_v)) for sg in segs]
    q8 = [([kv.kvcomm_quantize_deltas(model, a, scale) for a in sg.anchor_dk],
           [kv.kvcomm_quantize_deltas(model, a, scale) for a in sg.anchor_dv]) for sg in segs]
    n_slots = kv.kvcomm_weight_slots(model, S, kv.W_TOKEN)
    wts = torch.empty((n_slots, A), dtype=torch.float32, device=dev)
    nearest = torch.empty((n_slots,), dtype=torch.int32, device=dev)
    selected = torch.empty((A,), dtype=torch.int32, device=dev)
    ws = torch.empty((max(kv.kvcomm_anchor_weights_rule_workspace(model, S, A, kv.W_TOKEN, kv.RULE_COSINE_SOFTMAX),
                          kv.kvcomm_anchor_weights_rule_workspace(model, S, A, kv.W_TOKEN, kv.RULE_NEAREST), 256),),
                     dtype=torch.uint8, device=dev)
    pws = torch.empty((max(kv.kvcomm_anchor_predict_workspace(n_slots), 256),), dtype=torch.uint8, device=dev)
    pres = torch.empty((2,), dtype=torch.float32, device=dev)

    def rule(r):
        return lambda i: kv.kvcomm_anchor_weights_rule(model, r, segs[i % 3].base_k, segs[i % 3].anchor_k,
                                                       segs[i % 3].anchor_len, w.temperature, kv.W_TOKEN, wts, nearest,
                                                       selected, ws)

    def capture(i):
        sg = segs[i % 3]                                           # the next segment's base cache stands in for a real one
        o = segs[(i + 1) % 3]
        kv.kvcomm_capture_offsets(model, sg.base_k, sg.base_v, o.base_k, o.base_v, sg.delta_pos, outs[i % 3][0], outs[i % 3][1])

    def quantize(i):
        kv.kvcomm_quantize_deltas(model, segs[i % 3].anchor_dk[i % A], scale, q8[i % 3][0][i % A])

    def align_q8(i):
        sg, (qk, qv), o = segs[i % 3], q8[i % 3], out2[i % 3]
        kv.kvcomm_align_kv_q8(model, sg.base_k, sg.base_v, qk, qv, [scale] * A, [scale] * A, wts, sg.delta_pos, o[0], o[1],
                              sg.anchor_len, sg.anchor_delta_pos)

    def predict(i):
        kv.kvcomm_anchor_predict(wts, segs[0].anchor_len, S, 0.3, result_out=pres, workspace=pws)

    # the per-(layer, head, token) reading of the distance: one softmax per row instead of per token
    n_lh = kv.kvcomm_weight_slots(model, S, kv.W_LAYER_HEAD_TOKEN)
    wts_lh = torch.empty((n_lh, A), dtype=torch.float32, device=dev)
    near_lh = torch.empty((n_lh,), dtype=torch.int32, device=dev)
    ws_lh = torch.empty((max(kv.kvcomm_anchor_weights_workspace(model, S, A, kv.W_LAYER_HEAD_TOKEN), 256),),
                        dtype=torch.uint8, device=dev)

    def weights_lh(i):
        sg = segs[i % 3]
        kv.kvcomm_anchor_weights(model, sg.base_k, sg.anchor_k, sg.anchor_len, w.temperature, kv.W_LAYER_HEAD_TOKEN,
                                 wts_lh, near_lh, selected, ws_lh)

    def align_lh(i):
        sg, o = segs[i % 3], out2[i % 3]
        kv.kvcomm_align_kv(model, sg.base_k, sg.base_v, sg.anchor_dk, sg.anchor_dv, wts_lh, sg.delta_pos, o[0], o[1],
                           sg.anchor_len, sg.anchor_delta_pos, kv.W_LAYER_HEAD_TOKEN)

    cases = (("anchor_weights_rule nearest", rule(kv.RULE_NEAREST), rows * rb * (A + 1)),
             ("anchor_weights_rule cosine", rule(kv.RULE_COSINE_SOFTMAX), rows * rb * (A + 1)),
             ("capture_offsets", capture, rows * rb * 6),
             ("quantize_deltas", quantize, rows * w.head_dim * 3),
             ("align_kv_q8", align_q8, rows * w.head_dim * (4 * 2 + 2 * A)),
             ("anchor_predict", predict, n_slots * A * 4),
             ("anchor_weights per (layer, head, token)", weights_lh, rows * rb * (A + 1)),
             ("align_kv per (layer, head, token)", align_lh, rows * rb * 2 * (A + 2)))
    res = {}
    for label, fn, nbytes in cases:
        for i in range(6):
            fn(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(30):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 30
        res[label] = {"avg_call_us": ms * 1e3, "algorithmic_bytes": nbytes, "achieved_GBps": nbytes / ms / 1e6,
                      "frac_of_hbm_peak": nbytes / ms / 1e6 / HBM_PEAK_GBS}
    return res


def per_config(torch, kv, dev):
    """Every baseline configuration's kernels timed alone: one segment (anchor weights, then align into
    contiguous outputs) over rotating input sets, and the suffix attention of one agent; HIP events."""
    from paper_2510_12872_amd import hotpath, workloads

    def time_ms(fn, warm, n):
        for i in range(warm):
            fn(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(n):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    res = {}
    for name in ("llama8b_5agents", "pool_scaling_a4", "pool_scaling_a16", "pool_scaling_a32", "pool_scaling_a64",
                 "long_context", "llama70b"):
        w = workloads.WORKLOADS[name]
        model = hotpath.model_of(w)
        one = workloads.scaled(w, n_agents=1, n_segments=1)
        sets = 3 if one.align_bytes() < (8 << 30) else 2           # nothing stays in the 256 MB last-level cache
        segs = [workloads.make_segment(w, 0, j, dev) for j in range(sets)]
        outs = [(torch.empty_like(sg.base_k), torch.empty_like(sg.base_v)) for sg in segs]
        sc = hotpath.Scratch(model, w.seg_len, w.n_anchors, kv.W_TOKEN, dev)

        def run_w(i):
            sg = segs[i % sets]
            kv.kvcomm_anchor_weights(model, sg.base_k, sg.anchor_k, sg.anchor_len, w.temperature, kv.W_TOKEN, sc.weights,
                                     sc.nearest, sc.selected, sc.workspace)

        def run_a(i):
            sg, o = segs[i % sets], outs[i % sets]
            kv.kvcomm_align_kv(model, sg.base_k, sg.base_v, sg.anchor_dk, sg.anchor_dv, sc.weights, sg.delta_pos, o[0], o[1],
                               sg.anchor_len, sg.anchor_delta_pos)

        t_w, t_a = time_ms(run_w, sets, 30), time_ms(run_a, sets, 30)
        r = {"segment": f"S {w.seg_len}, A {w.n_anchors}, L {w.n_layers}",
             "weights_us": t_w * 1e3, "weights_frac_hbm": one.distance_bytes() / t_w / 1e6 / HBM_PEAK_GBS,
             "align_us": t_a * 1e3, "align_frac_hbm": one.align_bytes() / t_a / 1e6 / HBM_PEAK_GBS}
        del segs, outs, sc
        if w.tq > 0:
            ag = workloads.make_agent(w, 0, dev, with_segments=False)
            g = torch.Generator(device=dev)
            g.manual_seed(1)
            for c in (ag.cache_k, ag.cache_v):                       # the slots the alignment would fill
                c[:, :, w.prefix_len:w.n_ctx] = torch.randn(c[:, :, w.prefix_len:w.n_ctx].shape, generator=g,
                                                            device=dev).to(c.dtype)
            out = torch.empty_like(ag.q)
            t_t = time_ms(lambda i: kv.kvcomm_suffix_attn(model, ag.q, ag.cache_k, ag.cache_v, w.n_ctx, out=out), 80, 40)
            fl = workloads.scaled(w, n_agents=1).attn_flops()
            r.update({"attn_ms": t_t, "attn_tflops": fl / t_t / 1e9, "attn_frac_mfma": fl / t_t / 1e9 / MFMA_BF16_PEAK_TFLOPS})
            del ag, out
        res[name] = r
        torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    # the shader clock of an idle MI355X needs some tens of milliseconds of load to settle: ten warm-up
    # steps (about 80 ms) put the timed region at the sustained clock
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (profiling runs)")
    ap.add_argument("--no-events", action="store_true", help="no per-call HIP events in the timed region")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip what follows the timed region (other configurations, compressed deviations)")
    ap.add_argument("--configs-only", action="store_true",
                    help="only run the whole steps of configurations 3, 4 and 5 (profiling runs)")
    ap.add_argument("--config-names", default=None,
                    help="with --configs-only: comma-separated workload names instead of all of configurations 3-5")
    ap.add_argument("--no-overlap-info", action="store_true",
                    help="skip the two-stream steps that follow the timed region (profiling runs: every launch of "
                         "the trace then ran alone on the chip)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device copy five times (reference reading for HBM byte counters)")
    ap.add_argument("--hbm-calibration", action="store_true",
                    help="only run the stand-alone streaming probe: a read-only pass and a 1:1 copy over 4 GiB (what "
                         "plain kernels sustain from HBM on this box)")
    ap.add_argument("--per-config", action="store_true",
                    help="only time the kernels of every baseline configuration alone (one segment / one agent)")
    ap.add_argument("--overlap", action="store_true",
                    help="two streams: weights + align of agent i+1 run beside the attention of agent i "
                         "(per-kernel figures then come from a sequential pass before the timed region)")
    ap.add_argument("--attn-blocks", type=int, default=160,
                    help="two-stream steps: compute units the attention launch is confined to (0 = the plain launch)")
    ap.add_argument("--next-rows", action="store_true",
                    help="only time the entry points beyond the reuse step proper (weighting variants, offset "
                         "capture, anchor prediction, 8-bit deviations) on one segment of the workload")
    ap.add_argument("--mfma-calibration", action="store_true",
                    help="only time a library bf16 GEMM and the attention kernel on N(0,1) and on all-zero inputs "
                         "(how far the data-dependent power limit moves the matrix-core rate on this box)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1")
    if args.hbm_calibration:
        # a child process of its own, started before this one touches the GPU
        import subprocess
        probe = os.path.join(ROOT, "paper_2510_12872_amd", "tools", "hbm_stream_probe")
        if not os.path.exists(probe):
            sys.exit("bench.py: the streaming probe is not built (python -m paper_2510_12872_amd.build)")
        out = subprocess.run([probe], check=True, capture_output=True, text=True).stdout.strip().splitlines()[-1]
        res = json.loads(out)
        res["peak_GBps"] = HBM_PEAK_GBS
        print(json.dumps(res))
        return

    import torch

    import paper_2510_12872_amd as kv
    from paper_2510_12872_amd import hotpath, workloads

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    kv.load_library()  # fails loudly if the HIP library is missing
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)   # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read": src.numel() * 4, "bytes_written": dst.numel() * 4,
                                               "launches": 5}}))
        return
    if args.per_config:
        print(json.dumps({"per_config": per_config(torch, kv, dev)}))
        return
    if args.configs_only:
        names = args.config_names.split(",") if args.config_names else None
        pair = (torch.cuda.Stream(), torch.cuda.Stream())   # the first two streams of a process do not share a queue
        print(json.dumps({"configs": config_steps(torch, kv, dev, names, streams=pair) if names
                          else config_steps(torch, kv, dev, streams=pair)}))
        return
    w = workloads.LLAMA8B_5AGENTS
    model = hotpath.model_of(w)
    if args.mfma_calibration:
        print(json.dumps({"mfma_calibration": mfma_calibration(torch, kv, w, model, dev)}))
        return
    if args.next_rows:
        print(json.dumps({"next_rows": next_rows(torch, kv, w, model, dev), "workload": w.name,
                          "unit": "one 512-token segment, all layers and kv heads"}))
        return

    agents = [workloads.make_agent(w, a, dev) for a in range(w.n_agents)]
    outs = [torch.empty_like(ag.q) for ag in agents]
    scratches = [hotpath.AgentScratch(model, [w.seg_len] * w.n_segments, [w.n_anchors] * w.n_segments, kv.W_TOKEN, dev)
                 for _ in agents]
    # job lists of the batched calls: built once, the timed loop only marshals and launches
    wjobs, ajobs = [], []
    for ag, sc in zip(agents, scratches):
        wjobs.append([dict(seg_base_k=seg.base_k, anchor_base_k=seg.anchor_k, anchor_len=seg.anchor_len,
                           weights_out=sc.weights[j], nearest_out=sc.nearest[j], selected_out=sc.selected[j])
                      for j, seg in enumerate(ag.segments)])
        ajobs.append([dict(base_k=seg.base_k, base_v=seg.base_v, anchor_dk=seg.anchor_dk, anchor_dv=seg.anchor_dv,
                           anchor_len=seg.anchor_len, weights=sc.weights[j], delta_pos=seg.delta_pos,
                           anchor_delta_pos=seg.anchor_delta_pos,
                           out_k=ag.cache_k[:, :, w.seg_offset(j):w.seg_offset(j) + w.seg_len],
                           out_v=ag.cache_v[:, :, w.seg_offset(j):w.seg_offset(j) + w.seg_len])
                      for j, seg in enumerate(ag.segments)])
    torch.cuda.synchronize()

    ev = {"weights": [], "align": [], "attn": []}

    def timed(kind, record, fn):
        if not record:
            fn()
            return
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        ev[kind].append((e0, e1))

    def step(record):
        # per agent: all four segments matched in one launch per stage, aligned in one launch, then attention
        for ai, ag in enumerate(agents):
            timed("weights", record, lambda: kv.kvcomm_anchor_weights_batch(
                model, wjobs[ai], w.temperature, kv.W_TOKEN, workspace=scratches[ai].workspace))
            timed("align", record, lambda: kv.kvcomm_align_kv_batch(model, ajobs[ai], kv.W_TOKEN))
            timed("attn", record, lambda: kv.kvcomm_suffix_attn(model, ag.q, ag.cache_k, ag.cache_v, w.n_ctx,
                                                                out=outs[ai]))

    # Two-stream form of the step: weights + alignment of the next agent beside the attention of the current one,
    # the attention confined to --attn-blocks compute units (hotpath.TwoStreamPipeline).
    pipe = hotpath.TwoStreamPipeline(model, w.temperature, args.attn_blocks)

    def overlapped_steps(n):
        pipe.fork()
        for _ in range(n):
            for ai, ag in enumerate(agents):
                pipe.submit(ai, wjobs[ai], ajobs[ai], scratches[ai].workspace, ag.q, ag.cache_k, ag.cache_v, w.n_ctx,
                            outs[ai])
        pipe.join()

    for _ in range(args.warmup):
        step(False)
    if args.overlap:
        for _ in range(5):               # per-kernel durations, one kernel on the chip at a time
            step(not args.no_events)
        pipe.pick_attention_stream(overlapped_steps)
        overlapped_steps(3)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    if args.overlap:
        overlapped_steps(args.steps)
    else:
        for _ in range(args.steps):
            step(not args.no_events)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    overlap_ms = None
    if not args.overlap and not args.no_overlap_info:
        # For information, after the timed region: the same steps with the next agent's alignment beside the
        # attention of the current one (two streams).  `value` and the rooflines above do not use it.
        n_ov = max(1, min(args.steps, 30))
        pipe.pick_attention_stream(overlapped_steps)
        overlapped_steps(5)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        overlapped_steps(n_ov)
        torch.cuda.synchronize()
        overlap_ms = (time.perf_counter() - t1) / n_ov * 1e3

    def avg_ms(kind):
        return _stats(ev[kind])[0]

    def med_ms(kind):
        return _stats(ev[kind])[1]

    seg_w = workloads.scaled(w, n_agents=1)                 # one align / weights launch = the segments of one agent
    agent_w = workloads.scaled(w, n_agents=1)                # one attention launch = one agent
    kernels = {}
    t_align, t_weights, t_attn = avg_ms("align"), avg_ms("weights"), avg_ms("attn")
    if t_align:
        ach = seg_w.align_bytes() / (t_align * 1e-3) / 1e9
        kernels["align_kv"] = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                               "frac": ach / HBM_PEAK_GBS, "avg_launch_ms": t_align, "median_launch_ms": med_ms("align"),
                               "bytes_per_launch": seg_w.align_bytes(), "traffic": HBM_TRAFFIC_BYTES["align_kv"]}
    if t_weights:
        ach = seg_w.distance_bytes() / (t_weights * 1e-3) / 1e9
        kernels["anchor_weights"] = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                     "frac": ach / HBM_PEAK_GBS, "avg_launch_ms": t_weights, "median_launch_ms": med_ms("weights"),
                                     "bytes_per_launch": seg_w.distance_bytes(), "traffic": HBM_TRAFFIC_BYTES["anchor_weights"],
                                     "note": "two kernels per call (partial distances + softmax finalize)"}
    if t_attn:
        ach = agent_w.attn_flops() / (t_attn * 1e-3) / 1e12
        kernels["suffix_attn"] = {"bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                  "frac": ach / MFMA_BF16_PEAK_TFLOPS, "avg_launch_ms": t_attn, "median_launch_ms": med_ms("attn"),
                                  "flops_per_launch": agent_w.attn_flops(), "traffic": HBM_TRAFFIC_BYTES["suffix_attn"],
                                  "mfma_busy_frac_rocprof": SUFFIX_ATTN_MFMA_BUSY_FRAC}
    # dominant kernel = the one with the largest share of a step
    share = {"align_kv": (t_align or 0) * w.n_agents,
             "anchor_weights": (t_weights or 0) * w.n_agents,
             "suffix_attn": (t_attn or 0) * w.n_agents}
    dominant = max(share, key=share.get) if kernels else None
    roofline = None
    if dominant:
        k = kernels[dominant]
        roofline = {"kernel": dominant, "bound": k["bound"], "achieved": k["achieved"], "peak": k["peak"],
                    "unit": k["unit"], "frac": k["frac"], "traffic": k["traffic"]}

    result = {
        "metric": "aligned KV tokens/s (all layers), whole reuse step: anchor weights + align + suffix attention",
        "value": w.aligned_tokens / (elapsed / args.steps),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": w.name, "n_agents": w.n_agents, "segments_per_agent": w.n_segments,
                   "seg_len": w.seg_len, "n_anchors": w.n_anchors, "n_ctx": w.n_ctx, "tq": w.tq,
                   "layers": w.n_layers, "kv_heads": w.n_kv_heads, "q_heads": w.n_q_heads, "head_dim": w.head_dim,
                   "aligned_tokens_per_step": w.aligned_tokens},
        "align_tokens_per_s": (w.aligned_tokens / ((t_align + t_weights) * w.n_agents * 1e-3)
                               if t_align and t_weights else None),
        "suffix_attn_tflops": kernels.get("suffix_attn", {}).get("achieved"),
        "roofline": roofline,
        "kernels": kernels,
    }
    if args.overlap:
        result["overlap"] = (f"two streams, attention confined to {args.attn_blocks} CUs; roofline / kernels from a "
                             "sequential pass before the timed region")
    elif overlap_ms is not None:
        result["two_stream_overlap"] = {"ms_per_step": overlap_ms, "tokens_per_s": w.aligned_tokens / (overlap_ms * 1e-3),
                                        "attn_blocks": args.attn_blocks, "steps": n_ov,
                                        "note": "same steps on two streams: the next agent's weights + alignment beside the "
                                                "attention of the current one, the attention confined to attn_blocks CUs "
                                                "(kvcomm_suffix_attn_confined); not used for value"}
    if not args.no_extras and not args.overlap:
        # After the timed region, for the record: the same step on compressed deviations, then whole steps of the
        # other baseline configurations (3: pool scaling, 4: long context, 5: 70B shape).
        result["compressed_deviations"] = compressed_step(torch, kv, w, model, agents, outs, scratches, wjobs,
                                                          pipe=pipe if overlap_ms is not None else None)
        agents.clear(), outs.clear(), scratches.clear(), wjobs.clear(), ajobs.clear()   # config 5 needs the room
        torch.cuda.empty_cache()
        result["configs"] = config_steps(torch, kv, dev, streams=(pipe.s_align, pipe.s_attn) if overlap_ms is not None else None)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
