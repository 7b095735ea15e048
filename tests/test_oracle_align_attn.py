"""Pins for the oracle's offset approximation (O4) and suffix attention (O5).

O4 follows Eq. "ph_update" (weighted sum of anchor deviations added to the base
cache, keys first rotated to the new position).  It is pinned by the special
cases in which the rule collapses to something with a closed form, by linearity,
and by a brute-force restatement with numpy einsum on complex-valued keys.
O5 is the textbook causal softmax(QK^T/sqrt(d))V of Sec. 3.1 and is pinned by a
brute-force numpy/scipy evaluation with an explicit mask and by closed forms.
"""
import numpy as np
import scipy.special

import oracle

rng = np.random.default_rng(4321)
THETA = 1e4


def _problem(L=2, H=2, S=6, D=8, lens=(6, 6, 9), sigma=0.1):
    K = rng.standard_normal((L, H, S, D))
    V = rng.standard_normal((L, H, S, D))
    dK = [sigma * rng.standard_normal((L, H, n, D)) for n in lens]
    dV = [sigma * rng.standard_normal((L, H, n, D)) for n in lens]
    w = scipy.special.softmax(rng.standard_normal((len(lens), S)), axis=0)
    return K, V, dK, dV, w


# ----------------------------------------------------------------------------- O4
def test_align_zero_deviation_zero_delta_is_identity_bit_exact():
    K, V, dK, dV, w = _problem()
    z = [np.zeros_like(a) for a in dK]
    k2, v2 = oracle.align(K, V, z, z, w, 0, THETA)
    assert np.array_equal(k2, K) and np.array_equal(v2, V)


def test_align_zero_deviation_is_pure_rotation_and_values_ignore_delta():
    K, V, dK, dV, w = _problem()
    z = [np.zeros_like(a) for a in dK]
    k2, v2 = oracle.align(K, V, z, z, w, 192, THETA)
    np.testing.assert_allclose(k2, oracle.rope_rotate(K, 192, THETA), atol=1e-14)
    assert np.array_equal(v2, V)
    _, v3 = oracle.align(K, V, dK, dV, w, 5, THETA)
    _, v4 = oracle.align(K, V, dK, dV, w, 4096, THETA)
    assert np.array_equal(v3, v4)


def test_align_equal_deviations_make_weights_irrelevant():
    K, V, dK, dV, w = _problem(lens=(6, 6, 6))
    E, F = dK[0], dV[0]
    k2, v2 = oracle.align(K, V, [E] * 3, [F] * 3, w, 64, THETA)
    np.testing.assert_allclose(k2, oracle.rope_rotate(K, 64, THETA) + E, atol=1e-13)
    np.testing.assert_allclose(v2, V + F, atol=1e-13)
    w2 = scipy.special.softmax(rng.standard_normal(w.shape) * 3, axis=0)
    k3, v3 = oracle.align(K, V, [E] * 3, [F] * 3, w2, 64, THETA)
    np.testing.assert_allclose(k3, k2, atol=1e-13)


def test_align_single_anchor_and_anchor_frames():
    K, V, dK, dV, _ = _problem(lens=(7,))
    S = K.shape[2]
    w = np.ones((1, S))
    k2, v2 = oracle.align(K, V, dK, dV, w, 100, THETA)
    np.testing.assert_allclose(k2, oracle.rope_rotate(K, 100, THETA) + dK[0][:, :, :S], atol=1e-13)
    np.testing.assert_allclose(v2, V + dV[0][:, :, :S], atol=1e-13)
    # deviation recorded at position delta 30, applied at 100: it turns by the remaining 70
    k3, _ = oracle.align(K, V, dK, dV, w, 100, THETA, anc_delta=[30])
    np.testing.assert_allclose(
        k3, oracle.rope_rotate(K, 100, THETA) + oracle.rope_rotate(dK[0][:, :, :S], 70, THETA), atol=1e-13)
    # deviation recorded in the base frame (0): rotating commutes with the sum
    k4, _ = oracle.align(K, V, dK, dV, w, 100, THETA, anc_delta=[0])
    np.testing.assert_allclose(k4, oracle.rope_rotate(K + dK[0][:, :, :S], 100, THETA), atol=1e-13)
    # anc_delta equal to delta is the same as none
    k5, _ = oracle.align(K, V, dK, dV, w, 100, THETA, anc_delta=[100])
    np.testing.assert_allclose(k5, k2, atol=1e-14)


def test_align_brute_force_einsum_complex():
    """Independent restatement: complex RoPE + einsum over the anchor axis."""
    K, V, dK, dV, w = _problem(L=2, H=3, S=5, D=8, lens=(5, 8, 5, 6))
    L, H, S, D = K.shape
    delta, anc_delta = 37, np.array([37, 5, 0, 64])
    freq = THETA ** (-np.arange(D // 2) * 2.0 / D)

    def crot(x, dl):
        z = (x[..., : D // 2] + 1j * x[..., D // 2:]) * np.exp(1j * dl * freq)
        return np.concatenate([z.real, z.imag], axis=-1)

    stack_k = np.stack([crot(a[:, :, :S], delta - ad) for a, ad in zip(dK, anc_delta)])  # [A,L,H,S,D]
    stack_v = np.stack([a[:, :, :S] for a in dV])
    want_k = crot(K, delta) + np.einsum("at,alhtd->lhtd", w, stack_k)
    want_v = V + np.einsum("at,alhtd->lhtd", w, stack_v)
    got_k, got_v = oracle.align(K, V, dK, dV, w, delta, THETA, anc_delta=anc_delta)
    np.testing.assert_allclose(got_k, want_k, atol=1e-12)
    np.testing.assert_allclose(got_v, want_v, atol=1e-12)


def test_align_linearity_permutation_and_short_anchor_skipped():
    K, V, dK, dV, w = _problem(lens=(6, 6, 6))
    zeros = [np.zeros_like(a) for a in dK]
    k0, v0 = oracle.align(K, V, zeros, zeros, w, 9, THETA)
    k1, v1 = oracle.align(K, V, dK, dV, w, 9, THETA)
    k2, v2 = oracle.align(K, V, [2 * a for a in dK], [2 * a for a in dV], w, 9, THETA)
    np.testing.assert_allclose(k2 - k0, 2 * (k1 - k0), atol=1e-13)
    np.testing.assert_allclose(v2 - v0, 2 * (v1 - v0), atol=1e-13)
    perm = [2, 0, 1]
    kp, vp = oracle.align(K, V, [dK[i] for i in perm], [dV[i] for i in perm], w[perm], 9, THETA)
    np.testing.assert_allclose(kp, k1, atol=1e-13)
    np.testing.assert_allclose(vp, v1, atol=1e-13)
    # an anchor shorter than the segment contributes nothing, whatever its weight
    short_k = dK + [rng.standard_normal((2, 2, 3, 8))]
    short_v = dV + [rng.standard_normal((2, 2, 3, 8))]
    w4 = np.concatenate([w, np.full((1, 6), 0.5)])
    ks, vs = oracle.align(K, V, short_k, short_v, w4, 9, THETA)
    np.testing.assert_allclose(ks, k1, atol=1e-14)
    np.testing.assert_allclose(vs, v1, atol=1e-14)


def test_align_granularities_agree_when_weights_are_broadcast():
    K, V, dK, dV, w = _problem(lens=(6, 7))
    L, H, S, D = K.shape
    k0, v0 = oracle.align(K, V, dK, dV, w, 11, THETA, gran=oracle.GRAN_TOKEN)
    w1 = np.broadcast_to(w[:, None, None, :], (2, L, H, S)).reshape(2, -1)
    k1, v1 = oracle.align(K, V, dK, dV, w1, 11, THETA, gran=oracle.GRAN_LAYER_HEAD_TOKEN)
    assert np.array_equal(k0, k1) and np.array_equal(v0, v1)
    ws = np.array([[0.25], [0.75]])
    k2, _ = oracle.align(K, V, dK, dV, ws, 11, THETA, gran=oracle.GRAN_SEGMENT)
    k3, _ = oracle.align(K, V, dK, dV, np.repeat(ws, S, axis=1), 11, THETA, gran=oracle.GRAN_TOKEN)
    assert np.array_equal(k2, k3)
    # per-(layer, head, token) weights really are indexed per layer and head
    w1b = scipy.special.softmax(rng.standard_normal((2, L * H * S)), axis=0)
    k4, _ = oracle.align(K, V, dK, dV, w1b, 11, THETA, gran=oracle.GRAN_LAYER_HEAD_TOKEN)
    wl = w1b.reshape(2, L, H, S)
    want = oracle.rope_rotate(K, 11, THETA) + sum(wl[a][..., None] * dK[a][:, :, :S] for a in range(2))
    np.testing.assert_allclose(k4, want, atol=1e-13)


def test_reuse_step_chains_distance_weights_align():
    L, H, S, D = 2, 2, 4, 8
    seg_k = rng.standard_normal((L, H, S, D))
    seg_v = rng.standard_normal((L, H, S, D))
    anc_k = [rng.standard_normal((L, H, S, D)) for _ in range(3)]
    anc_k[1] = seg_k + 1e-3 * rng.standard_normal((L, H, S, D))   # near-identical anchor
    dK = [rng.standard_normal((L, H, S, D)) for _ in range(3)]
    dV = [rng.standard_normal((L, H, S, D)) for _ in range(3)]
    r = oracle.reuse_step(seg_k, seg_v, anc_k, dK, dV, 16, THETA, tau=1e-3)
    assert np.all(r["nearest"] == 1)
    np.testing.assert_allclose(r["out_k"], oracle.rope_rotate(seg_k, 16, THETA) + dK[1], atol=1e-9)
    np.testing.assert_allclose(r["out_v"], seg_v + dV[1], atol=1e-9)


# ----------------------------------------------------------------------------- O5
def _attn_inputs(L=2, Hq=4, Hkv=2, D=8, n_ctx=5, tq=4):
    q = rng.standard_normal((L, Hq, tq, D))
    k = rng.standard_normal((L, Hkv, n_ctx + tq, D))
    v = rng.standard_normal((L, Hkv, n_ctx + tq, D))
    return q, k, v


def test_attn_brute_force_numpy_mask():
    for (n_ctx, tq, Hq, Hkv) in [(5, 4, 4, 2), (0, 6, 3, 3), (7, 1, 8, 2)]:
        q, k, v = _attn_inputs(Hq=Hq, Hkv=Hkv, n_ctx=n_ctx, tq=tq)
        L, _, _, D = q.shape
        G = Hq // Hkv
        kk = np.repeat(k, G, axis=1)        # query head hq reads kv head hq // G
        vv = np.repeat(v, G, axis=1)
        s = np.einsum("lhid,lhjd->lhij", q, kk) / np.sqrt(D)
        i = np.arange(tq)[:, None]
        j = np.arange(n_ctx + tq)[None, :]
        s = np.where(j <= n_ctx + i, s, -np.inf)
        p = scipy.special.softmax(s, axis=-1)
        want = np.einsum("lhij,lhjd->lhid", p, vv)
        got, lse = oracle.suffix_attn(q, k, v, n_ctx, want_lse=True)
        np.testing.assert_allclose(got, want, atol=1e-12)
        np.testing.assert_allclose(lse, scipy.special.logsumexp(s, axis=-1), atol=1e-12)


def test_attn_closed_forms():
    # a single visible key: the output is that key's value
    q, k, v = _attn_inputs(n_ctx=0, tq=1)
    np.testing.assert_allclose(oracle.suffix_attn(q, k, v, 0), np.repeat(v, 2, axis=1), atol=1e-14)
    # all keys equal: uniform attention, output = running mean of the visible values
    q, k, v = _attn_inputs(n_ctx=3, tq=4)
    k[:] = k[:, :, :1, :]
    out = oracle.suffix_attn(q, k, v, 3)
    for i in range(4):
        want = np.repeat(v[:, :, : 3 + i + 1].mean(axis=2), 2, axis=1)
        np.testing.assert_allclose(out[:, :, i], want, atol=1e-13)
    # an explicit scale is honoured: scale 0 also gives uniform attention
    q, k, v = _attn_inputs(n_ctx=3, tq=2)
    out = oracle.suffix_attn(q, k, v, 3, scale=0.0)
    np.testing.assert_allclose(out[:, :, 1], np.repeat(v.mean(axis=2), 2, axis=1), atol=1e-13)


def test_attn_causality_and_gqa_grouping():
    q, k, v = _attn_inputs(n_ctx=4, tq=5)
    out = oracle.suffix_attn(q, k, v, 4)
    k2, v2 = k.copy(), v.copy()
    k2[:, :, 4 + 3:] += 5.0        # keys after query 2's position
    v2[:, :, 4 + 3:] -= 7.0
    out2 = oracle.suffix_attn(q, k2, v2, 4)
    assert np.array_equal(out[:, :, :3], out2[:, :, :3])
    assert not np.allclose(out[:, :, 3:], out2[:, :, 3:])
    # heads 0,1 share kv head 0; heads 2,3 share kv head 1
    q[:, 1] = q[:, 0]
    q[:, 2] = q[:, 0]
    out = oracle.suffix_attn(q, k, v, 4)
    assert np.array_equal(out[:, 0], out[:, 1])
    assert not np.allclose(out[:, 0], out[:, 2])


def test_attn_rotation_of_q_and_k_by_common_offset_changes_nothing():
    # ties O1 to O5: scores depend on relative positions only
    q, k, v = _attn_inputs(D=16, n_ctx=3, tq=3)
    out = oracle.suffix_attn(q, k, v, 3)
    out2 = oracle.suffix_attn(oracle.rope_rotate(q, 50, THETA), oracle.rope_rotate(k, 50, THETA), v, 3)
    np.testing.assert_allclose(out, out2, atol=1e-12)
