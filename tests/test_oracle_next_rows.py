"""Pins for the oracle's offset capture (O6), anchor prediction (O7) and weighting variants (O8).

O6 is the fallback branch of Algorithm 1 (the offset between the real and the base cache fills a new
anchor); it is pinned as the exact inverse of the offset approximation.  O7 is Eq. "pred" with the
entropy read as -sum w log w (sensitivity table: reuse rises with gamma); pinned by scipy's entropy and
the closed forms log(k) / 0.  O8 are the nearest-anchor and cosine-similarity variants of the appendix
on the approximation method; pinned by numpy / scipy routines and geometric special cases.
"""
import numpy as np
import scipy.spatial.distance
import scipy.special
import scipy.stats

import oracle

rng = np.random.default_rng(99)
THETA = 5e5


# ----------------------------------------------------------------------------- O6
def test_capture_inverts_align_and_values_ignore_delta():
    L, H, S, D = 2, 3, 5, 16
    bk, bv, rk, rv = (rng.standard_normal((L, H, S, D)) for _ in range(4))
    dk, dv = oracle.capture(bk, bv, rk, rv, 300, THETA)
    w = np.ones((1, S))
    k2, v2 = oracle.align(bk, bv, [dk], [dv], w, 300, THETA)
    np.testing.assert_allclose(k2, rk, atol=1e-12)
    np.testing.assert_allclose(v2, rv, atol=1e-12)
    # value offsets are a plain difference whatever the position delta
    _, dv2 = oracle.capture(bk, bv, rk, rv, 7, THETA)
    assert np.array_equal(dv, rv - bv) and np.array_equal(dv2, dv)
    # zero delta: key offsets are a plain difference too; real == rotated base: zero offset
    dk0, _ = oracle.capture(bk, bv, rk, rv, 0, THETA)
    assert np.array_equal(dk0, rk - bk)
    dkz, dvz = oracle.capture(bk, bv, oracle.rope_rotate(bk, 300, THETA), bv, 300, THETA)
    assert np.max(np.abs(dkz)) < 1e-13 and np.all(dvz == 0)
    # the key offset is taken against the ROTATED base (a sign / frame mistake shows here)
    np.testing.assert_allclose(dk, rk - oracle.rope_rotate(bk, 300, THETA), atol=1e-13)


# ----------------------------------------------------------------------------- O7
def test_predict_entropy_matches_scipy_and_closed_forms():
    A, n = 5, 7
    w = scipy.special.softmax(rng.standard_normal((A, n)) * 2, axis=0)
    sel = np.ones(A, dtype=np.intc)
    lens = [10] * A
    new, ent, mean = oracle.predict(w, sel, lens, 10, 0.3)
    np.testing.assert_allclose(ent, scipy.stats.entropy(w, axis=0), rtol=1e-12)
    assert abs(mean - ent.mean()) < 1e-14
    assert new == int(mean > 0.3 * np.log(A))
    # uniform weights: entropy log(k), the largest possible -> new anchor for every gamma < 1
    wu = np.full((4, 3), 0.25)
    new, ent, mean = oracle.predict(wu, [1] * 4, [8] * 4, 8, 0.99)
    np.testing.assert_allclose(ent, np.log(4), rtol=1e-14)
    assert new == 1
    assert oracle.predict(wu, [1] * 4, [8] * 4, 8, 1.01)[0] == 0
    # one-hot weights: entropy 0 -> shareable (0 * log 0 counts as 0)
    wo = np.zeros((4, 3))
    wo[2] = 1.0
    new, ent, _ = oracle.predict(wo, [1] * 4, [8] * 4, 8, 0.3)
    assert new == 0 and np.all(ent == 0)


def test_predict_length_rule_and_selection():
    w = np.full((3, 2), 1 / 3)
    # longer than every anchor -> new anchor, whatever the entropy says
    assert oracle.predict(np.array([[1.0], [0.0], [0.0]]), [0, 0, 0], [4, 5, 6], 7, 0.3)[0] == 1
    # as long as the longest anchor is not "longer": the decision falls to the entropy test
    wsel = np.array([[0.0], [0.0], [1.0]])
    assert oracle.predict(wsel, [0, 0, 1], [4, 5, 7], 7, 0.3)[0] == 0
    # threshold uses the number of CANDIDATE anchors, and unselected weights never count
    w2 = np.array([[0.5, 0.5], [0.5, 0.5], [0.9, 0.9]])
    new, ent, _ = oracle.predict(w2, [1, 1, 0], [9, 9, 3], 9, 0.99)
    np.testing.assert_allclose(ent, np.log(2), rtol=1e-14)
    assert new == 1                                 # log 2 > 0.99 log 2
    assert oracle.predict(w2, [1, 1, 0], [9, 9, 3], 9, 1.0)[0] == 0
    # gamma monotonicity: a larger gamma can only turn "new anchor" into "shareable"
    wm = scipy.special.softmax(rng.standard_normal((6, 4)), axis=0)
    dec = [oracle.predict(wm, [1] * 6, [5] * 6, 5, g)[0] for g in (0.0, 0.3, 0.6, 0.9, 1.2)]
    assert dec == sorted(dec, reverse=True) and dec[0] == 1 and dec[-1] == 0


# ----------------------------------------------------------------------------- O8
def _caches(L=2, H=2, S=4, D=8, lens=(4, 6, 4)):
    seg = rng.standard_normal((L, H, S, D))
    anc = [rng.standard_normal((L, H, n, D)) for n in lens]
    return seg, anc


def test_cosine_matches_scipy_all_granularities():
    seg, anc = _caches()
    L, H, S, D = seg.shape
    for gran in (oracle.GRAN_TOKEN, oracle.GRAN_LAYER_HEAD_TOKEN, oracle.GRAN_SEGMENT):
        sim, sel = oracle.cosine(seg, anc, gran)
        assert sel.tolist() == [1, 1, 1]
        for a, ak in enumerate(anc):
            y = ak[:, :, :S]
            if gran == oracle.GRAN_TOKEN:
                want = [1 - scipy.spatial.distance.cosine(seg[:, :, t].ravel(), y[:, :, t].ravel()) for t in range(S)]
            elif gran == oracle.GRAN_LAYER_HEAD_TOKEN:
                want = [1 - scipy.spatial.distance.cosine(seg[l, h, t], y[l, h, t])
                        for l in range(L) for h in range(H) for t in range(S)]
            else:
                want = [1 - scipy.spatial.distance.cosine(seg.ravel(), y.ravel())]
            np.testing.assert_allclose(sim[a], want, atol=1e-12)


def test_cosine_special_cases():
    seg, anc = _caches(lens=(4, 4, 3, 4))
    anc[0] = 3.5 * seg            # parallel: similarity 1, scale invariant
    anc[1] = -seg                 # anti-parallel: -1
    anc[3] = np.zeros_like(seg)   # zero vector: defined as 0
    sim, sel = oracle.cosine(seg, anc)
    assert sel.tolist() == [1, 1, 0, 1]
    np.testing.assert_allclose(sim[0], 1.0, atol=1e-12)
    np.testing.assert_allclose(sim[1], -1.0, atol=1e-12)
    assert np.all(sim[2] == 0) and np.all(sim[3] == 0)
    w, best = oracle.weights_from_sim(sim, sel, tau=1.0)
    assert np.all(best == 0) and np.all(w[2] == 0)
    np.testing.assert_allclose(w[[0, 1, 3]], scipy.special.softmax(sim[[0, 1, 3]], axis=0), rtol=1e-12)
    # a common rotation of segment and anchors changes no similarity
    simr, _ = oracle.cosine(oracle.rope_rotate(seg, 11, 1e4), [oracle.rope_rotate(a, 11, 1e4) for a in anc])
    np.testing.assert_allclose(simr, sim, atol=1e-12)
    w2, _ = oracle.weights_from_sim(sim, sel, tau=1e-4)
    np.testing.assert_allclose(w2[0], 1.0, atol=1e-12)
    # exactly equal similarities: equal weights, and the most similar anchor is the one of lowest index
    tied = np.array([[0.25, 0.9], [0.75, 0.9], [0.75, 0.1], [0.75, 0.9]])
    wt, bt = oracle.weights_from_sim(tied, np.array([1, 1, 1, 1], dtype=np.int32), tau=0.5)
    assert bt.tolist() == [1, 0]
    assert wt[1, 0] == wt[2, 0] == wt[3, 0] and wt[0, 1] == wt[1, 1] == wt[3, 1]
    wt, bt = oracle.weights_from_sim(tied, np.array([1, 0, 1, 1], dtype=np.int32), tau=0.5)
    assert bt.tolist() == [2, 0] and np.all(wt[1] == 0)


def test_nearest_is_argmin_one_hot_and_limit_of_softmax():
    d = np.abs(rng.standard_normal((5, 9)))
    d[3] = d[1]                                    # tie between anchors 1 and 3
    d[1, :] = d[3, :] = d.min(0) * 0.5
    sel = np.array([1, 1, 0, 1, 1], dtype=np.intc)
    w, nearest = oracle.weights_nearest(d, sel)
    assert np.all(nearest == 1)                    # lowest index among equals
    assert np.all(w.sum(0) == 1) and np.all(w[1] == 1) and set(np.unique(w)) == {0.0, 1.0}
    # agrees with the arg-min the softmax weights report, and is its tau -> 0 limit when untied
    d2 = np.abs(rng.standard_normal((5, 9)))
    w_n, near2 = oracle.weights_nearest(d2, sel)
    w_s, near3 = oracle.weights(d2, sel, tau=1e-6)
    assert np.array_equal(near2, near3)
    np.testing.assert_allclose(w_s, w_n, atol=1e-12)
    dm = np.where(sel[:, None] == 1, d2, np.inf)
    assert np.array_equal(near2, np.argmin(dm, axis=0))
    assert np.all(oracle.weights_nearest(d2, [0] * 5)[1] == -1)


# ----------------------------------------------------------------------------- O9
def test_e4m3_codec_against_library_and_closed_forms():
    """The 8-bit storage format of compressed deviations: every code against torch's float8_e4m3fn (an
    independent implementation of the OCP format), hand-computed codes, ties to even, saturation."""
    import torch
    codes = np.arange(256, dtype=np.uint8)
    lib = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    mine = np.array([oracle.e4m3_decode(c) for c in codes])
    assert np.isnan(mine[0x7f]) and np.isnan(mine[0xff]) and np.isnan(lib[0x7f])
    ok = ~np.isnan(lib)
    assert np.array_equal(mine[ok], lib[ok])
    # closed forms: 0 0111 000 = 1; largest finite 0 1111 110 = 448; smallest subnormal 2^-9; smallest normal 2^-6
    assert oracle.e4m3_decode(0x38) == 1.0 and oracle.e4m3_decode(0x7e) == 448.0
    assert oracle.e4m3_decode(0x01) == 2.0 ** -9 and oracle.e4m3_decode(0x08) == 2.0 ** -6
    assert oracle.e4m3_decode(0xb8) == -1.0
    # encoding: exact values round-trip; random values agree with the library inside the range
    for c in codes[ok]:
        v = oracle.e4m3_decode(c)
        if v == 0.0:
            continue
        assert oracle.e4m3_encode(v) == c
    x = np.concatenate([rng.standard_normal(4000) * 0.05 * 1024, rng.uniform(-448, 448, 2000),
                        rng.uniform(-2 ** -6, 2 ** -6, 2000)])
    want = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([oracle.e4m3_encode(v) for v in x], dtype=np.uint8)
    same_value = np.array([oracle.e4m3_decode(a) == oracle.e4m3_decode(b) for a, b in zip(got, want)])
    assert same_value.all()                                  # (+0 / -0 codes may differ, values may not)
    # ties go to the even mantissa: halfway 1.0|1.125 -> 1.0 ; halfway 1.125|1.25 -> 1.25 ; subnormal half steps
    assert oracle.e4m3_encode(1.0625) == 0x38 and oracle.e4m3_encode(1.1875) == 0x3a
    assert oracle.e4m3_encode(2.0 ** -10) == 0x00 and oracle.e4m3_encode(3 * 2.0 ** -10) == 0x02
    # just above a tie rounds up, saturation, sign
    assert oracle.e4m3_encode(1.0626) == 0x39
    assert oracle.e4m3_encode(1e6) == 0x7e and oracle.e4m3_encode(-1e6) == 0xfe and oracle.e4m3_encode(449.0) == 0x7e
    assert oracle.e4m3_encode(-0.3) == (0x80 | oracle.e4m3_encode(0.3))


def test_quantize_error_bound_and_scale():
    x = rng.standard_normal(5000) * 0.05
    scale = 2.0 ** -10
    q = oracle.quantize(x, scale)
    y = oracle.dequantize(q, scale)
    big = np.abs(x) >= scale * 2.0 ** -6
    assert np.all(np.abs(y[big] - x[big]) <= np.abs(x[big]) * 2.0 ** -4)
    assert np.all(np.abs(y[~big] - x[~big]) <= scale * 2.0 ** -10)
    # scaling input and scale together leaves the codes unchanged (the scale is a power of two)
    assert np.array_equal(oracle.quantize(x * 4, scale * 4), q)
    assert np.array_equal(oracle.dequantize(q, 2 * scale), 2 * y)
