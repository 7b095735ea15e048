"""Pins for the oracle's RoPE rotation (O1), distances (O2) and weights (O3).

None of these tests re-types the oracle's own formula: each checks it against a
closed form, a library routine (numpy / scipy), a brute-force restatement in a
different formulation (complex multiplication for RoPE) or an invariant the
paper fixes (Sec. 3.1: the rotation is orthogonal and additive in the position;
Eq. "pred" / Eq. "ph_update": softmax of negative l2 distance across anchors).
"""
import os

import numpy as np
import pytest
import scipy.special

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
rng = np.random.default_rng(1234)


# ----------------------------------------------------------------------------- O1
def test_rope_zero_delta_is_identity_bit_exact():
    x = rng.standard_normal((5, 64))
    assert np.array_equal(oracle.rope_rotate(x, 0, 1e4), x)


def test_rope_golden_closed_forms():
    """tests/golden/rope_closed_form.txt: hand-derived rotations (quarter / half / full turns)."""
    rows = []
    with open(os.path.join(GOLDEN, "rope_closed_form.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                rows.append(line)
    assert len(rows) >= 4
    for row in rows:
        D, theta, delta, xin, yout = row.split("|")
        x = np.array([float(v) for v in xin.split()])
        y = np.array([float(v) for v in yout.split()])
        delta = eval(delta, {"pi": np.pi})  # the fixture writes multiples of pi
        got = oracle.rope_rotate(x, delta, float(theta))
        assert got.shape == (int(D),)
        np.testing.assert_allclose(got, y, atol=1e-12)


def test_rope_d2_is_plane_rotation_matrix():
    # D = 2: a single pair with frequency theta^0 = 1, so R_delta is the 2x2 rotation by delta.
    for delta in [0.3, -1.7, 5.0]:
        R = np.array([[np.cos(delta), -np.sin(delta)], [np.sin(delta), np.cos(delta)]])
        x = rng.standard_normal(2)
        np.testing.assert_allclose(oracle.rope_rotate(x, delta, 1e4), R @ x, atol=1e-14)


def test_rope_matches_complex_multiplication():
    # Independent formulation: z_i = x_i + j x_{i+D/2};  z_i -> z_i * exp(j * delta * theta^(-2i/D)).
    D, theta, delta = 16, 5e5, 37
    x = rng.standard_normal((3, D))
    z = x[:, : D // 2] + 1j * x[:, D // 2:]
    ang = delta * np.exp(-np.log(theta) * (2 * np.arange(D // 2) / D))
    z2 = z * np.exp(1j * ang)
    want = np.concatenate([z2.real, z2.imag], axis=1)
    np.testing.assert_allclose(oracle.rope_rotate(x, delta, theta), want, atol=1e-12)


def test_rope_unit_vector_touches_only_its_pair():
    D = 8
    for i in range(D // 2):
        e = np.zeros(D)
        e[i] = 1.0
        y = oracle.rope_rotate(e, 3, 1e4)
        mask = np.ones(D, bool)
        mask[[i, i + D // 2]] = False
        assert np.all(y[mask] == 0.0)
        assert abs(y[i] ** 2 + y[i + D // 2] ** 2 - 1.0) < 1e-14
    # frequencies fall with the pair index: the first pair turns fastest
    e0 = np.zeros(D); e0[0] = 1
    e3 = np.zeros(D); e3[3] = 1
    assert abs(oracle.rope_rotate(e0, 1, 1e4)[D // 2]) > abs(oracle.rope_rotate(e3, 1, 1e4)[3 + D // 2])
    # and the turn is counter-clockwise in the (i, i+D/2) plane for positive delta
    assert oracle.rope_rotate(e0, 1, 1e4)[D // 2] > 0


def test_rope_composition_and_orthogonality():
    D, theta = 64, 1e4
    x = rng.standard_normal((4, D))
    y = rng.standard_normal((4, D))
    a, b = 64, 193
    ab = oracle.rope_rotate(oracle.rope_rotate(x, a, theta), b, theta)
    np.testing.assert_allclose(ab, oracle.rope_rotate(x, a + b, theta), atol=1e-12)
    back = oracle.rope_rotate(oracle.rope_rotate(x, a, theta), -a, theta)
    np.testing.assert_allclose(back, x, atol=1e-12)
    rx = oracle.rope_rotate(x, a, theta)
    np.testing.assert_allclose(np.linalg.norm(rx, axis=1), np.linalg.norm(x, axis=1), rtol=1e-13)
    # <R_a q, R_b k> depends only on b - a (the property attention relies on)
    lhs = np.sum(oracle.rope_rotate(x, a, theta) * oracle.rope_rotate(y, b, theta), axis=1)
    rhs = np.sum(x * oracle.rope_rotate(y, b - a, theta), axis=1)
    np.testing.assert_allclose(lhs, rhs, atol=1e-11)


# ----------------------------------------------------------------------------- O2
def _caches(L=2, H=3, S=5, D=8, lens=(5, 7, 5)):
    seg = rng.standard_normal((L, H, S, D))
    anc = [rng.standard_normal((L, H, n, D)) for n in lens]
    return seg, anc


def test_distances_match_numpy_norm_all_granularities():
    seg, anc = _caches()
    L, H, S, D = seg.shape
    d0, sel = oracle.distances(seg, anc, oracle.GRAN_TOKEN)
    d1, _ = oracle.distances(seg, anc, oracle.GRAN_LAYER_HEAD_TOKEN)
    d2, _ = oracle.distances(seg, anc, oracle.GRAN_SEGMENT)
    assert sel.tolist() == [1, 1, 1]
    for a, ak in enumerate(anc):
        diff = seg - ak[:, :, :S, :]
        for t in range(S):
            assert abs(d0[a, t] - np.linalg.norm(diff[:, :, t, :].ravel())) < 1e-12
        want1 = np.linalg.norm(diff, axis=3).reshape(-1)        # [L,H,S] flattened
        np.testing.assert_allclose(d1[a], want1, atol=1e-12)
        assert abs(d2[a, 0] - np.linalg.norm(diff.ravel())) < 1e-12
    # granularities are consistent: squares add up
    np.testing.assert_allclose((d1.reshape(len(anc), L * H, S) ** 2).sum(1), d0 ** 2, rtol=1e-12)
    np.testing.assert_allclose((d0 ** 2).sum(1), d2[:, 0] ** 2, rtol=1e-12)


def test_distances_selection_rule_and_zero_for_identical():
    seg, anc = _caches(lens=(4, 5, 9))
    anc[1] = seg.copy()
    d, sel = oracle.distances(seg, anc)
    assert sel.tolist() == [0, 1, 1]          # shorter anchor is not selected, equal length is
    assert np.all(d[0] == 0.0) and np.all(d[1] == 0.0) and np.all(d[2] > 0)
    # only the first S tokens of a longer anchor count
    anc2 = [a.copy() for a in anc]
    anc2[2][:, :, 5:, :] += 100.0
    d2, _ = oracle.distances(seg, anc2)
    assert np.array_equal(d, d2)


def test_distances_invariant_under_common_rotation():
    seg, anc = _caches(D=16)
    d, _ = oracle.distances(seg, anc)
    segr = oracle.rope_rotate(seg, 77, 1e4)
    ancr = [oracle.rope_rotate(a, 77, 1e4) for a in anc]
    dr, _ = oracle.distances(segr, ancr)
    np.testing.assert_allclose(d, dr, rtol=1e-12)


# ----------------------------------------------------------------------------- O3
def test_weights_match_scipy_softmax_and_sum_to_one():
    d = np.abs(rng.standard_normal((6, 11))) * 3
    sel = np.ones(6, dtype=np.intc)
    for tau in [1.0, 0.25, 4.0]:
        w, nearest = oracle.weights(d, sel, tau)
        np.testing.assert_allclose(w, scipy.special.softmax(-d / tau, axis=0), rtol=1e-12)
        np.testing.assert_allclose(w.sum(0), 1.0, rtol=1e-13)
        assert np.array_equal(nearest, np.argmin(d, axis=0))


def test_weights_single_anchor_and_masked_anchors():
    d = np.abs(rng.standard_normal((1, 7)))
    w, nearest = oracle.weights(d, [1])
    assert np.all(w == 1.0) and np.all(nearest == 0)
    d = np.abs(rng.standard_normal((4, 7)))
    sel = np.array([1, 0, 1, 0], dtype=np.intc)
    d[1] = 0.0  # an unselected anchor must not win even at distance 0
    w, nearest = oracle.weights(d, sel)
    assert np.all(w[1] == 0.0) and np.all(w[3] == 0.0)
    np.testing.assert_allclose(w[[0, 2]], scipy.special.softmax(-d[[0, 2]], axis=0), rtol=1e-12)
    assert set(nearest.tolist()) <= {0, 2}
    w, nearest = oracle.weights(d, [0, 0, 0, 0])
    assert np.all(w == 0.0) and np.all(nearest == -1)


def test_weights_identical_anchor_takes_all_as_temperature_vanishes():
    seg, anc = _caches(lens=(5, 5, 5, 5))
    anc[2] = seg.copy()
    d, sel = oracle.distances(seg, anc)
    prev = None
    for tau in [1.0, 0.1, 1e-2, 1e-4]:
        w, nearest = oracle.weights(d, sel, tau)
        assert np.all(nearest == 2)
        if prev is not None:
            assert np.all(w[2] >= prev)
        prev = w[2]
    np.testing.assert_allclose(prev, 1.0, atol=1e-12)


def test_weights_permutation_equivariance_ties_and_shift():
    d = np.abs(rng.standard_normal((5, 9)))
    sel = np.ones(5, dtype=np.intc)
    w, _ = oracle.weights(d, sel)
    perm = np.array([3, 0, 4, 1, 2])
    wp, _ = oracle.weights(d[perm], sel)
    np.testing.assert_allclose(wp, w[perm], rtol=1e-14)  # the denominator's summation order moves
    # duplicated anchors get exactly equal weights and the lowest index is the nearest
    d[4] = d[1]
    d[1] = d[4] = d.min(0) * 0.5
    w, nearest = oracle.weights(d, sel)
    assert np.array_equal(w[1], w[4]) and np.all(nearest == 1)
    # softmax depends on distance differences only
    w2, _ = oracle.weights(d + 1000.0, sel)
    np.testing.assert_allclose(w2, w, rtol=1e-9)
    # huge distances do not overflow / produce NaN
    w3, _ = oracle.weights(d * 1e6, sel)
    assert np.all(np.isfinite(w3)) and np.allclose(w3.sum(0), 1.0)
