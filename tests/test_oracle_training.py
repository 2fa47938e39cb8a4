"""Pins for the oracle's training-side steps (Algorithm 2 pre-steps, Theorem 4 gradient).

None of these re-types the oracle's formulas: the mask terms are checked by finite differences of
the group means (a different oracle routine), the STE terms by how they must scale, by the clamp
mask, and by their tie to the estimator's alpha and beta; the pre-steps by their invariants.
"""
import json
import os

import numpy as np
import pytest

from oracle import estimate as oest
from oracle import training as otr

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _filter_with_mask(rng, n, scale=0.4):
    w = np.clip(rng.standard_normal(n) * scale, -1.0, 1.0)
    w -= w.mean()
    r = oest.estimate_filter(w)
    return w, np.asarray(r["e"], dtype=np.float64), r


# ------------------------------------------------------------------ MeanCenter / Clamp
def test_mean_center_invariants():
    rng = np.random.default_rng(21)
    W = rng.standard_normal((6, 5, 3, 4)) * 0.7 + 0.3
    cf = otr.mean_center(W, "filter")
    cc = otr.mean_center(W, "channel")
    assert np.allclose(cf.reshape(6, -1).mean(axis=1), 0.0, atol=1e-15)
    assert np.allclose(cc.mean(axis=1), 0.0, atol=1e-15)
    # differences inside the centred unit are untouched
    assert np.allclose(cf[2, 1, 0, 3] - cf[2, 4, 2, 0], W[2, 1, 0, 3] - W[2, 4, 2, 0], atol=1e-15)
    assert np.allclose(cc[3, 0, 1, 2] - cc[3, 4, 1, 2], W[3, 0, 1, 2] - W[3, 4, 1, 2], atol=1e-15)
    # a constant added per unit disappears; centring twice changes nothing
    shift_f = rng.standard_normal((6, 1, 1, 1))
    shift_c = rng.standard_normal((6, 1, 3, 4))
    assert np.allclose(otr.mean_center(W + shift_f, "filter"), cf, atol=1e-14)
    assert np.allclose(otr.mean_center(W + shift_c, "channel"), cc, atol=1e-14)
    assert np.allclose(otr.mean_center(cf, "filter"), cf, atol=1e-15)
    # the two conventions differ unless the taps of a filter share one channel mean
    assert not np.allclose(cf, cc)
    with pytest.raises(ValueError):
        otr.mean_center(W, "rows")


def test_clamp_and_order_of_the_two_steps():
    W = np.array([[[[2.0, -3.0, 0.25, 0.75]]]])            # one filter, n = 4, mean 0
    assert otr.clamp(W).ravel().tolist() == [1.0, -1.0, 0.25, 0.75]
    # centre first, then clamp (Algorithm 2's order): mean of [4, 0, 0, 0] is 1 -> [3, -1, -1, -1] -> [1, -1, -1, -1]
    V = np.array([[[[4.0, 0.0, 0.0, 0.0]]]])
    assert otr.mean_center_clamp(V).ravel().tolist() == [1.0, -1.0, -1.0, -1.0]
    # the other order would give clamp -> [1, 0, 0, 0] -> centre -> [0.75, -0.25, ...]
    assert otr.mean_center(otr.clamp(V)).ravel().tolist() == [0.75, -0.25, -0.25, -0.25]
    assert otr.mean_center_clamp(V, lo=-0.5, hi=2.0).ravel().tolist() == [2.0, -0.5, -0.5, -0.5]


# ------------------------------------------------------------------ Theorem 4
def test_mask_terms_are_the_derivatives_of_the_group_means():
    """d alpha / dW_i = e_i / K and d beta / dW_i = (1 - e_i) / (n - K) with e held fixed: the parts of
    G~1 and G~2 that remain where the STE terms vanish (|W_i| > 1)."""
    rng = np.random.default_rng(22)
    n = 37
    w = rng.standard_normal(n) * 3.0                      # mostly outside [-1, 1]
    e = np.asarray(oest.estimate_filter(w)["e"], dtype=np.float64)
    G1, G2 = otr.gradient_terms(w, e)
    a0, b0 = oest.group_means(w, e)
    h = 1e-6
    for i in range(n):
        wp = w.copy()
        wp[i] += h
        a1, b1 = oest.group_means(wp, e)
        da, db = (a1 - a0) / h, (b1 - b0) / h
        if abs(w[i]) > 1.0:
            assert G1[i] == pytest.approx(da, abs=1e-8)
            assert G2[i] == pytest.approx(db, abs=1e-8)
        # the diagonal of dW~/dW with e fixed is the sum of the two mask terms
        wt0 = otr.binarized_filter(e, a0, b0)
        wt1 = otr.binarized_filter(e, a1, b1)
        diag = (wt1[i] - wt0[i]) / h
        ste_part = (G1[i] + G2[i]) - diag
        if abs(w[i]) > 1.0:
            assert ste_part == pytest.approx(0.0, abs=1e-8)
    assert np.sum(G1[np.abs(w) > 1]) <= 1.0 + 1e-12 and np.sum(G2[np.abs(w) > 1]) <= 1.0 + 1e-12


def test_mask_terms_sum_to_one_per_group():
    rng = np.random.default_rng(23)
    w = rng.standard_normal(50) * 5.0 + 20.0               # every |w| > 1: only the mask terms remain
    e = np.asarray(oest.estimate_filter(w)["e"], dtype=np.float64)
    G1, G2 = otr.gradient_terms(w, e)
    assert G1.sum() == pytest.approx(1.0, rel=1e-13) and G2.sum() == pytest.approx(1.0, rel=1e-13)
    assert np.all(G1[e == 0] == 0.0) and np.all(G2[e == 1] == 0.0)


def test_ste_terms_scale_quadratically_and_follow_the_clamp_mask():
    rng = np.random.default_rng(24)
    w, e, _ = _filter_with_mask(rng, 64, scale=0.3)
    n, K = w.size, int(e.sum())
    base = e / K + (1.0 - e) / (n - K)
    G = otr.gradient_factor(w, e)
    for c in (0.5, 0.25):
        Gc = otr.gradient_factor(c * w, e)                  # same mask; norms and values both scale by c
        assert np.allclose(Gc - base, c * c * (G - base), rtol=1e-12, atol=1e-15)
    # entries pushed outside [-1, 1] lose their STE term but still count in the l1 norms
    w2 = w.copy()
    big = int(np.argmax(w2 * e))
    w2[big] = 1.5
    G2 = otr.gradient_factor(w2, e)
    assert G2[big] == pytest.approx(base[big], rel=1e-13)
    other = int(np.argmax(e * (np.arange(n) != big)))
    grew = (G2[other] - base[other]) / (G[other] - base[other])
    assert grew == pytest.approx(np.abs(w2 * e).sum() / np.abs(w * e).sum(), rel=1e-12)


def test_ste_scalars_are_alpha_and_beta_when_each_group_has_one_sign():
    rng = np.random.default_rng(25)
    for _ in range(20):
        w, e, r = _filter_with_mask(rng, 48)
        if np.any(w[e == 1] < 0) != np.all(w[e == 1] < 0) or np.any(w[e == 0] < 0) != np.all(w[e == 0] < 0):
            continue                                        # a group with both signs: the l1 norm is not |sum|
        n, K = w.size, int(e.sum())
        G1, G2 = otr.gradient_terms(w, e)
        assert np.allclose(G1, e / K + abs(r["alpha"]) * w * e, rtol=1e-12, atol=1e-15)
        assert np.allclose(G2, (1 - e) / (n - K) + abs(r["beta"]) * w * (1 - e), rtol=1e-12, atol=1e-15)
        return
    pytest.fail("no one-signed split drawn")


def test_hand_worked_example():
    """Theorem 4 worked by hand for n = 4, K = 2 (values in the fixture's comment)."""
    with open(os.path.join(GOLDEN, "theorem4_hand_example.json")) as fh:
        g = json.load(fh)
    G1, G2 = otr.gradient_terms(np.array(g["w"]), np.array(g["e"]))
    assert G1.tolist() == g["G1"] and G2.tolist() == g["G2"]
    up = np.array(g["upstream"])
    got = otr.weight_gradient(np.array([g["w"]]), np.array([g["e"]]), up.reshape(1, -1))
    assert got.ravel().tolist() == g["dW"]


def test_full_or_empty_mask_is_refused():
    with pytest.raises(ValueError):
        otr.gradient_terms(np.array([0.1, 0.2]), np.array([1, 1]))
    with pytest.raises(ValueError):
        otr.gradient_terms(np.array([0.1, 0.2]), np.array([0, 0]))
