"""Pins of the estimation oracle (CPU only).

Each test ties oracle/estimate.py to something other than itself: exact
rational brute force over every mask, hand arithmetic stored under
tests/golden, closed-form identities of Theorem 2, and a library 2-means.
"""
import json
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import estimate as est


def frac(s):
    return Fraction(s)


def exact_error(w, mask):
    """||W - W~||^2 with the exact group means, in rational arithmetic."""
    wq = [Fraction(float(x)) for x in w]
    g1 = [x for x, m in zip(wq, mask) if m]
    g0 = [x for x, m in zip(wq, mask) if not m]
    m1 = sum(g1) / len(g1)
    m0 = sum(g0) / len(g0)
    return sum((x - m1) ** 2 for x in g1) + sum((x - m0) ** 2 for x in g0)


def draws():
    rng = np.random.default_rng(20240607)
    out = []
    for n in (2, 3, 4, 5, 7, 8, 10, 12):
        out.append(rng.standard_normal(n).astype(np.float32))
        out.append((rng.standard_normal(n) * 0.05 + 0.3).astype(np.float32))
        out.append(rng.laplace(0.01, 0.03, n).astype(np.float32))
        out.append(np.abs(rng.standard_normal(n)).astype(np.float32))          # one-sided
        out.append(-np.abs(rng.standard_normal(n)).astype(np.float32) - 0.5)   # all negative
        out.append(rng.integers(-2, 3, n).astype(np.float32))                  # many duplicates
    return out


def test_worked_example(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "alg1_worked_example.json")))
    w = np.array(g["W"], dtype=np.float32)
    # the stored fractions themselves, re-derived exactly from Algorithm 1's formulas
    ws = sorted(Fraction(x) for x in g["W"])
    assert [float(x) for x in ws] == g["sorted"]
    P = [sum(ws[: i + 1]) for i in range(8)]
    assert P == [frac(s) for s in g["P"]]
    D = [P[i - 1] ** 2 / i + (P[7] - P[i - 1]) ** 2 / (8 - i) for i in range(1, 8)]
    assert D == [frac(s) for s in g["D"]]
    assert sum(x * x for x in ws) - max(D) == frac(g["error"])
    # the oracle against the stored values
    order, Po, Do = est.split_scores(w)
    assert np.array_equal(w[order].astype(np.float64), np.array(g["sorted"]))
    assert np.allclose(Po, [float(x) for x in P], rtol=0, atol=1e-15)
    assert np.allclose(Do, [float(x) for x in D], rtol=1e-15, atol=0)
    r = est.estimate_filter(w)
    assert r["i_star"] == g["i_star"] and r["K"] == g["K"]
    assert r["alpha_is_upper"] == g["alpha_is_upper"]
    assert r["alpha"] == float(frac(g["alpha"])) and r["beta"] == float(frac(g["beta"]))
    assert r["mu_lower"] == float(frac(g["mu_lower"])) and r["mu_upper"] == float(frac(g["mu_upper"]))
    assert r["e"].tolist() == g["e"]
    assert r["thr_val"] == g["thr_val"] and r["thr_idx"] == g["thr_idx"]
    err = float(np.sum((w.astype(np.float64) - est.reconstruct(r["e"], r["alpha"], r["beta"])) ** 2))
    assert err == float(frac(g["error"]))


@pytest.mark.parametrize("k", range(len(draws())))
def test_brute_force_over_all_masks(k):
    """Theorem 2: the sorted split found by the oracle is a global minimiser over all 2^n - 2 masks."""
    w = draws()[k]
    bf = est.brute_force(w)
    r = est.estimate_filter(w)
    assert exact_error(w, r["e"]) == bf["min_err"]
    ones = frozenset(np.flatnonzero(r["e"]).tolist())
    zeros = frozenset(np.flatnonzero(1 - r["e"]).tolist())
    assert frozenset((ones, zeros)) in bf["partitions"]
    # and the oracle's own scalars are the closed-form means of its mask
    a, b = est.group_means(w, r["e"])
    assert abs(a - r["alpha"]) <= 1e-15 * max(1, abs(a)) and abs(b - r["beta"]) <= 1e-15 * max(1, abs(b))


def test_brute_force_n16():
    rng = np.random.default_rng(7)
    w = (rng.standard_normal(16) * 0.1 + 0.02).astype(np.float32)
    bf = est.brute_force(w)
    r = est.estimate_filter(w)
    assert exact_error(w, r["e"]) == bf["min_err"]
    assert len(bf["partitions"]) == 1


def test_any_other_beta_is_worse():
    """beta = +W^T(1-e)/(n-K): flipping its sign (as one listing prints it) raises the error."""
    rng = np.random.default_rng(3)
    w = (rng.standard_normal(64) * 0.05 + 0.04).astype(np.float32)
    r = est.estimate_filter(w)
    e = r["e"]
    good = np.sum((w - est.reconstruct(e, r["alpha"], r["beta"])) ** 2)
    bad = np.sum((w - est.reconstruct(e, r["alpha"], -r["beta"])) ** 2)
    assert good < bad


@pytest.mark.parametrize("n", [2, 9, 64, 576, 1600, 4097])
def test_identities(n):
    rng = np.random.default_rng(n)
    for w in (rng.standard_normal(n) * 0.05 + rng.uniform(-0.02, 0.02),
              rng.laplace(0.005, 0.03, n)):
        w = w.astype(np.float32)
        w64 = w.astype(np.float64)
        r = est.estimate_filter(w)
        wt = est.reconstruct(r["e"], r["alpha"], r["beta"])
        err = np.sum((w64 - wt) ** 2)
        nsq = np.sum(w64 ** 2)
        # appendix, last line of the proof of Theorem 2: E = ||W||^2 - D
        assert abs(err - (nsq - r["maxD"])) <= 1e-12 * nsq
        # the two group sums add up to T: K alpha + (n-K) beta = sum W
        assert abs(r["K"] * r["alpha"] + (n - r["K"]) * r["beta"] - w64.sum()) <= 1e-12 * np.abs(w64).sum()
        assert 1 <= r["K"] <= n - 1 and int(r["e"].sum()) == r["K"]
        # alpha names the mean of greater magnitude (Section 4.1)
        assert abs(r["alpha"]) >= abs(r["beta"])
        # the split is a threshold: every lower element <= every upper element, and the
        # midpoint of the two means separates them (fixed point of 1-D 2-means)
        low = est.lower_group_from_descriptor(w, r["thr_val"], r["thr_idx"])
        assert w64[low].max() <= w64[~low].min()
        mid = 0.5 * (r["mu_lower"] + r["mu_upper"])
        assert w64[low].max() <= mid + 1e-12 and w64[~low].min() >= mid - 1e-12
        # XNOR-Net's alpha*sign(W) is a special case, so it cannot do better (Section 4.1)
        assert err <= np.sum((w64 - est.xnor_reconstruction(w)) ** 2) * (1 + 1e-12)
        # no other split of the sorted order scores higher
        _, _, D = est.split_scores(w)
        assert r["maxD"] == D.max() and r["i_star"] == np.flatnonzero(D == D.max())[-1] + 1


def test_library_two_means_agrees():
    """The objective is 1-D 2-means; a library k-means cannot beat the oracle and, restarted, reaches it."""
    from sklearn.cluster import KMeans
    rng = np.random.default_rng(11)
    for n in (40, 200):
        w = np.concatenate([rng.normal(-0.2, 0.05, n // 4), rng.normal(0.1, 0.08, n - n // 4)]).astype(np.float32)
        r = est.estimate_filter(w)
        err = float(np.sum((w.astype(np.float64) - est.reconstruct(r["e"], r["alpha"], r["beta"])) ** 2))
        km = KMeans(n_clusters=2, n_init=20, random_state=0).fit(w.astype(np.float64).reshape(-1, 1))
        assert err <= km.inertia_ * (1 + 1e-9)
        assert abs(err - km.inertia_) <= 1e-6 * err
        lab = km.labels_ if km.cluster_centers_[1, 0] > km.cluster_centers_[0, 0] else 1 - km.labels_
        low = est.lower_group_from_descriptor(w, r["thr_val"], r["thr_idx"])
        assert np.array_equal(lab == 0, low)


def test_symmetric_filter_is_xnor():
    """Section 4.2: mean-centred W with K = n/2 reproduces XNOR-Net: alpha = -beta = mean|W|."""
    rng = np.random.default_rng(5)
    h = np.abs(rng.standard_normal(32)).astype(np.float32) + 0.01
    w = np.concatenate([h, -h])
    rng.shuffle(w)
    r = est.estimate_filter(w)
    assert r["K"] == 32 and r["alpha_is_upper"] == 1
    assert r["alpha"] == pytest.approx(np.mean(np.abs(w.astype(np.float64))), rel=1e-14)
    assert r["alpha"] == pytest.approx(-r["beta"], rel=1e-14)
    assert np.array_equal(r["e"], (w > 0).astype(np.uint8))
    assert np.allclose(est.reconstruct(r["e"], r["alpha"], r["beta"]), est.xnor_reconstruction(w), rtol=1e-14)


@pytest.mark.parametrize("seed", range(6))
def test_both_passes_give_the_same_partition(seed):
    """Algorithm 1 with its descending pass taken as well: the same two groups, whichever pass is kept."""
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(5, 300))
    w = (rng.standard_normal(n) * 0.05 + rng.uniform(-0.05, 0.05)).astype(np.float32)
    r = est.estimate_filter(w)
    tp = est.two_pass_choice(w)
    # the second pass sees the first one's scores backwards: equal maxima, and with a single maximiser mirrored positions
    assert tp["D_ascending"] == tp["D_descending"] and not tp["descending"]
    order, _, D = est.split_scores(w)
    if np.count_nonzero(D == D.max()) == 1:
        assert tp["K_ascending"] + tp["K_descending"] == n
    # brute force over the descending order itself: running sums of the weights taken from the top
    desc = w.astype(np.float64)[order][::-1]
    T = desc.sum()
    P = np.cumsum(desc)[: n - 1]
    j = np.arange(1, n)
    D_top = P * P / j + (T - P) * (T - P) / (n - j)
    assert np.allclose(D_top, D[::-1], rtol=1e-9, atol=1e-12)
    chosen = frozenset(order[: tp["K"]].tolist())
    ones = frozenset(np.flatnonzero(r["e"]).tolist())
    zeros = frozenset(np.flatnonzero(1 - r["e"]).tolist())
    assert chosen in (ones, zeros)
    assert tp["D_ascending"] == pytest.approx(r["maxD"], rel=1e-12)


def test_labelling_and_ties():
    # lower group has the greater magnitude -> alpha is the lower mean, K = i*
    w = np.array([-1.0, -0.9, 0.1, 0.0, 0.05, 0.1], dtype=np.float32)
    r = est.estimate_filter(w)
    assert r["alpha_is_upper"] == 0 and r["K"] == 2 and r["alpha"] < 0
    assert r["e"].tolist() == [1, 1, 0, 0, 0, 0]
    # equal magnitudes -> the upper group is alpha
    r = est.estimate_filter(np.array([-1.0, 1.0], dtype=np.float32))
    assert (r["alpha"], r["beta"], r["K"], r["alpha_is_upper"]) == (1.0, -1.0, 1, 1)
    assert r["e"].tolist() == [0, 1] and (r["thr_val"], r["thr_idx"]) == (-1.0, 0)


def test_duplicates_zeros_and_constant_filter():
    # constant filter: D is flat, the largest i wins, alpha = beta = the constant
    r = est.estimate_filter(np.full(7, 0.25, dtype=np.float32))
    assert r["i_star"] == 6 and r["alpha"] == 0.25 and r["beta"] == 0.25
    assert r["thr_idx"] == 5 and r["e"].tolist() == [0, 0, 0, 0, 0, 0, 1]
    # duplicates across the split are separated by original index (stable rank)
    w = np.array([0.0, 1.0, 1.0, -0.0, 1.0, 0.0], dtype=np.float32)
    order = est.stable_order(w)
    assert order.tolist() == [0, 3, 5, 1, 2, 4]      # -0.0 ties with +0.0
    for i_split in range(1, 6):
        low = np.zeros(6, bool)
        low[order[:i_split]] = True
        last = order[i_split - 1]
        assert np.array_equal(est.lower_group_from_descriptor(w, w[last], last), low)
    r = est.estimate_filter(w)
    assert r["i_star"] == 3 and r["e"].tolist() == [0, 1, 1, 0, 1, 0]
    assert np.array_equal(est.mask_from_descriptor(w, r["thr_val"], r["thr_idx"], r["alpha_is_upper"]), r["e"])


@pytest.mark.parametrize("seed", range(4))
def test_descriptor_rebuilds_mask(seed):
    rng = np.random.default_rng(seed)
    w = np.round(rng.standard_normal(500) * 4).astype(np.float32) / 8      # heavy duplication
    r = est.estimate_filter(w)
    assert np.array_equal(est.mask_from_descriptor(w, r["thr_val"], r["thr_idx"], r["alpha_is_upper"]), r["e"])


def test_batched_layer_and_errors():
    rng = np.random.default_rng(1)
    W = rng.standard_normal((5, 3, 2, 2)).astype(np.float32)
    out = est.estimate_alpha_beta(W)
    assert out["e"].shape == W.shape
    for f in range(5):
        r = est.estimate_filter(W[f])
        assert out["K"][f] == r["K"] and out["alpha"][f] == r["alpha"] and out["beta"][f] == r["beta"]
    with pytest.raises(ValueError):
        est.estimate_filter(np.array([1.0], dtype=np.float32))


# ------------------------------------------------------------------ the sign-split baseline
def test_sign_split_is_the_best_scaled_sign_vector_by_brute_force():
    """XNOR-Net's choice (the special case Section 4.1 names): among all alpha * b with b in {+1,-1}^n the
    least-squares optimum is b = sign(w), alpha = mean |w|.  Checked over every b for small n."""
    import itertools
    rng = np.random.default_rng(12)
    for n in (3, 6, 9):
        w = rng.standard_normal(n)
        r = est.estimate_sign_split(w[None, :])
        mine = np.sum((w - est.reconstruct(r["e"][0], r["alpha"][0], r["beta"][0])) ** 2)
        best = min(np.sum((w - (np.dot(w, b) / n) * np.array(b)) ** 2)
                   for b in itertools.product((1.0, -1.0), repeat=n))
        assert mine == pytest.approx(best, rel=1e-12)
        # and alpha is the minimiser for that sign vector
        b = np.where(w >= 0, 1.0, -1.0)
        for da in (-1e-3, 1e-3):
            assert np.sum((w - (r["alpha"][0] + da) * b) ** 2) > mine


def test_sign_split_descriptor_rebuilds_the_mask():
    rng = np.random.default_rng(13)
    rows = [rng.standard_normal(40), np.abs(rng.standard_normal(40)), -np.abs(rng.standard_normal(40)) - 0.1,
            np.array([0.0, -0.0, 1.0, -1.0, -1.0, 2.0, -3.0, -1.0]),            # zeros count as +, tied largest negative
            np.round(rng.standard_normal(64) * 2) / 2]
    for w in rows:
        r = est.estimate_sign_split(w[None, :].astype(np.float32))
        e = est.mask_from_descriptor(w.astype(np.float32), r["thr_val"][0], r["thr_idx"][0], r["alpha_is_upper"][0])
        assert np.array_equal(e, (w >= 0).astype(np.uint8))
        assert r["K"][0] == int((w >= 0).sum())
        assert r["alpha"][0] == pytest.approx(np.abs(w.astype(np.float32).astype(np.float64)).mean(), rel=1e-15)
        assert r["beta"][0] == -r["alpha"][0]


def test_distribution_aware_error_never_exceeds_the_sign_split_error():
    """Section 4.1: the optimal (alpha, beta, e) can only improve on the distribution-agnostic choice."""
    rng = np.random.default_rng(14)
    for _ in range(20):
        w = (rng.standard_normal(200) * rng.uniform(0.01, 1) + rng.uniform(-0.5, 0.5)).astype(np.float32)
        d = est.estimate_filter(w)
        x = est.estimate_sign_split(w[None, :])
        w64 = w.astype(np.float64)
        e_dab = np.sum((w64 - est.reconstruct(d["e"], d["alpha"], d["beta"])) ** 2)
        e_xnor = np.sum((w64 - est.reconstruct(x["e"][0], x["alpha"][0], x["beta"][0])) ** 2)
        assert e_dab <= e_xnor * (1 + 1e-12)


# ------------------------------------------------------------------ restricted search (bounded change of K)
def _error_of_split(w, i):
    """||W - W~||^2 of the split 'i smallest | rest' with the two group means, from the definition."""
    ws = np.sort(np.asarray(w, dtype=np.float64), kind="stable")
    lo, hi = ws[:i], ws[i:]
    return float(((lo - lo.mean()) ** 2).sum() + ((hi - hi.mean()) ** 2).sum())


def test_bounded_search_with_a_wide_window_is_the_plain_estimate():
    rng = np.random.default_rng(31)
    for n in (2, 3, 17, 200):
        w = rng.standard_normal(n)
        full = est.estimate_filter(w)
        for kp, up in ((1, 0), (n - 1, 1), (n // 2 + 1, 0)):
            got = est.estimate_filter_bounded(w, min(kp, n - 1), up, n)
            assert got["i_star"] == full["i_star"] and got["alpha"] == full["alpha"] and got["K"] == full["K"]
            assert np.array_equal(got["e"], full["e"])


def test_bounded_search_minimises_the_error_inside_the_window():
    rng = np.random.default_rng(32)
    for trial in range(30):
        n = int(rng.integers(5, 80))
        w = rng.standard_normal(n) + (rng.random(n) < 0.3) * 2.0
        K_prev = int(rng.integers(1, n))
        up = int(rng.integers(0, 2))
        d = int(rng.integers(0, 6))
        i_prev = n - K_prev if up else K_prev
        lo, hi = max(1, i_prev - d), min(n - 1, i_prev + d)
        assert est.split_window(n, K_prev, up, d) == (lo, hi)
        errs = {i: _error_of_split(w, i) for i in range(lo, hi + 1)}
        best = min(errs, key=lambda i: (errs[i], -i))
        got = est.estimate_filter_bounded(w, K_prev, up, d)
        assert lo <= got["i_star"] <= hi
        assert errs[got["i_star"]] <= errs[best] * (1 + 1e-12) + 1e-15
        # no split inside the window does better; one outside may
        full = est.estimate_filter(w)
        assert _error_of_split(w, full["i_star"]) <= errs[got["i_star"]] + 1e-12
        # means and labelling follow the chosen partition
        a, b = est.group_means(w, got["e"].astype(np.float64))
        assert got["alpha"] == pytest.approx(a, rel=1e-13) and got["beta"] == pytest.approx(b, rel=1e-13)
        assert abs(got["alpha"]) >= abs(got["beta"])
        assert got["K"] == int(got["e"].sum())


def test_bounded_search_with_no_room_keeps_the_previous_partition():
    rng = np.random.default_rng(33)
    w = rng.standard_normal(40)
    for K_prev, up in ((7, 0), (7, 1), (39, 0), (1, 1)):
        got = est.estimate_filter_bounded(w, K_prev, up, 0)
        i_prev = 40 - K_prev if up else K_prev
        assert got["i_star"] == i_prev
        order = np.argsort(w, kind="stable")
        low = np.zeros(40, dtype=bool)
        low[order[:i_prev]] = True
        assert np.array_equal(est.lower_group_from_descriptor(w, got["thr_val"], got["thr_idx"]), low)
    # a previous K outside 1 .. n-1 is pulled back inside
    assert est.split_window(40, 0, 0, 3) == (1, 4)
    assert est.split_window(40, 55, 0, 3) == (36, 39)
    assert est.split_window(40, 5, 1, 10 ** 9) == (1, 39)
