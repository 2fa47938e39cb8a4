"""Oracle (test infrastructure): optimal two-value representation of a filter.

Written from the paper (arXiv 1804.02941): Section 4.1 (Theorem 2 and its
proof in the appendix), Section 4.3.1 and Algorithm 1 (finding the optimal K),
Corollary 1 (weight binarization).  Float64 throughout, serial sums, no
blocking or fusion.

Problem (Section 4.1).  A filter is a flat vector W of n = c*w*h real weights.
It is replaced by W~ = alpha*e + beta*(1-e) with e in {0,1}^n, e != 0, e != 1,
K = e^T e, so as to minimise ||W - W~||^2.  Theorem 2: for a fixed e the best
scalars are the two group means alpha = W^T e / K, beta = W^T (1-e) / (n-K);
the error is then ||W||^2 - D with D = (W^T e)^2 / K + (W^T (1-e))^2 / (n-K);
and for a fixed K the best e selects the K smallest or the K largest weights,
so the optimum is a split of the sorted vector.

Readings taken where the text is silent or inconsistent (each is restated in
the design notes of the repository):

* The split index i runs over 1 .. n-1.  Algorithm 1's loop bound reaches
  i = n, where n - i = 0; Theorem 2 excludes e = 1, so i = n is not a split.
* One ascending pass suffices: the descending pass of Algorithm 1 scores the
  same partitions (D_desc(j) = D_asc(n-j)) with the complementary labelling.
  ``two_pass_choice`` states what taking both passes yields, for the tests.
* Ties in D are resolved towards the largest i (the ">=" of Algorithm 1).
* Which group is called alpha: Section 4.1 says alpha captures the value of
  greater magnitude.  On equal magnitudes the upper group is alpha.
* beta is the plain mean of the other group (Theorem 2); the minus sign that
  Algorithm 2 prints in front of it is taken as a typo.
* "top K" means largest or smallest by signed value (Theorem 2), not by
  magnitude, and the mask is defined by stable rank (value, then original
  index), not by sgn() of the kept values, which would drop kept zeros.
* T, the sum of all weights, is taken as the last prefix sum P_n, so that
  T - P_n is exactly zero.
* The restricted search (``estimate_filter_bounded``): Section 5 only remarks
  that K should change by slight amounts between iterations; the window is
  taken on the split position (see ``split_window``).
"""
from __future__ import annotations

from fractions import Fraction

import numpy as np


def stable_order(w: np.ndarray) -> np.ndarray:
    """Indices that sort w ascending, ties by original index; -0.0 == +0.0.

    Algorithm 1, "Sort(W)".
    """
    w = np.asarray(w, dtype=np.float64) + 0.0  # -0.0 + 0.0 = +0.0
    return np.argsort(w, kind="stable")


def split_scores(w: np.ndarray):
    """Sorted order, prefix sums P_1..P_n and scores D_1..D_{n-1} of one filter.

    Algorithm 1, the loop body: P_i = P_{i-1} + W_(i),
    D_i = P_i^2 / i + (T - P_i)^2 / (n - i).  Returned D has length n-1 and
    D[i-1] is D_i.
    """
    w = np.asarray(w, dtype=np.float64).ravel()
    n = w.size
    if n < 2:
        raise ValueError("a filter needs at least two weights (e != 0 and e != 1)")
    order = stable_order(w)
    ws = w[order]
    P = np.cumsum(ws, dtype=np.float64)  # serial left-to-right running sum, in sorted order
    T = P[n - 1]
    i = np.arange(1, n, dtype=np.float64)
    Pi = P[: n - 1]
    D = Pi * Pi / i + (T - Pi) * (T - Pi) / (n - i)
    return order, P, D


def estimate_filter(w: np.ndarray) -> dict:
    """Optimal (alpha, beta, K, e) of one filter and its split descriptor.

    Theorem 2 + Algorithm 1 (ascending pass) + the labelling sentence of
    Section 4.1.  Keys of the result:

    i_star          size of the lower group (1 .. n-1), largest maximiser of D
    maxD            D at i_star
    mu_lower/upper  the two group means (float64)
    alpha, beta     float64; alpha is the mean of greater magnitude
    K               size of the alpha group
    alpha_is_upper  1 if the alpha group is the upper (larger-valued) group
    e               uint8 mask of the alpha group, in original index order
    thr_val         float64 value of the largest element of the lower group
    thr_idx         original index of that element: i is in the lower group iff
                    w_i < thr_val or (w_i == thr_val and i <= thr_idx)
    """
    return _estimate_in_window(w, 1, np.asarray(w).size - 1)


def split_window(n: int, K_prev: int, alpha_is_upper_prev: int, max_change: int):
    """Splits allowed when the previous iteration's split may move by at most max_change.

    Section 5 remarks that for natural images K must be kept from changing by
    more than slight amounts, and gives no rule.  Reading taken here: the
    partition may move by at most max_change elements, i.e. the size i of the
    lower group stays within max_change of its previous value (i_prev = K_prev
    if the alpha group was the lower one, n - K_prev otherwise), inside 1 .. n-1.
    K itself then changes by at most max_change as long as the same group stays
    the alpha group.
    """
    i_prev = n - int(K_prev) if alpha_is_upper_prev else int(K_prev)
    i_prev = min(max(i_prev, 1), n - 1)
    d = min(max(int(max_change), 0), n)
    return max(1, i_prev - d), min(n - 1, i_prev + d)


def estimate_filter_bounded(w: np.ndarray, K_prev: int, alpha_is_upper_prev: int, max_change: int) -> dict:
    """``estimate_filter`` with the split restricted to ``split_window``: the best D inside the
    window (ties towards the larger i, as everywhere), labelled by magnitude as usual."""
    n = np.asarray(w).size
    lo, hi = split_window(n, K_prev, alpha_is_upper_prev, max_change)
    return _estimate_in_window(w, lo, hi)


def _estimate_in_window(w: np.ndarray, i_lo: int, i_hi: int) -> dict:
    w = np.asarray(w, dtype=np.float64).ravel()
    n = w.size
    order, P, D = split_scores(w)
    maxD = D[i_lo - 1:i_hi].max()
    i_star = int(np.flatnonzero(D[i_lo - 1:i_hi] == maxD)[-1]) + i_lo
    T = P[n - 1]
    mu_lower = P[i_star - 1] / i_star
    mu_upper = (T - P[i_star - 1]) / (n - i_star)
    alpha_is_upper = 1 if abs(mu_upper) >= abs(mu_lower) else 0
    in_lower = np.zeros(n, dtype=bool)
    in_lower[order[:i_star]] = True
    if alpha_is_upper:
        alpha, beta, K, e = mu_upper, mu_lower, n - i_star, ~in_lower
    else:
        alpha, beta, K, e = mu_lower, mu_upper, i_star, in_lower
    last_lower = int(order[i_star - 1])
    return dict(
        n=n, i_star=i_star, maxD=float(maxD), T=float(T),
        mu_lower=float(mu_lower), mu_upper=float(mu_upper),
        alpha=float(alpha), beta=float(beta), K=int(K),
        alpha_is_upper=int(alpha_is_upper), e=e.astype(np.uint8),
        thr_val=float(w[last_lower]), thr_idx=last_lower,
    )


def estimate_alpha_beta(W: np.ndarray) -> dict:
    """All filters of a layer: W is [F, n] (any trailing shape is flattened).

    Section 4.3.1: the filters of a layer are handled together as a 2-D array;
    each row is an independent instance of ``estimate_filter``.
    """
    W = np.asarray(W)
    F = W.shape[0]
    W2 = W.reshape(F, -1)
    rows = [estimate_filter(W2[f]) for f in range(F)]
    out = {}
    for key in ("i_star", "K", "alpha_is_upper", "thr_idx"):
        out[key] = np.array([r[key] for r in rows], dtype=np.int64)
    for key in ("alpha", "beta", "maxD", "thr_val", "mu_lower", "mu_upper", "T"):
        out[key] = np.array([r[key] for r in rows], dtype=np.float64)
    out["e"] = np.stack([r["e"] for r in rows]).reshape(W.shape)
    return out


def score_of_split(w: np.ndarray, i_split: int) -> float:
    """D_i of one filter at lower-group size i_split (Algorithm 1's D_i)."""
    _, _, D = split_scores(w)
    return float(D[i_split - 1])


def lower_group_from_descriptor(w: np.ndarray, thr_val: float, thr_idx: int) -> np.ndarray:
    """Boolean mask of the lower group, rebuilt from the split descriptor."""
    w = np.asarray(w, dtype=np.float64).ravel()
    idx = np.arange(w.size)
    return (w < thr_val) | ((w == thr_val) & (idx <= thr_idx))


def mask_from_descriptor(w, thr_val, thr_idx, alpha_is_upper) -> np.ndarray:
    """Mask e of the alpha group from the split descriptor (Corollary 1's mask)."""
    low = lower_group_from_descriptor(w, thr_val, thr_idx)
    return (~low if alpha_is_upper else low).astype(np.uint8)


def reconstruct(e: np.ndarray, alpha: float, beta: float) -> np.ndarray:
    """W~ = alpha*e + beta*(1-e)  (Section 4.1; Corollary 1)."""
    e = np.asarray(e, dtype=np.float64)
    return alpha * e + beta * (1.0 - e)


def group_means(w: np.ndarray, e: np.ndarray):
    """alpha = W^T e / K, beta = W^T (1-e) / (n-K) for a given mask (Theorem 2)."""
    w = np.asarray(w, dtype=np.float64).ravel()
    e = np.asarray(e, dtype=np.float64).ravel()
    K = e.sum()
    n = w.size
    return float(w @ e / K), float(w @ (1.0 - e) / (n - K))


def two_pass_choice(w: np.ndarray) -> dict:
    """The outcome of Algorithm 1 when both of its passes are taken.

    The descending order scores the same partitions as the ascending one, read
    backwards: its split of size j is the ascending split of size n - j with
    the two groups' roles exchanged, and D is symmetric in the groups.  So the
    scores of the second pass are ``split_scores``' D reversed.  Each pass
    keeps the largest index among the maxima of its own scores, and the second
    pass replaces the first only with a strictly greater score.  Returns both
    passes' (K, D), the K that is kept and whether the second pass supplied it
    (its mask would then be the K largest weights).
    """
    _, _, D = split_scores(w)
    D_desc = D[::-1]

    def last_argmax(scores):
        return int(scores.size - 1 - np.argmax(scores[::-1]))

    k_asc, k_desc = last_argmax(D) + 1, last_argmax(D_desc) + 1
    d_asc, d_desc = float(D[k_asc - 1]), float(D_desc[k_desc - 1])
    descending = d_desc > d_asc
    return dict(K_ascending=k_asc, D_ascending=d_asc, K_descending=k_desc, D_descending=d_desc,
                K=k_desc if descending else k_asc, descending=descending)


def brute_force(w) -> dict:
    """Exact minimum of ||W - W~||^2 over every mask e != 0, e != 1.

    Exhaustive over the 2^n - 2 masks with the closed-form group means of
    Theorem 2, in exact rational arithmetic (the float inputs are converted
    exactly).  Only for n <= 16.  Returns the minimum error as a Fraction and
    the list of minimising partitions, each as a frozenset holding the two
    index sets (so a mask and its complement count once).
    """
    wq = [Fraction(float(x)) for x in np.asarray(w).ravel()]
    n = len(wq)
    if not 2 <= n <= 16:
        raise ValueError("brute force is limited to 2 <= n <= 16")
    sq = sum(x * x for x in wq)
    total = sum(wq)
    best, parts = None, []
    for bits in range(1, (1 << n) - 1):
        if bits & 1:  # the complement, which has bit 0 clear, covers this partition
            continue
        idx = [i for i in range(n) if bits >> i & 1]
        K = len(idx)
        s = sum(wq[i] for i in idx)
        err = sq - (s * s / K + (total - s) * (total - s) / (n - K))
        part = frozenset((frozenset(idx), frozenset(set(range(n)) - set(idx))))
        if best is None or err < best:
            best, parts = err, [part]
        elif err == best:
            parts.append(part)
    return dict(min_err=best, partitions=parts)


def xnor_reconstruction(w: np.ndarray) -> np.ndarray:
    """The distribution-agnostic special case of Section 4.1: mean|W| * sign(W)."""
    w = np.asarray(w, dtype=np.float64).ravel()
    return np.mean(np.abs(w)) * np.where(w >= 0, 1.0, -1.0)


def estimate_sign_split(W: np.ndarray) -> dict:
    """The XNOR-Net / binary-weight special case for every filter (Section 4.1: the distribution-
    agnostic choice e = [w >= 0], alpha = mean |w|, beta = -alpha), in the same output form as
    estimate_alpha_beta so that the same packing and layer code consumes it.

    The lower group is the negative weights; K counts the non-negative ones (0 <= K <= n).  The
    descriptor names the largest negative value and the last index holding it; a filter without
    negative weights has thr_val = -inf (nothing is below it).
    """
    W = np.asarray(W)
    F = W.shape[0]
    W2 = W.reshape(F, -1).astype(np.float64)
    n = W2.shape[1]
    alpha = np.abs(W2).mean(axis=1)
    e = (W2 >= 0).astype(np.uint8)
    K = e.sum(axis=1).astype(np.int64)
    thr_val = np.full(F, -np.inf)
    thr_idx = np.zeros(F, dtype=np.int64)
    for f in range(F):
        neg = np.flatnonzero(W2[f] < 0)
        if neg.size:
            v = W2[f, neg].max()
            thr_val[f] = v
            thr_idx[f] = np.flatnonzero(W2[f] == v).max()
    return dict(alpha=alpha, beta=-alpha, K=K, e=e.reshape(W.shape), thr_val=thr_val, thr_idx=thr_idx,
                alpha_is_upper=np.ones(F, dtype=np.uint8), n=n)


def all_partitions_of_sorted(w):
    """Helper for tests: every (lower, upper) split of the stable sorted order."""
    order = stable_order(w)
    n = len(order)
    return [(frozenset(order[:i].tolist()), frozenset(order[i:].tolist())) for i in range(1, n)]


