"""Oracle (test infrastructure): the weight-side steps of one training iteration.

Written from the paper (arXiv 1804.02941): Algorithm 2 (mean-centre and clamp
the real weights, binarize every filter, form W~) and Theorem 4 with the
gradient derivation in the appendix (G~ = G~1 + G~2).  Float64, plain numpy,
one filter at a time.  Only tests, the smoke check and the benchmark's CPU
baseline may import this module; the library never does.

Readings taken where the text is silent or inconsistent (each is restated in
the design notes of the repository):

* MeanCenter.  Algorithm 2 names the step but not its axis.  Two conventions
  are provided: "filter" subtracts from every filter the mean of its n = c*w*h
  weights (the unit Theorem 2 and Algorithm 1 work on), "channel" subtracts,
  for every filter and every spatial tap, the mean over the input channels.
  Clamp follows MeanCenter, in the order Algorithm 2 lists them.
* In Theorem 4 and its derivation sgn(T_k) stands for the mask e (the
  derivation substitutes e = sgn(T_k)) and sgn(W - T_k) for 1 - e: the
  derivative of alpha = W^T e / K with respect to W, e held fixed, is e / K.
  Both are taken as the 0/1 masks, not as signs of the kept values.
* T_k = topk(W, K) is the n-vector that keeps the entries of the alpha group
  and is zero elsewhere; W - T_k keeps the entries of the beta group.
* STE(V)^i is V^i where |W^i| <= 1 and 0 elsewhere, as the theorem prints it
  (the value, not an indicator).
* The scalars in front of the STE terms are the printed l1 norms
  ||T_k||_1 / K and ||W - T_k||_1 / (n - K), not alpha and beta (they agree in
  magnitude when each group holds one sign only).
* The theorem gives the local factor G~ = dW~/dW in element-wise form.  The
  gradient applied to the real weights is taken as the element-wise product
  of the upstream gradient dC/dW~ with G~.
"""
from __future__ import annotations

import numpy as np


def mean_center(W: np.ndarray, axis: str = "filter") -> np.ndarray:
    """MeanCenter of Algorithm 2 on weights W[F][C][kh][kw]."""
    W = np.asarray(W, dtype=np.float64)
    if W.ndim != 4:
        raise ValueError("W must be [F][C][kh][kw]")
    if axis == "filter":
        return W - W.mean(axis=(1, 2, 3), keepdims=True)
    if axis == "channel":
        return W - W.mean(axis=1, keepdims=True)
    raise ValueError("axis must be 'filter' or 'channel'")


def clamp(W: np.ndarray, lo: float = -1.0, hi: float = 1.0) -> np.ndarray:
    """Clamp of Algorithm 2."""
    return np.minimum(np.maximum(np.asarray(W, dtype=np.float64), lo), hi)


def mean_center_clamp(W: np.ndarray, axis: str = "filter", lo: float = -1.0, hi: float = 1.0) -> np.ndarray:
    """The two pre-steps of Algorithm 2 in the order it lists them."""
    return clamp(mean_center(W, axis), lo, hi)


def binarized_filter(e: np.ndarray, alpha: float, beta: float) -> np.ndarray:
    """W~ of one filter as Algorithm 2 forms it: alpha on the mask, beta off it."""
    e = np.asarray(e, dtype=np.float64)
    return alpha * e + beta * (1.0 - e)


def gradient_terms(w: np.ndarray, e: np.ndarray):
    """Theorem 4 for one filter: (G~1, G~2) as n-vectors.

    w is the (mean-centred, clamped) real filter, e its 0/1 mask with K ones,
    0 < K < n.
    """
    w = np.asarray(w, dtype=np.float64).ravel()
    e = np.asarray(e, dtype=np.float64).ravel()
    n = w.size
    K = int(e.sum())
    if not 0 < K < n:
        raise ValueError("the mask must be neither empty nor full")
    inside = (np.abs(w) <= 1.0).astype(np.float64)
    T_k = w * e                       # topk(W, K): the alpha group's entries, zero elsewhere
    rest = w - T_k                    # the beta group's entries
    ste_T = T_k * inside
    ste_rest = rest * inside
    G1 = (e / K) * e + (np.abs(T_k).sum() / K) * ste_T
    G2 = ((1.0 - e) / (n - K)) * (1.0 - e) + (np.abs(rest).sum() / (n - K)) * ste_rest
    return G1, G2


def gradient_factor(w: np.ndarray, e: np.ndarray) -> np.ndarray:
    """G~ = G~1 + G~2 of Theorem 4 for one filter."""
    G1, G2 = gradient_terms(w, e)
    return G1 + G2


def weight_gradient(W: np.ndarray, E: np.ndarray, upstream=None) -> np.ndarray:
    """Rows of W[F][n] and masks E[F][n] -> dC/dW[F][n] = upstream * G~ (G~ itself without upstream)."""
    W = np.asarray(W, dtype=np.float64)
    E = np.asarray(E)
    out = np.empty_like(W)
    for f in range(W.shape[0]):
        out[f] = gradient_factor(W[f], E[f])
    if upstream is not None:
        out = out * np.asarray(upstream, dtype=np.float64)
    return out
