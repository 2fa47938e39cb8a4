"""Pins of the layer oracle (CPU only): library convolution, closed forms, the popcount identity."""
import json
import os
from fractions import Fraction

import numpy as np
import pytest
import torch
import torch.nn.functional as Fn

from oracle import estimate as est
from oracle import layers as lay
from oracle import packing as pk


def rand_pm1(rng, shape):
    return np.where(rng.random(shape) < 0.5, 1, -1).astype(np.int8)


@pytest.mark.parametrize("C,H,W,F,kh,kw,pad,stride", [
    (3, 6, 7, 4, 3, 3, (1, 1), (1, 1)),
    (5, 9, 8, 3, 5, 5, (0, 0), (1, 1)),
    (4, 11, 10, 2, 3, 5, (2, 1), (2, 3)),
    (2, 7, 7, 6, 7, 7, (0, 0), (1, 1)),
    (8, 5, 5, 3, 1, 1, (0, 0), (1, 1)),
])
def test_conv_matches_library_cross_correlation(C, H, W, F, kh, kw, pad, stride):
    """The layer is the ordinary (PyTorch) cross-correlation with zero padding."""
    rng = np.random.default_rng(C * 100 + H)
    a = rand_pm1(rng, (2, C, H, W))
    Wt = rng.standard_normal((F, C, kh, kw))
    ref = Fn.conv2d(torch.from_numpy(a.astype(np.float64)), torch.from_numpy(Wt), stride=stride, padding=pad)
    ref = ref.permute(0, 2, 3, 1).numpy()
    y = lay.conv2d(a, Wt, pad, stride)
    assert y.shape == ref.shape
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-12)
    pts = [(b, oy, ox, f) for b in range(2) for oy in (0, y.shape[1] - 1) for ox in (0, y.shape[2] // 2) for f in (0, F - 1)]
    got = lay.conv2d_at(a, Wt, pad, stride, pts)
    assert np.allclose(got, [ref[p] for p in pts], rtol=1e-12, atol=1e-12)


def test_fc_is_matmul():
    rng = np.random.default_rng(2)
    a = rand_pm1(rng, (5, 70))
    Wt = rng.standard_normal((9, 70))
    assert np.allclose(lay.fc(a, Wt), a.astype(np.float64) @ Wt.T)
    a4 = a[:, :, None, None]
    assert np.allclose(lay.conv2d(a4, Wt[:, :, None, None])[:, 0, 0, :], lay.fc(a, Wt))


def test_binarize_edge_cases():
    x = np.array([[0.0, -0.0, 1e-30, -1e-30, np.nan, np.inf, -np.inf, 2.0]], dtype=np.float32)
    assert lay.binarize_activations(x).tolist() == [[1, 1, 1, -1, -1, 1, -1, 1]]
    tau = np.array([0, 0, 1, -1, 0, 0, 0, 2.0], dtype=np.float32)
    assert lay.binarize_activations(x, tau).tolist() == [[1, 1, -1, 1, -1, 1, -1, 1]]
    x4 = np.zeros((1, 2, 2, 2), dtype=np.float32)
    x4[0, 1] = 0.5
    assert lay.binarize_activations(x4, np.array([0.0, 1.0], np.float32))[0, :, 0, 0].tolist() == [1, -1]


def test_all_plus_one_input_returns_filter_sum():
    """With a = +1 everywhere and no padding y = sum_i w~_i = K alpha + (n-K) beta = sum_i w_i."""
    rng = np.random.default_rng(9)
    W = (rng.standard_normal((6, 4, 3, 3)) * 0.05 + 0.01).astype(np.float32)
    r = est.estimate_alpha_beta(W)
    Wt = lay.two_valued_filters(r["e"], r["alpha"], r["beta"])
    a = np.ones((2, 4, 8, 8), dtype=np.int8)
    y = lay.conv2d(a, Wt)
    T = W.astype(np.float64).reshape(6, -1).sum(axis=1)
    assert np.allclose(y, np.broadcast_to(T, y.shape), rtol=1e-12, atol=1e-14)
    # with padding the corner output only sees the taps inside the image
    yp = lay.conv2d(a, Wt, pad=(1, 1))
    corner = Wt[:, :, 1:, 1:].reshape(6, -1).sum(axis=1)
    assert np.allclose(yp[0, 0, 0], corner, rtol=1e-12, atol=1e-14)
    s1, sA = lay.integer_terms(a, r["e"], pad=(1, 1))
    assert sA[0, 0, 0] == 4 * 4 and sA[0, 0, 3] == 4 * 6 and sA[0, 3, 3] == 4 * 9
    assert np.array_equal(s1[0, 3, 3], r["K"])


@pytest.mark.parametrize("pad,stride", [((0, 0), (1, 1)), ((1, 1), (1, 1)), ((2, 2), (2, 2))])
def test_two_term_decomposition(pad, stride):
    """y = alpha*s1 + beta*s2 with the exact integer sums equals the direct float64 layer."""
    rng = np.random.default_rng(13)
    W = (rng.laplace(0.004, 0.03, (7, 37, 3, 3))).astype(np.float32)
    r = est.estimate_alpha_beta(W)
    Wt = lay.two_valued_filters(r["e"], r["alpha"], r["beta"])
    a = rand_pm1(rng, (2, 37, 6, 5))
    y = lay.conv2d(a, Wt, pad, stride)
    s1, sA = lay.integer_terms(a, r["e"], pad, stride)
    y2 = lay.layer_from_integer_terms(s1, sA, r["alpha"], r["beta"])
    # the direct sum rounds at the scale of sum_i |w~_i|; the two-term form at |alpha s1| + |beta s2|
    scale = np.abs(Wt).reshape(7, -1).sum(axis=1)
    assert np.all(np.abs(y - y2) <= 1e-14 * scale)
    assert np.all(lay.magnitude_bound(s1, sA, r["alpha"], r["beta"]) <= scale * (1 + 1e-12))
    # popcount form, bit vectors over the valid window, checked output by output
    ph, pw = pad
    for (b, oy, ox, f) in [(0, 0, 0, 0), (1, y.shape[1] - 1, y.shape[2] - 1, 6), (0, 1, 1, 3)]:
        av, ev = [], []
        for c in range(37):
            for ky in range(3):
                for kx in range(3):
                    iy, ix = oy * stride[0] - ph + ky, ox * stride[1] - pw + kx
                    if 0 <= iy < 6 and 0 <= ix < 5:
                        av.append(a[b, c, iy, ix])
                        ev.append(r["e"][f, c, ky, kx])
        t1, t2, pAE, pA, pE = lay.popcount_terms_1d(av, ev)
        assert t1 == s1[b, oy, ox, f] and t2 == sA[b, oy, ox] - s1[b, oy, ox, f]
        assert t1 == sum(int(x) * int(e) for x, e in zip(av, ev))
        assert t2 == sum(int(x) * (1 - int(e)) for x, e in zip(av, ev))


def test_hand_example(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "alg1_worked_example.json")))
    a = np.array(g["a"], dtype=np.int8)
    e = np.array(g["e"], dtype=np.uint8)
    s1, s2, pAE, pA, pE = lay.popcount_terms_1d(a, e)
    assert (pA, pAE, s1, s2) == (g["popc_A"], g["popc_A_and_E"], g["s1"], g["s2"])
    alpha, beta = float(Fraction(g["alpha"])), float(Fraction(g["beta"]))
    Wt = lay.two_valued_filters(e[None, :], [alpha], [beta])
    assert lay.fc(a[None, :], Wt)[0, 0] == float(Fraction(g["y"]))
    i1, iA = lay.integer_terms(a[None, :], e[None, :])
    assert i1[0, 0] == g["s1"] and iA[0] - i1[0, 0] == g["s2"]
    # through the packed words as well
    A = pk.pack_activations(a[None, :])
    E, ecnt = pk.pack_weights(e[None, :])
    assert int(pk.popcount32(A[0] & E[:, 0]).sum()) == g["popc_A_and_E"]
    assert int(pk.popcount32(A[0]).sum()) == g["popc_A"] and ecnt[0, 0] == g["K"]


def test_xnor_special_case():
    """alpha = -beta: y = alpha * (2*popc(XNOR(A,E)) - n), XNOR-Net's product (Section 4.1)."""
    rng = np.random.default_rng(21)
    n = 200
    e = (rng.random((3, n)) < 0.5).astype(np.uint8)
    a = rand_pm1(rng, (4, n))
    alpha = np.array([0.3, 0.05, 1.5])
    y = lay.fc(a, lay.two_valued_filters(e, alpha, -alpha))
    A = a > 0
    for b in range(4):
        for f in range(3):
            xnor = np.count_nonzero(~(A[b] ^ (e[f] > 0)))
            assert y[b, f] == pytest.approx(alpha[f] * (2 * xnor - n), rel=1e-12)


def test_packed_words_reproduce_integer_terms():
    """popc over packed words with zero bits at padded taps gives s1, and pA gives sA."""
    rng = np.random.default_rng(33)
    C, H, W_, F = 70, 5, 6, 5
    a = rand_pm1(rng, (2, C, H, W_))
    e = (rng.random((F, C, 3, 3)) < 0.4).astype(np.uint8)
    A = pk.pack_activations(a)
    E, ecnt = pk.pack_weights(e)
    Cw = pk.words_per_pixel(C)
    s1, sA = lay.integer_terms(a, e, pad=(1, 1))
    for (b, oy, ox, f) in [(0, 0, 0, 0), (1, 4, 5, 4), (0, 2, 3, 2), (1, 0, 5, 1)]:
        p1 = pA = c1 = m = 0
        for ky in range(3):
            for kx in range(3):
                iy, ix = oy - 1 + ky, ox - 1 + kx
                if not (0 <= iy < H and 0 <= ix < W_):
                    continue
                tap = ky * 3 + kx
                words = A[b, iy, ix]
                p1 += int(pk.popcount32(words & E[tap * Cw:(tap + 1) * Cw, f]).sum())
                pA += int(pk.popcount32(words).sum())
                c1 += int(ecnt[f, tap])
                m += C
        assert 2 * p1 - c1 == s1[b, oy, ox, f]
        assert 2 * pA - m == sA[b, oy, ox]


# ------------------------------------------------------------------ WBin (weights-only binarized layer)
def test_weights_only_layer_against_library_and_two_term_form():
    """Section 5.1's WBin: real input, two-valued filters.  Checked against a library cross-correlation
    and against beta * sum(x) + (alpha - beta) * sum over the mask, brute force, on a small case."""
    rng = np.random.default_rng(61)
    B, C, H, W, F, kh, kw = 2, 5, 7, 6, 4, 3, 2
    x = rng.standard_normal((B, C, H, W))
    e = (rng.random((F, C, kh, kw)) < 0.4).astype(np.uint8)
    alpha, beta = rng.standard_normal(F), rng.standard_normal(F) * 0.3
    for pad, stride in (((0, 0), (1, 1)), ((1, 1), (1, 1)), ((2, 1), (2, 1))):
        got = lay.weights_only_layer(x, e, alpha, beta, pad, stride)
        Wt = np.where(e == 1, alpha[:, None, None, None], beta[:, None, None, None])
        ref = torch.nn.functional.conv2d(torch.from_numpy(x), torch.from_numpy(Wt), padding=pad, stride=stride)
        assert np.allclose(got, ref.permute(0, 2, 3, 1).numpy(), rtol=1e-12, atol=1e-12)
        xp = np.pad(x, ((0, 0), (0, 0), (pad[0], pad[0]), (pad[1], pad[1])))
        Bo, Ho, Wo, _ = got.shape
        for b in range(B):
            for oy in range(Ho):
                for ox in range(Wo):
                    win = xp[b, :, oy * stride[0]:oy * stride[0] + kh, ox * stride[1]:ox * stride[1] + kw]
                    for f in range(F):
                        two = beta[f] * win.sum() + (alpha[f] - beta[f]) * win[e[f] == 1].sum()
                        assert got[b, oy, ox, f] == pytest.approx(two, rel=1e-11, abs=1e-12)
        mag = lay.weights_only_magnitude(x, e, alpha, beta, pad, stride)
        assert np.all(mag >= np.abs(got) - 1e-12)
    # fully connected form, and +1/-1 inputs reduce to the binarized layer
    xf = rng.standard_normal((3, 11))
    ef = (rng.random((4, 11)) < 0.5).astype(np.uint8)
    assert np.allclose(lay.weights_only_layer(xf, ef, alpha, beta),
                       xf @ np.where(ef == 1, alpha[:, None], beta[:, None]).T, rtol=1e-13)
    a = np.where(x >= 0, 1, -1).astype(np.int8)
    s1, sA = lay.integer_terms(a, e, (1, 1), (1, 1))
    assert np.allclose(lay.weights_only_layer(a, e, alpha, beta, (1, 1), (1, 1)),
                       lay.layer_from_integer_terms(s1, sA, alpha, beta), rtol=1e-12, atol=1e-12)
