"""Oracle (test infrastructure): the binarized layer, evaluated directly.

Written from the paper (arXiv 1804.02941): Section 4 (inputs of a binarized
layer take the values +1 / -1), Section 4.3.2 (the forward pass is the ordinary
convolution of the binary input with the two-valued filter W~ of Corollary 1),
Section 5.1 (no bias on binarized layers) and the appendix note that the fully
binarized block has the structure of XNOR-Net's.

Everything here works on UNPACKED values in float64 (or exact integers) and is
written as the definition: a sum over taps and channels of input times weight.

Readings taken where the text is silent:

* sign(0) = +1: a = +1 iff x >= tau (so -0.0 gives +1 and NaN gives -1); tau
  is an optional per-channel threshold (0 when absent), which is what a
  positive-scale batch normalisation followed by sign amounts to.
* Zero padding is applied to the already binarized tensor: a padded tap
  contributes 0, it is neither +1 nor -1.
* The layer is a cross-correlation (no kernel flip), no bias, no activation
  scaling factor: y = sum_i a_i * w~_i.

* WBin (Section 5.1: only the weights binarized): the same layer applied to the
  real-valued input, nothing else changed (``weights_only_layer``).

Layouts: activations are NCHW here (the conventional statement of the
problem); outputs are returned as [B, Ho, Wo, F].
"""
from __future__ import annotations

import numpy as np


def binarize_activations(x: np.ndarray, tau=None) -> np.ndarray:
    """a = +1 where x >= tau_c else -1; x is [B, C, H, W] or [B, C].  int8 result."""
    x = np.asarray(x)
    if tau is None:
        t = 0.0
    else:
        t = np.asarray(tau, dtype=x.dtype).reshape((1, -1) + (1,) * (x.ndim - 2))
    return np.where(x >= t, 1, -1).astype(np.int8)


def two_valued_filters(e: np.ndarray, alpha, beta) -> np.ndarray:
    """W~_f = alpha_f * e_f + beta_f * (1 - e_f) for every filter (Corollary 1).

    e is [F, ...] of 0/1; alpha, beta are [F].  float64 result of e's shape.
    """
    e = np.asarray(e, dtype=np.float64)
    shp = (-1,) + (1,) * (e.ndim - 1)
    a = np.asarray(alpha, dtype=np.float64).reshape(shp)
    b = np.asarray(beta, dtype=np.float64).reshape(shp)
    return a * e + b * (1.0 - e)


def out_size(H, k, pad, stride):
    return (H + 2 * pad - k) // stride + 1


def _padded(a, pad_h, pad_w, dtype):
    a = np.asarray(a).astype(dtype)
    return np.pad(a, ((0, 0), (0, 0), (pad_h, pad_h), (pad_w, pad_w)))


def conv2d(a, Wt, pad=(0, 0), stride=(1, 1), dtype=np.float64) -> np.ndarray:
    """y[b,oy,ox,f] = sum_{c,ky,kx} a[b,c,oy*s-p+ky,ox*s-p+kx] * Wt[f,c,ky,kx].

    Section 4.3.2's forward product.  a is [B,C,H,W] (values +1/-1), Wt is
    [F,C,kh,kw]; taps that fall outside the image contribute zero.  One
    channel-contraction (a library matmul) per tap, summed over the taps.
    With dtype=np.int64 and integer operands the result is exact.
    """
    Wt = np.asarray(Wt).astype(dtype)
    F, C, kh, kw = Wt.shape
    ph, pw = pad
    sh, sw = stride
    ap = _padded(a, ph, pw, dtype)
    B, _, Hp, Wp = ap.shape
    Ho = (Hp - kh) // sh + 1
    Wo = (Wp - kw) // sw + 1
    y = np.zeros((B, Ho, Wo, F), dtype=dtype)
    for ky in range(kh):
        for kx in range(kw):
            win = ap[:, :, ky:ky + sh * (Ho - 1) + 1:sh, kx:kx + sw * (Wo - 1) + 1:sw]
            y += np.einsum("bchw,fc->bhwf", win, Wt[:, :, ky, kx], optimize=True)
    return y


def conv2d_at(a, Wt, pad, stride, points) -> np.ndarray:
    """The same sum for selected outputs only; points is a list of (b,oy,ox,f).

    Plain loops over the window, so that single outputs of a large layer can
    be checked one by one.
    """
    a = np.asarray(a)
    Wt = np.asarray(Wt, dtype=np.float64)
    _, C, H, W = a.shape
    _, _, kh, kw = Wt.shape
    ph, pw = pad
    sh, sw = stride
    out = np.zeros(len(points), dtype=np.float64)
    for j, (b, oy, ox, f) in enumerate(points):
        acc = 0.0
        for ky in range(kh):
            iy = oy * sh - ph + ky
            if iy < 0 or iy >= H:
                continue
            for kx in range(kw):
                ix = ox * sw - pw + kx
                if ix < 0 or ix >= W:
                    continue
                acc += float(np.dot(a[b, :, iy, ix].astype(np.float64), Wt[f, :, ky, kx]))
        out[j] = acc
    return out


def fc(a, Wt, dtype=np.float64) -> np.ndarray:
    """y[b,f] = sum_k a[b,k] * Wt[f,k]  (the 1x1-spatial case of the layer)."""
    return np.asarray(a).astype(dtype) @ np.asarray(Wt).astype(dtype).T


def integer_terms(a, e, pad=(0, 0), stride=(1, 1)):
    """Exact integers behind one layer output, from the unpacked values.

    s1[b,oy,ox,f] = sum_i a_i e_i, sA[b,oy,ox] = sum_i a_i (both over the taps
    inside the image).  Since W~ = alpha e + beta (1-e) (Section 4.1),
    y = alpha*s1 + beta*(sA - s1).  a is [B,C,H,W] or [B,K]; e is [F,C,kh,kw]
    or [F,K].
    """
    a = np.asarray(a)
    e = np.asarray(e)
    if a.ndim == 2:
        s1 = fc(a, e, dtype=np.int64)
        sA = a.astype(np.int64).sum(axis=1)
        return s1, sA
    s1 = conv2d(a, e, pad, stride, dtype=np.int64)
    ones = np.ones((1,) + e.shape[1:], dtype=np.int64)
    sA = conv2d(a, ones, pad, stride, dtype=np.int64)[..., 0]
    return s1, sA


def layer_from_integer_terms(s1, sA, alpha, beta) -> np.ndarray:
    """y = alpha_f * s1 + beta_f * s2 with s2 = sA - s1, in float64."""
    s1 = np.asarray(s1, dtype=np.float64)
    s2 = np.asarray(sA, dtype=np.float64)[..., None] - s1
    return np.asarray(alpha, dtype=np.float64) * s1 + np.asarray(beta, dtype=np.float64) * s2


def magnitude_bound(s1, sA, alpha, beta) -> np.ndarray:
    """|alpha_f|*|s1| + |beta_f|*|s2|: the scale a two-term fp32 sum is accurate to."""
    s1 = np.asarray(s1, dtype=np.float64)
    s2 = np.asarray(sA, dtype=np.float64)[..., None] - s1
    return np.abs(np.asarray(alpha, dtype=np.float64)) * np.abs(s1) + \
        np.abs(np.asarray(beta, dtype=np.float64)) * np.abs(s2)


def popcount_terms_1d(a_pm1, e01):
    """The popcount form of one dot product, from bit vectors.

    With A = [a == +1] and E = e as bits over the n valid positions:
    sum a_i e_i = 2*popc(A & E) - popc(E) and
    sum a_i (1-e_i) = 2*(popc(A) - popc(A & E)) - (n - popc(E)).
    Follows from a_i = 2*A_i - 1 and W~ = alpha e + beta (1-e) (Section 4.1).
    Returns (s1, s2, popc(A&E), popc(A), popc(E)).
    """
    A = np.asarray(a_pm1).ravel() > 0
    E = np.asarray(e01).ravel() > 0
    n = A.size
    pAE = int(np.count_nonzero(A & E))
    pA = int(np.count_nonzero(A))
    pE = int(np.count_nonzero(E))
    return 2 * pAE - pE, 2 * (pA - pAE) - (n - pE), pAE, pA, pE


# --------------------------------------------------------------------------
# Between two binarized layers (Section 4: the next layer's inputs are again
# +1 / -1; the Sketch-A-Net architecture that Section 5.1 trains, taken from the
# work it cites, max-pools 3x3 / stride 2 between binarized layers).  Written as the definition: pool the real-valued
# output, then take the sign.
# --------------------------------------------------------------------------

def max_pool(y: np.ndarray, kh: int, kw: int, sh: int, sw: int) -> np.ndarray:
    """Max over kh x kw windows inside the image; y is [B, H, W, F], result [B, Ho, Wo, F]."""
    y = np.asarray(y)
    B, H, W, F = y.shape
    Ho, Wo = (H - kh) // sh + 1, (W - kw) // sw + 1
    out = np.full((B, Ho, Wo, F), -np.inf, dtype=y.dtype)
    for ky in range(kh):
        for kx in range(kw):
            out = np.maximum(out, y[:, ky:ky + (Ho - 1) * sh + 1:sh, kx:kx + (Wo - 1) * sw + 1:sw, :])
    return out


def next_layer_input(y: np.ndarray, tau=None, pool=None) -> np.ndarray:
    """The +1/-1 input of the following binarized layer from this layer's output y [B, Ho, Wo, F].

    pool = (kh, kw, sh, sw) or None.  Result is NCHW int8, as binarize_activations returns it.
    """
    if pool is not None:
        y = max_pool(y, *pool)
    return binarize_activations(np.transpose(np.asarray(y), (0, 3, 1, 2)), tau)


def weights_only_layer(x, e, alpha, beta, pad=(0, 0), stride=(1, 1)) -> np.ndarray:
    """The WBin variant of Section 5.1: only the weights are binarized, the input keeps its real values.

    y = x (*) W~ with W~ = alpha e + beta (1-e) (Section 4.1, 4.3.2), zero padding, no bias.
    x is [B,C,H,W] (or [B,K] with e [F,K]); returns [B,Ho,Wo,F] (or [B,F]) in float64.
    """
    Wt = two_valued_filters(e, alpha, beta)
    x = np.asarray(x, dtype=np.float64)
    if x.ndim == 2:
        return fc(x, Wt)
    return conv2d(x, Wt, pad, stride)


def weights_only_magnitude(x, e, alpha, beta, pad=(0, 0), stride=(1, 1)) -> np.ndarray:
    """sum_i |x_i| |w~_i| per output: the scale a floating-point evaluation of the layer is accurate to."""
    return weights_only_layer(np.abs(np.asarray(x, dtype=np.float64)), e, np.abs(np.asarray(alpha, dtype=np.float64)),
                              np.abs(np.asarray(beta, dtype=np.float64)), pad, stride)
