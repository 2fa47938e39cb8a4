"""GPU parity of the training-side weight steps (MeanCenter + Clamp, W~, Theorem 4) through the C ABI.

fp32 outputs are single roundings of double-precision values, compared with the float64 oracle to
1e-6 relative (plus the rounding of the clamp limits); W~ holds alpha or beta exactly.
"""
import numpy as np
import pytest
import torch

from oracle import estimate as oest
from oracle import training as otr
from paper_1804_02941_amd import binding as dab
from paper_1804_02941_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu

RTOL = 1e-6

# [F, C, kh, kw]: ragged rows, one tap (fully connected), more taps than threads, conv6 of the trunk
WEIGHT_SHAPES = [(5, 3, 2, 3), (16, 64, 5, 5), (7, 45, 1, 1), (3, 2, 17, 17), (33, 100, 3, 3), (12, 256, 7, 7),
                 (3, 1100, 1, 4)]
# rows longer than the estimator takes (and than the register-resident kernels): centring only
LONG_SHAPES = [(2, 4100, 2, 2)]


def weights(shape, seed):
    rng = np.random.default_rng(seed)
    F, C, kh, kw = shape
    W = wl.skewed_mixture_weights(rng, np.random.default_rng(seed + 1), F, C * kh * kw, C * kh * kw)
    W = W.reshape(shape).astype(np.float32)
    W *= np.float32(0.8 / max(np.abs(W).max(), 1e-6))                 # inside [-1, 1] with a few clamped below
    W[0].flat[0] = 1.75                                               # and some that the clamp and the STE mask cut
    W[-1].flat[-1] = -2.5
    return W


@pytest.mark.parametrize("shape", WEIGHT_SHAPES + LONG_SHAPES)
@pytest.mark.parametrize("axis", ["filter", "channel"])
def test_mean_center_clamp(shape, axis):
    W = weights(shape, 40)
    code = dab.DAB_CENTER_FILTER if axis == "filter" else dab.DAB_CENTER_CHANNEL
    for lo, hi in ((-1.0, 1.0), (-0.25, 0.5)):
        got = dab.dab_mean_center_clamp(gu.to_gpu(W), code, lo, hi).cpu().numpy()
        want = otr.mean_center_clamp(W, axis, lo, hi)
        assert got.shape == W.shape
        assert np.allclose(got, want, rtol=RTOL, atol=1e-7)
        assert got.min() >= lo and got.max() <= hi
    # in place
    t = gu.to_gpu(W)
    dab.dab_mean_center_clamp(t, code, -1.0, 1.0, out=t)
    assert np.allclose(t.cpu().numpy(), otr.mean_center_clamp(W, axis), rtol=RTOL, atol=1e-7)


@pytest.mark.parametrize("shape", WEIGHT_SHAPES)
def test_binarized_weights_and_gradient(shape):
    """Algorithm 2's weight side in order: centre + clamp, estimate, W~, Theorem 4."""
    F = shape[0]
    Wc = dab.dab_mean_center_clamp(gu.to_gpu(weights(shape, 41)))
    W2 = Wc.reshape(F, -1)
    est = dab.dab_estimate_alpha_beta(W2)
    Wt = dab.dab_binarized_weights(W2, est["alpha"], est["beta"], est["thr_val"], est["thr_idx"], est["alpha_is_upper"])
    G = dab.dab_weight_gradient(W2, est["thr_val"], est["thr_idx"], est["alpha_is_upper"])
    rng = np.random.default_rng(42)
    up = rng.standard_normal(W2.shape).astype(np.float32)
    dW = dab.dab_weight_gradient(W2, est["thr_val"], est["thr_idx"], est["alpha_is_upper"], upstream=gu.to_gpu(up))
    torch.cuda.synchronize()
    w = W2.cpu().numpy()
    est_np = {k: v.cpu().numpy() for k, v in est.items()}
    e, _ = gu.check_estimate(w, est_np)                               # masks of the GPU's (verified) splits
    # W~: alpha where e, beta elsewhere, exactly
    want_wt = np.where(e == 1, est_np["alpha"][:, None], est_np["beta"][:, None]).astype(np.float32)
    assert np.array_equal(Wt.cpu().numpy(), want_wt)
    for f in range(F):
        assert np.array_equal(want_wt[f].astype(np.float64),
                              otr.binarized_filter(e[f], float(est_np["alpha"][f]), float(est_np["beta"][f])))
    # Theorem 4
    assert np.allclose(G.cpu().numpy(), otr.weight_gradient(w, e), rtol=RTOL, atol=0)
    assert np.allclose(dW.cpu().numpy(), otr.weight_gradient(w, e, up), rtol=RTOL, atol=0)


def test_gradient_with_weights_outside_the_clamp_range():
    """The STE mask: unclamped weights with |w| > 1 keep only the mask terms."""
    rng = np.random.default_rng(43)
    w = (rng.standard_normal((9, 301)) * 1.5).astype(np.float32)
    est = dab.dab_estimate_alpha_beta(gu.to_gpu(w))
    G = dab.dab_weight_gradient(gu.to_gpu(w), est["thr_val"], est["thr_idx"], est["alpha_is_upper"])
    torch.cuda.synchronize()
    e, _ = gu.check_estimate(w, {k: v.cpu().numpy() for k, v in est.items()})
    assert (np.abs(w) > 1).sum() > 100
    assert np.allclose(G.cpu().numpy(), otr.weight_gradient(w, e), rtol=RTOL, atol=0)


def test_sign_split_descriptor_and_errors():
    """The sign-split (XNOR-Net) descriptor drives the same kernels; error paths return codes."""
    rng = np.random.default_rng(44)
    w = np.clip(rng.standard_normal((6, 130)) * 0.4, -1, 1).astype(np.float32)
    t = gu.to_gpu(w)
    est = dab.dab_estimate_sign_split(t)
    Wt = dab.dab_binarized_weights(t, est["alpha"], est["beta"], est["thr_val"], est["thr_idx"], est["alpha_is_upper"])
    G = dab.dab_weight_gradient(t, est["thr_val"], est["thr_idx"], est["alpha_is_upper"])
    torch.cuda.synchronize()
    a = est["alpha"].cpu().numpy()
    assert np.array_equal(Wt.cpu().numpy(), np.where(w >= 0, a[:, None], -a[:, None]).astype(np.float32))
    assert np.allclose(G.cpu().numpy(), otr.weight_gradient(w, (w >= 0).astype(np.uint8)), rtol=RTOL, atol=0)
    # a row longer than the register-resident kernels take
    w = np.clip(rng.standard_normal((2, 16400)) * 0.6, -1.2, 1.2).astype(np.float32)
    t2 = gu.to_gpu(w)
    est = dab.dab_estimate_sign_split(t2)
    G = dab.dab_weight_gradient(t2, est["thr_val"], est["thr_idx"], est["alpha_is_upper"])
    Wt = dab.dab_binarized_weights(t2, est["alpha"], est["beta"], est["thr_val"], est["thr_idx"], est["alpha_is_upper"])
    torch.cuda.synchronize()
    a = est["alpha"].cpu().numpy()
    assert np.array_equal(Wt.cpu().numpy(), np.where(w >= 0, a[:, None], -a[:, None]).astype(np.float32))
    assert np.allclose(G.cpu().numpy(), otr.weight_gradient(w, (w >= 0).astype(np.uint8)), rtol=RTOL, atol=0)
    lib = dab.lib()
    p = t.data_ptr()
    assert lib.dab_mean_center_clamp(p, 6, 130, 1, 2, -1.0, 1.0, p, None) == dab.DAB_ERR_UNSUPPORTED
    assert lib.dab_mean_center_clamp(p, 6, 130, 1, 0, 1.0, -1.0, p, None) == dab.DAB_ERR_SHAPE
    assert lib.dab_mean_center_clamp(None, 6, 130, 1, 0, -1.0, 1.0, p, None) == dab.DAB_ERR_NULL
    assert lib.dab_weight_gradient(p, 6, 1, p, p, p, None, p, None) == dab.DAB_ERR_SHAPE
    assert lib.dab_binarized_weights(p, 0, 130, p, p, p, p, p, p, None) == dab.DAB_ERR_SHAPE
