"""GPU parity of the weights-only binarized layer (WBin of Section 5.1) through the C ABI.

The kernel splits every fp32 input exactly into three bf16 pieces and multiplies them with 0 / 1
masks on the matrix cores, so only the fp32 accumulation rounds.  Outputs are compared with the
float64 oracle relative to sum |x_i||w~_i| (the scale a floating-point evaluation is accurate
to); inputs made of small integers must come out exactly.
"""
import zlib

import numpy as np
import pytest
import torch

from oracle import layers as olay
from paper_1804_02941_amd import binding as dab
from paper_1804_02941_amd import workloads as wl
from paper_1804_02941_amd.workloads import Layer

import gpu_util as gu
from test_gpu_parity import SMALL_LAYERS, weight_rows
from test_gpu_fullsize import sample_points

pytestmark = pytest.mark.gpu

# fp32 accumulation of exact terms: measured errors are a few 1e-7 of the scale; the bound
# (3n/16 + T) * 2^-24 exceeds 1e-5 only for reductions longer than ~900 terms, where the
# tolerance follows it
def tolerance(n, T):
    return max(1e-5, 0.25 * (3 * n / 16 + T) * 2.0 ** -24)


def run_wbin(L, x_nchw, W, alpha=None, beta=None):
    """Estimate, pack weights, weights-only layer.  Returns (Y numpy, e, alpha64, beta64)."""
    est_np, est = gu.gpu_estimate(W)
    W4 = W.reshape(L.F, L.C, L.kh, L.kw)
    e, _ = gu.check_estimate(W4, est_np)
    E, _ = dab.dab_pack_weights(gu.to_gpu(W4), est["thr_val"], est["thr_idx"], est["alpha_is_upper"])
    a_t = est["alpha"] if alpha is None else gu.to_gpu(alpha)
    b_t = est["beta"] if beta is None else gu.to_gpu(beta)
    if L.is_fc:
        Y = dab.dab_wbin_fc(gu.to_gpu(x_nchw.reshape(x_nchw.shape[0], -1)), E, a_t, b_t)
    else:
        d = dab.dab_conv_desc(x_nchw.shape[0], L.C, L.H, L.W, L.F, L.kh, L.kw, L.pad, L.pad, L.stride, L.stride)
        Y = dab.dab_wbin_conv2d(d, gu.to_gpu(np.transpose(x_nchw, (0, 2, 3, 1))), E, a_t, b_t)
    torch.cuda.synchronize()
    return Y.cpu().numpy(), e, a_t.cpu().numpy().astype(np.float64), b_t.cpu().numpy().astype(np.float64)


def check_wbin(L, x, W):
    Y, e, a64, b64 = run_wbin(L, x, W)
    pad, stride = (L.pad, L.pad), (L.stride, L.stride)
    xx = x if not L.is_fc else x.reshape(x.shape[0], -1)
    ee = e if not L.is_fc else e.reshape(L.F, -1)
    ref = olay.weights_only_layer(xx, ee, a64, b64, pad, stride)
    mag = olay.weights_only_magnitude(xx, ee, a64, b64, pad, stride)
    err = np.abs(Y.reshape(ref.shape) - ref)
    tol = tolerance(L.n, L.kh * L.kw)
    assert np.all(err <= tol * mag + 1e-30), f"max error {np.max(err / np.maximum(mag, 1e-30)):.2e} of the scale (tolerance {tol:.1e})"
    return float(np.max(err / np.maximum(mag, 1e-30)))


def real_inputs(rng, shape):
    """Real activations with a wide dynamic range, exact zeros and negative values."""
    x = rng.standard_normal(shape) * np.exp(rng.uniform(-6, 3, shape))
    x[rng.random(shape) < 0.2] = 0.0
    return x.astype(np.float32)


@pytest.mark.parametrize("L", SMALL_LAYERS, ids=lambda L: L.name)
@pytest.mark.parametrize("B", [1, 3])
def test_small_conv_layers(L, B):
    rng = np.random.default_rng(zlib.crc32(L.name.encode()) % 1000 + 7 * B)    # (hash() of a string is salted per process)
    check_wbin(L, real_inputs(rng, (B, L.C, L.H, L.W)), weight_rows(rng, L.F, L.n, "mixture"))


def test_mid_sized_layer_runs_the_persistent_kernel_unsplit():
    """More than 512 output blocks but too few tiles to fill the chip: the main kernel, no split."""
    rng = np.random.default_rng(74)
    L = Layer("mid", C=24, H=16, W=16, F=300, kh=3, kw=3, pad=1)
    check_wbin(L, real_inputs(rng, (8, L.C, L.H, L.W)), weight_rows(rng, L.F, L.n, "mixture"))


@pytest.mark.parametrize("B,K,F", [(1, 2, 1), (5, 70, 9), (64, 512, 512), (65, 1000, 130), (130, 9216, 40)])
def test_small_fc_layers(B, K, F):
    rng = np.random.default_rng(B + K + F + 1)
    L = Layer("fc", C=K, H=1, W=1, F=F, kh=1, kw=1)
    check_wbin(L, real_inputs(rng, (B, K)), weight_rows(rng, F, K, "gauss" if K > 2 else "onesided"))


def test_integer_inputs_are_exact():
    """18-bit integers need all three bf16 pieces; with alpha = 1, beta = 0 the output is the integer
    sum over the mask, exactly (short reductions, so every partial sum fits 24 bits)."""
    rng = np.random.default_rng(71)
    for L in (Layer("i1", C=5, H=6, W=7, F=40, kh=3, kw=3, pad=1), Layer("i2", C=20, H=4, W=4, F=130, kh=1, kw=2),
              Layer("ifc", C=60, H=1, W=1, F=33, kh=1, kw=1)):
        B = 3
        xi = rng.integers(-(1 << 17), 1 << 17, size=(B, L.C, L.H, L.W))
        W = weight_rows(rng, L.F, L.n, "mixture")
        ones, zeros = np.ones(L.F, dtype=np.float32), np.zeros(L.F, dtype=np.float32)
        Y, e, _, _ = run_wbin(L, xi.astype(np.float32), W, alpha=ones, beta=zeros)
        pad, stride = (L.pad, L.pad), (L.stride, L.stride)
        if L.is_fc:
            want = olay.fc(xi.reshape(B, -1), e.reshape(L.F, -1), dtype=np.int64)
        else:
            want = olay.conv2d(xi, e, pad, stride, dtype=np.int64)
        assert np.array_equal(Y.reshape(want.shape).astype(np.int64), want)
        # beta = 1, alpha = 1: the plain window sum (the per-pixel sums and their box sum)
        Y, e, _, _ = run_wbin(L, xi.astype(np.float32), W, alpha=ones, beta=ones)
        if L.is_fc:
            want = xi.reshape(B, -1).sum(axis=1)[:, None] * np.ones((1, L.F), dtype=np.int64)
        else:
            want = olay.conv2d(xi, np.ones_like(e), pad, stride, dtype=np.int64)
        assert np.array_equal(Y.reshape(want.shape).astype(np.int64), want)


def test_plus_minus_one_inputs_give_the_binarized_layer():
    """On +1 / -1 inputs the weights-only layer is the fully binarized one."""
    rng = np.random.default_rng(72)
    L = Layer("pm1", C=70, H=9, W=8, F=50, kh=3, kw=3, pad=1)
    x = rng.standard_normal((2, L.C, L.H, L.W)).astype(np.float32)
    W = weight_rows(rng, L.F, L.n, "mixture")
    a = np.where(x >= 0, 1.0, -1.0).astype(np.float32)
    Yw, e, a64, b64 = run_wbin(L, a, W)
    full = gu.gpu_layer(L, x, W)
    s1, sA = olay.integer_terms(a.astype(np.int8), e, (1, 1), (1, 1))
    bound = olay.magnitude_bound(s1, sA, a64, b64)
    assert np.all(np.abs(Yw - full["Y"].reshape(Yw.shape)) <= 2 * gu.Y_RTOL * bound + 1e-30)


def test_conv2_shape_at_batch_128_sampled():
    """config 2 (conv2 of the trunk, batch 128) in the launch shape a full layer uses; sampled outputs."""
    L, x, w = wl.config2(batch=128)
    Y, e, a64, b64 = run_wbin(L, x, w)
    pts = sample_points(np.random.default_rng(73), 128, L.Ho, L.Wo, L.F, 300)
    pad, stride = (L.pad, L.pad), (L.stride, L.stride)
    Wt = olay.two_valued_filters(e, a64, b64)
    ref = olay.conv2d_at(x, Wt, pad, stride, pts)
    mag = olay.conv2d_at(np.abs(x), np.abs(Wt), pad, stride, pts)
    Y = Y.reshape(128, L.Ho, L.Wo, L.F)
    got = np.array([Y[b, oy, ox, f] for b, oy, ox, f in pts], dtype=np.float64)
    assert np.all(np.abs(got - ref) <= tolerance(L.n, L.kh * L.kw) * mag + 1e-30)


def test_errors():
    lib = dab.lib()
    t = torch.zeros(4096, dtype=torch.float32, device=gu.DEV)
    import ctypes
    d = dab.dab_conv_desc(1, 16, 4, 4, 8, 3, 3, 1, 1, 1, 1)
    p = t.data_ptr()
    assert lib.dab_wbin_conv2d(ctypes.byref(d), p, p, p, p, p, None, 0, None) == dab.DAB_ERR_WORKSPACE
    assert lib.dab_wbin_conv2d(ctypes.byref(d), None, p, p, p, p, p, 1 << 20, None) == dab.DAB_ERR_NULL
    assert lib.dab_wbin_fc(0, 16, 8, p, p, p, p, p, p, 1 << 20, None) == dab.DAB_ERR_SHAPE
    assert lib.dab_wbin_conv2d_workspace_bytes(ctypes.byref(d)) > 0


@pytest.mark.parametrize("k,pad,stride", [(1, 1, 1), (2, 2, 1), (3, 3, 2)])
def test_padding_that_reaches_the_kernel_extent(k, pad, stride):
    """Windows that lie entirely in the zero border give zero."""
    L = Layer(f"wbin_k{k}p{pad}", C=96, H=9, W=8, F=70, kh=k, kw=k, pad=pad, stride=stride)
    rng = np.random.default_rng(zlib.crc32(L.name.encode()))
    x = real_inputs(rng, (4, L.C, L.H, L.W))
    W = weight_rows(rng, L.F, L.n, "gauss").reshape(L.F, L.C, k, k)
    check_wbin(L, x, W)
