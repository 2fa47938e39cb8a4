"""GPU parity of the re-binarizing epilogue and of pooling on packed signs (through the C ABI).

The bit [y >= tau] is decided in the kernel's fp32, so two things are checked: the fused output
equals, bit for bit, dab_pack_activations applied to the fp32 output of dab_binconv2d / dab_binfc
(same decision in the same precision), and it equals the oracle's float64 decision wherever y is
not within the fp32 tolerance of the threshold (there either bit is valid).
"""
import zlib

import numpy as np
import pytest
import torch

from oracle import layers as olay
from oracle import packing as opk
from paper_1804_02941_amd import binding as dab
from paper_1804_02941_amd import workloads as wl
from paper_1804_02941_amd.workloads import Layer

import gpu_util as gu
from test_gpu_parity import SMALL_LAYERS, weight_rows

pytestmark = pytest.mark.gpu


def run_both(L, x, W, tau_in, tau_out):
    """fp32 path and fused path on the same packed operands; returns numpy views and the estimate."""
    est_np, est = gu.gpu_estimate(W)
    W4 = W.reshape(L.F, L.C, L.kh, L.kw)
    E, _ = dab.dab_pack_weights(gu.to_gpu(W4), est["thr_val"], est["thr_idx"], est["alpha_is_upper"])
    tin = gu.to_gpu(tau_in) if tau_in is not None else None
    tout = gu.to_gpu(tau_out) if tau_out is not None else None
    B = x.shape[0]
    if L.is_fc:
        A = dab.dab_pack_activations(gu.to_gpu(x), dab.DAB_LAYOUT_NHWC, tin).reshape(B, -1)
        Y = dab.dab_binfc(A, E, est["alpha"], est["beta"], L.C)
        bits = dab.dab_binfc_bits(A, E, est["alpha"], est["beta"], L.C, tout)
    else:
        A = dab.dab_pack_activations(gu.to_gpu(np.transpose(x, (0, 2, 3, 1))), dab.DAB_LAYOUT_NHWC, tin)
        d = dab.dab_conv_desc(B, L.C, L.H, L.W, L.F, L.kh, L.kw, L.pad, L.pad, L.stride, L.stride)
        Y = dab.dab_binconv2d(d, A, E, est["alpha"], est["beta"])
        bits = dab.dab_binconv2d_bits(d, A, E, est["alpha"], est["beta"], tout)
    two_step = dab.dab_pack_activations(Y.reshape(B, L.Ho, L.Wo, L.F).contiguous(), dab.DAB_LAYOUT_NHWC, tout)
    torch.cuda.synchronize()
    return est_np, gu.u32(bits).reshape(B, L.Ho, L.Wo, -1), gu.u32(two_step), Y.cpu().numpy().reshape(B, L.Ho, L.Wo, L.F)


def check_rebinarize(L, x, W, tau_in, tau_out):
    est, bits, two_step, Y = run_both(L, x, W, tau_in, tau_out)
    assert np.array_equal(bits, two_step), "fused bits differ from packing the fp32 output"
    # oracle decision in float64 with the GPU's (already verified elsewhere) split and fp32 alpha, beta
    e, _ = gu.check_estimate(W.reshape(L.F, L.C, L.kh, L.kw), est)
    x4 = x if x.ndim == 4 else x[:, :, None, None]
    a = olay.binarize_activations(x4, tau_in)
    pad, stride = (L.pad, L.pad), (L.stride, L.stride)
    alpha, beta = est["alpha"].astype(np.float64), est["beta"].astype(np.float64)
    y_ref = olay.conv2d(a, olay.two_valued_filters(e, alpha, beta), pad, stride)
    s1, sA = olay.integer_terms(a, e, pad, stride)
    bound = olay.magnitude_bound(s1, sA, alpha, beta)
    t = np.zeros(L.F) if tau_out is None else tau_out.astype(np.float64)
    want = opk.pack_activations(olay.next_layer_input(y_ref, t))
    clear = np.abs(y_ref - t) > gu.Y_RTOL * np.maximum(np.abs(y_ref), bound)        # [B,Ho,Wo,F]
    got_pm1 = opk.unpack_activations(bits, L.F)                                     # NCHW +1/-1
    want_pm1 = opk.unpack_activations(want, L.F)
    same = np.transpose(got_pm1 == want_pm1, (0, 2, 3, 1))
    assert np.all(same | ~clear), "a bit differs from the oracle away from the threshold"
    assert clear.mean() > 0.99
    # bits past F are zero
    if L.F % 32:
        assert np.all(bits[..., -1] >> (L.F % 32) == 0)


@pytest.mark.parametrize("L", SMALL_LAYERS, ids=lambda L: L.name)
def test_small_conv_layers_rebinarized(L):
    rng = np.random.default_rng(zlib.crc32(L.name.encode()) % 1000)    # (hash() of a string is salted per process)
    x = rng.standard_normal((3, L.C, L.H, L.W)).astype(np.float32)
    W = weight_rows(rng, L.F, L.n, "mixture")
    tau_out = (rng.standard_normal(L.F) * 0.5).astype(np.float32)
    check_rebinarize(L, x, W, None, tau_out)
    check_rebinarize(L, x, W, None, None)


@pytest.mark.parametrize("C,F", [(160, 230), (64, 70), (256, 129)])
def test_filter_counts_that_end_inside_a_word_in_the_persistent_kernel(C, F):
    """Enough pixels for the persistent one-launch kernel and a filter count that is not a multiple of
    32: the bits past F in every pixel's last word are zero (they once took the unmasked compare)."""
    L = Layer(f"ragged_f{F}", C=C, H=14, W=10, F=F, kh=3, kw=3, pad=2)
    rng = np.random.default_rng(C * 1000 + F)
    x = rng.standard_normal((33, L.C, L.H, L.W)).astype(np.float32)
    W = weight_rows(rng, L.F, L.n, "mixture")
    tau_out = (rng.standard_normal(L.F) * 0.5).astype(np.float32)
    check_rebinarize(L, x, W, None, tau_out)
    check_rebinarize(L, x, W, None, None)


@pytest.mark.parametrize("B,K,F", [(1, 2, 1), (5, 70, 9), (64, 512, 512), (65, 1000, 130), (300, 4096, 48), (130, 9216, 40)])
def test_small_fc_layers_rebinarized(B, K, F):
    rng = np.random.default_rng(B * K + F)
    L = Layer("fc", C=K, H=1, W=1, F=F, kh=1, kw=1)
    x = rng.standard_normal((B, K)).astype(np.float32)
    W = weight_rows(rng, F, K, "gauss")
    check_rebinarize(L, x, W, None, (rng.standard_normal(F) * 0.3).astype(np.float32))


@pytest.mark.parametrize("C,H,W,kh,kw,sh,sw", [(128, 31, 31, 3, 3, 2, 2), (256, 15, 15, 3, 3, 2, 2), (37, 9, 7, 2, 3, 1, 2),
                                               (5, 4, 4, 4, 4, 1, 1), (70, 6, 5, 1, 1, 1, 1)])
def test_pool_bits(C, H, W, kh, kw, sh, sw):
    rng = np.random.default_rng(C + H)
    y = np.round(rng.standard_normal((3, H, W, C)) * 4).astype(np.float32) / 4       # ties with tau on purpose
    tau = (np.round(rng.standard_normal(C) * 2) / 4).astype(np.float32)
    A = dab.dab_pack_activations(gu.to_gpu(y), dab.DAB_LAYOUT_NHWC, gu.to_gpu(tau))
    pooled = dab.dab_pool_bits(A, C, kh, kw, sh, sw)
    torch.cuda.synchronize()
    want = opk.pack_activations(olay.next_layer_input(y.astype(np.float64), tau, pool=(kh, kw, sh, sw)))
    assert np.array_equal(gu.u32(pooled), want)


def test_config3_fused_chain_matches_fp32_chain():
    """Config 3 at batch 256 with bits handed from layer to layer (pooling on the bits): every
    stage is identical to packing the fp32 output of the plain path run on the same input bits."""
    dev = torch.device("cuda:0")
    imgs = wl.sketch_images(256)
    w1, ws = wl.config3_weights()
    x = wl.config3_conv1_features(imgs, w1, device=dev).permute(0, 2, 3, 1).contiguous()
    A = dab.dab_pack_activations(x, dab.DAB_LAYOUT_NHWC, x.mean(dim=(0, 1, 2)).contiguous())
    rng = np.random.default_rng(3)
    for L, W in zip(wl.CFG3_LAYERS, ws):
        Wt = torch.from_numpy(W).to(dev)
        est = dab.dab_estimate_alpha_beta(Wt.reshape(L.F, -1))
        E, _ = dab.dab_pack_weights(Wt, est["thr_val"], est["thr_idx"], est["alpha_is_upper"])
        tau_out = gu.to_gpu((rng.standard_normal(L.F) * 0.2).astype(np.float32))
        if L.is_fc:
            A2 = A.reshape(256, -1)
            Y = dab.dab_binfc(A2, E, est["alpha"], est["beta"], L.C)
            bits = dab.dab_binfc_bits(A2, E, est["alpha"], est["beta"], L.C, tau_out)
            ref = dab.dab_pack_activations(Y, dab.DAB_LAYOUT_NHWC, tau_out).reshape(bits.shape)
        else:
            d = dab.dab_conv_desc(256, L.C, L.H, L.W, L.F, L.kh, L.kw, L.pad, L.pad, L.stride, L.stride)
            assert tuple(A.shape) == (256, L.H, L.W, dab.words_per_pixel(L.C))
            Y = dab.dab_binconv2d(d, A, E, est["alpha"], est["beta"])
            bits = dab.dab_binconv2d_bits(d, A, E, est["alpha"], est["beta"], tau_out)
            ref = dab.dab_pack_activations(Y, dab.DAB_LAYOUT_NHWC, tau_out)
            if L.pool_after:
                pooled_y = torch.nn.functional.max_pool2d(Y.permute(0, 3, 1, 2), 3, 2).permute(0, 2, 3, 1).contiguous()
                ref = dab.dab_pack_activations(pooled_y, dab.DAB_LAYOUT_NHWC, tau_out)
                bits = dab.dab_pool_bits(bits, L.F, 3, 3, 2, 2)
        torch.cuda.synchronize()
        assert torch.equal(bits, ref), L.name
        A = bits


def test_error_codes_of_the_new_entry_points():
    d = dab.dab_conv_desc(8192, 9216, 1, 1, 512, 1, 1, 0, 0, 1, 1)   # a long reduction over many rows: operands are expanded into a workspace
    A = torch.zeros((8192, 1, 1, 288), dtype=torch.int32, device="cuda:0")
    E = torch.zeros((288, 512), dtype=torch.int32, device="cuda:0")
    ab = torch.ones(512, dtype=torch.float32, device="cuda:0")
    import ctypes
    out = torch.zeros((8192, 1, 1, 16), dtype=torch.int32, device="cuda:0")
    small = torch.empty(256, dtype=torch.uint8, device="cuda:0")
    rc = dab.lib().dab_binconv2d_bits(ctypes.byref(d), A.data_ptr(), E.data_ptr(), ab.data_ptr(), ab.data_ptr(), None,
                                      out.data_ptr(), small.data_ptr(), 256, None)
    assert rc == 4                                                   # workspace too small
    rc = dab.lib().dab_binconv2d_bits(ctypes.byref(d), A.data_ptr(), E.data_ptr(), ab.data_ptr(), ab.data_ptr(), None,
                                      None, small.data_ptr(), 256, None)
    assert rc == 1                                                   # no output buffer
    A = torch.zeros((1, 8, 8, 2), dtype=torch.int32, device="cuda:0")
    rc = dab.lib().dab_pool_bits(A.data_ptr(), 1, 64, 8, 8, 9, 3, 1, 1, out.data_ptr(), None)
    assert rc == 2                                                   # window larger than the image
