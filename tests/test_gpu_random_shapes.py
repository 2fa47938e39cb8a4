"""Seeded random sweeps over layer shapes and job mixes (through the C ABI, on the GPU).

The fixed cases of the other files sit on the boundaries somebody thought of; these draw shapes
across all product kernels (channel counts that are and are not multiples of 32 / 256, padding up
to the kernel extent, strides, filter counts that end inside a word, fully-connected shapes) and
mixes of layers for the grouped calls, and check what is unique: integer sums and estimates
against the oracle, the packed-sign output against packing the fp32 output, the grouped calls
against the separate ones.
"""
import numpy as np
import pytest
import torch

from paper_1804_02941_amd import binding as dab
from paper_1804_02941_amd import workloads as wl

from oracle import packing as opk
from oracle import training as otr

import gpu_util as gu
from test_gpu_parity import weight_rows
from test_gpu_training import check_bounded
from test_gpu_fullsize import _structured_masks

pytestmark = pytest.mark.gpu


def draw_shape(rng, big=False):
    """(B, C, H, W, F, kh, kw, pad, stride) of a layer: many-channel, odd-channel, many-pixel or fully-connected."""
    kind = int(rng.integers(0, 4))
    if kind == 0:
        C = int(rng.choice([256, 512, 768, 1024])); kh = int(rng.choice([1, 2, 3])); kw = int(rng.choice([1, 2, 3]))
        H = int(rng.integers(kh, 9)); W = int(rng.integers(kw, 9)); F = int(rng.integers(1, 300 if big else 140))
        B = int(rng.integers(1, 40 if big else 5))
    elif kind == 1:
        C = int(rng.integers(1, 300)); kh = int(rng.integers(1, 6)); kw = int(rng.integers(1, 6))
        H = int(rng.integers(kh, 20 if big else 14)); W = int(rng.integers(kw, 20 if big else 14))
        F = int(rng.integers(1, 300 if big else 200)); B = int(rng.integers(1, 10 if big else 4))
    elif kind == 2:
        C = int(rng.choice([32, 64, 96, 128, 160, 256])); kh = kw = int(rng.choice([1, 3, 5]))
        H = int(rng.integers(kh + 6, 40 if big else 24)); W = int(rng.integers(kw + 6, 40 if big else 24))
        F = int(rng.integers(60, 400 if big else 300)); B = int(rng.integers(2, 40 if big else 8))
    else:
        C = int(rng.choice([64, 200, 512, 1280, 2048, 4096] + ([9216] if big else []))); kh = kw = 1; H = W = 1
        F = int(rng.integers(1, 600 if big else 300)); B = int(rng.integers(1, 1200 if big else 200))
    pad = int(rng.integers(0, max(kh, kw) + 1)) if 1 < kh * kw <= 32 else 0
    stride = int(rng.integers(1, 4))
    return B, C, H, W, F, kh, kw, pad, stride


def usable(s, max_n=None):
    B, C, H, W, F, kh, kw, pad, stride = s
    return H + 2 * pad >= kh and W + 2 * pad >= kw and C * kh * kw >= 2 and (max_n is None or C * kh * kw <= max_n)


def test_random_layers_against_the_oracle():
    rng = np.random.default_rng(20241)
    done = 0
    while done < 120:
        s = draw_shape(rng)
        if not usable(s, 13312):
            continue
        B, C, H, W, F, kh, kw, pad, stride = s
        L = wl.Layer(f"random{done}", C=C, H=H, W=W, F=F, kh=kh, kw=kw, pad=pad, stride=stride)
        x = rng.standard_normal((B, C, H, W)).astype(np.float32)
        w = weight_rows(rng, F, L.n, str(rng.choice(["gauss", "mixture"])))
        tau = (rng.standard_normal(C) * 0.3).astype(np.float32) if rng.integers(0, 2) else None
        try:
            gu.check_layer(L, x, w, tau=tau, layout="nhwc")
        except AssertionError as e:
            raise AssertionError(f"{s}: {e}") from e
        done += 1


def test_random_layers_packed_sign_output_equals_packing_the_fp32_output():
    rng = np.random.default_rng(20242)
    torch.manual_seed(20242)
    dev = "cuda:0"
    done = 0
    while done < 300:
        s = draw_shape(rng, big=True)
        if not usable(s):
            continue
        B, C, H, W, F, kh, kw, pad, stride = s
        Cw, Fp = (C + 31) // 32, 64 * ((F + 63) // 64)
        A = torch.randint(-2**31, 2**31 - 1, (B, H, W, Cw), dtype=torch.int32, device=dev)
        E = torch.randint(-2**31, 2**31 - 1, (kh * kw * Cw, Fp), dtype=torch.int32, device=dev)
        if C % 32:                                                  # bits past C are zero in packed operands
            A[..., -1] &= (1 << (C % 32)) - 1
            E.view(kh * kw, Cw, Fp)[:, -1, :] &= (1 << (C % 32)) - 1
        E[:, F:] = 0
        alpha = torch.rand(F, device=dev) + 0.1
        beta = -torch.rand(F, device=dev) - 0.1
        tau = torch.randn(F, device=dev) * 3.0 if rng.integers(0, 2) else None
        d = dab.dab_conv_desc(B, C, H, W, F, kh, kw, pad, pad, stride, stride)
        Y, s1 = dab.dab_binconv2d(d, A, E, alpha, beta, want_s1=True)
        bits = dab.dab_binconv2d_bits(d, A, E, alpha, beta, tau)
        ref = dab.dab_pack_activations(Y, dab.DAB_LAYOUT_NHWC, tau)
        torch.cuda.synchronize()
        assert torch.equal(bits.reshape(ref.shape), ref), s
        assert int(s1.abs().max()) <= C * kh * kw, s
        done += 1


def test_random_mixes_through_prepare_layers_equal_the_separate_calls():
    rng = np.random.default_rng(20243)
    kinds = ["gauss", "mixture", "laplace", "dupes", "onesided"]
    for mix in range(40):
        wjobs, desc = [], []
        for _ in range(int(rng.integers(1, 7))):
            cls = int(rng.integers(0, 5))
            n = int([rng.integers(2, 2305), rng.integers(2305, 4609), rng.integers(4609, 9217), rng.integers(9217, 13313),
                     rng.choice([2304, 2305, 4608, 4609, 9216, 9217, 13312, 256, 257])][cls])
            T = next((t for t in (25, 9, 4, 3, 2) if n % t == 0), 1)
            kh, kw = {25: (5, 5), 9: (3, 3), 4: (2, 2), 3: (1, 3), 2: (2, 1), 1: (1, 1)}[T]
            C = n // T
            many = rng.integers(0, 12) == 0 and n <= 4608           # enough rows to be handed to the sort kernel
            F = int(rng.integers(1536, 1800)) if many else int(rng.integers(1, 200))
            kind = str(rng.choice(kinds))
            W = weight_rows(rng, F, n, kind).reshape(F, C, kh, kw)
            if rng.integers(0, 4) == 0:
                W[int(rng.integers(0, F))] = float(rng.standard_normal())                # a constant filter
            Wt = gu.to_gpu(W)
            wjobs.append(dict(W=Wt, est=dab.estimate_outputs(F, Wt.device), packed=dab.pack_weights_outputs(F, C, kh, kw, Wt.device)))
            desc.append((F, C, kh, kw, kind))
        pitems = []
        for _ in range(int(rng.integers(1, 6))):
            C = int(rng.choice([1, 3, 31, 64, 70, 128, 192, 256, 300, 512, 1024]))
            B, H, Wd = int(rng.integers(1, 40)), int(rng.integers(1, 12)), int(rng.integers(1, 12))
            X = gu.to_gpu(rng.standard_normal((B, H, Wd, C)).astype(np.float32))
            tau = gu.to_gpu(rng.standard_normal(C).astype(np.float32) * 0.3) if rng.integers(0, 2) else None
            pitems.append((X, tau, torch.full((B, H, Wd, dab.words_per_pixel(C)), -1, dtype=torch.int32, device=X.device)))
        if sum(d[0] for d in desc) < len(pitems):
            continue                                                # (fewer filters than tensors: the call refuses)
        dab.dab_prepare_layers(dab.weight_jobs(wjobs), dab.pack_jobs(pitems))
        torch.cuda.synchronize()
        for j, dsc in zip(wjobs, desc):
            F = dsc[0]
            ref = dab.dab_estimate_alpha_beta(j["W"].reshape(F, -1))
            E, ecnt = dab.dab_pack_weights(j["W"], ref["thr_val"], ref["thr_idx"], ref["alpha_is_upper"])
            torch.cuda.synchronize()
            if all(torch.equal(j["est"][k], ref[k]) for k in ref):
                assert torch.equal(j["packed"][0], E) and torch.equal(j["packed"][1], ecnt), dsc
            else:
                # only rows with splits tied to rounding may differ (a constant filter): then both are the oracle's maximum
                gu.check_estimate(j["W"].cpu().numpy(), {k: v.cpu().numpy() for k, v in j["est"].items()})
        for (X, tau, A) in pitems:
            R = dab.dab_pack_activations(X, dab.DAB_LAYOUT_NHWC, tau)
            torch.cuda.synchronize()
            assert torch.equal(A, R.reshape(A.shape)), tuple(X.shape)


ROW_LENGTHS = [2, 3, 64, 192, 193, 255, 256, 257, 768, 769, 1280, 1792, 1793, 2304, 2305, 2816, 2817, 3584, 3585, 4095, 4096,
               4608, 4609, 5632, 7168, 7169, 8192, 8193, 9216, 9217, 11264, 11265, 13312]      # the kernels' class limits


def test_random_rows_through_the_estimators():
    """Rows of every length class and kind (duplicates, one-sided, constant, two-valued) through the plain, the
    windowed and the allocation-free estimator and the training-side kernels, against the oracle."""
    rng = np.random.default_rng(20244)
    for it in range(120):
        n = int(rng.choice(ROW_LENGTHS)) if rng.integers(0, 3) == 0 else int(rng.integers(2, 13313))
        F = int(rng.integers(1, 40)) if n > 3000 else int(rng.integers(1, 300))
        w = weight_rows(rng, F, n, str(rng.choice(["gauss", "mixture", "laplace", "dupes", "onesided"])))
        if rng.integers(0, 5) == 0:
            w[int(rng.integers(0, F))] = float(rng.standard_normal())
        if rng.integers(0, 8) == 0:
            w[int(rng.integers(0, F))] = np.where(rng.random(n) < 0.5, 0.25, -0.5).astype(np.float32)
        t = gu.to_gpu(w)
        which = int(rng.integers(0, 4))
        if which == 0:
            got = dab.dab_estimate_alpha_beta(t)
            torch.cuda.synchronize()
            gu.check_estimate(w, {k: v.cpu().numpy() for k, v in got.items()})
        elif which == 1:
            prev = dab.dab_estimate_alpha_beta(t)
            w1 = (w + 0.05 * np.float32(np.sqrt(2.0 / n)) * rng.standard_normal((F, n))).astype(np.float32)
            d = int(rng.choice([0, 1, 2, max(2, n // 50), n, 2 ** 31 - 1]))
            got = dab.dab_estimate_alpha_beta_bounded(gu.to_gpu(w1), prev["K"], prev["alpha_is_upper"], d)
            torch.cuda.synchronize()
            check_bounded(w1, {k: v.cpu().numpy() for k, v in got.items()}, prev["K"].cpu().numpy(),
                          prev["alpha_is_upper"].cpu().numpy(), d)
        elif which == 2:
            W2 = dab.dab_mean_center_clamp(t.reshape(F, n, 1, 1)).reshape(F, n)
            est = dab.dab_estimate_alpha_beta(W2)
            Wt = dab.dab_binarized_weights(W2, est["alpha"], est["beta"], est["thr_val"], est["thr_idx"], est["alpha_is_upper"])
            up = rng.standard_normal((F, n)).astype(np.float32)
            dW = dab.dab_weight_gradient(W2, est["thr_val"], est["thr_idx"], est["alpha_is_upper"], upstream=gu.to_gpu(up))
            torch.cuda.synchronize()
            wc, est_np = W2.cpu().numpy(), {k: v.cpu().numpy() for k, v in est.items()}
            assert np.allclose(wc, otr.mean_center_clamp(w.reshape(F, n, 1, 1), "filter").reshape(F, n), rtol=1e-5, atol=1e-7)
            e, _ = gu.check_estimate(wc, est_np)
            assert np.array_equal(Wt.cpu().numpy(), np.where(e == 1, est_np["alpha"][:, None], est_np["beta"][:, None]).astype(np.float32))
            ref = otr.weight_gradient(wc, e, up)
            assert np.allclose(dW.cpu().numpy(), ref, rtol=1e-5, atol=1e-6 * np.abs(ref).max()), (F, n)
        else:
            a = dab.dab_estimate_alpha_beta(t)
            b = dab.dab_estimate_alpha_beta_noalloc(t, dab.estimate_outputs(F, t.device))
            torch.cuda.synchronize()
            for k in a:
                assert torch.equal(a[k], b[k]), (k, F, n)


def closed_form_check(rng, B, C, H, W, F, kh, kw, pad, stride):
    """Every output of the fp32 and of the packed-sign launch of one layer against values built with numpy indexing
    only: masks that select whole windows, single weights, channel ranges or tap rows make s1 a difference of
    channel prefix sums, and alpha = 1.5, beta = 0.5 make y = s1 + sA / 2 exact in fp32 (so the signs are fixed too)."""
    L = wl.Layer("closed", C=C, H=H, W=W, F=F, kh=kh, kw=kw, pad=pad, stride=stride)
    shape = dict(B=B, C=C, H=H, W=W, F=F, kh=kh, kw=kw, pad=pad, stride=stride)
    a = (rng.integers(0, 2, size=(B, C, H, W), dtype=np.int8) * 2 - 1)
    e, spec = _structured_masks(L, rng)
    A = gu.to_gpu(opk.pack_activations(a).view(np.int32)).reshape(B, H, W, -1)
    E = gu.to_gpu(opk.pack_weights(e)[0].view(np.int32))
    alpha = torch.full((F,), 1.5, dtype=torch.float32, device="cuda:0")
    beta = torch.full((F,), 0.5, dtype=torch.float32, device="cuda:0")
    tau_np = (rng.integers(-6, 7, size=F) * 0.5).astype(np.float32)
    d = dab.dab_conv_desc(B, C, H, W, F, kh, kw, pad, pad, stride, stride)
    Y = dab.dab_binconv2d(d, A, E, alpha, beta)
    bits = dab.dab_binconv2d_bits(d, A, E, alpha, beta, gu.to_gpu(tau_np))
    torch.cuda.synchronize()
    cp = np.zeros((B, C + 1, H + 2 * pad, W + 2 * pad), dtype=np.int32)              # channel prefix sums, zero border
    np.cumsum(a, axis=1, dtype=np.int32, out=cp[:, 1:, pad:pad + H, pad:pad + W])

    def window_sum(plane, taps):
        out = np.zeros((B, L.Ho, L.Wo), dtype=np.int32)
        for (i, j) in taps:
            out += plane[:, i:i + stride * (L.Ho - 1) + 1:stride, j:j + stride * (L.Wo - 1) + 1:stride]
        return out

    sA = window_sum(cp[:, C], [(i, j) for i in range(kh) for j in range(kw)])
    want, cache = np.empty((B, L.Ho, L.Wo, F), np.float32), {}
    for f, (c0, c1, taps) in enumerate(spec):
        key = (c0, c1, tuple(taps))
        if key not in cache:
            cache[key] = window_sum(cp[:, c1] - cp[:, c0], taps)
        want[..., f] = cache[key].astype(np.float32) + 0.5 * sA.astype(np.float32)
    assert np.array_equal(Y.cpu().numpy().reshape(want.shape), want), shape
    signs = np.where(want >= tau_np, 1, -1).astype(np.int8)
    want_bits = opk.pack_activations(np.transpose(signs, (0, 3, 1, 2)))
    assert np.array_equal(gu.u32(bits).reshape(want_bits.shape), want_bits), shape


def test_random_mid_sized_layers_whole_tensor_against_closed_forms():
    """Thousands to a hundred thousand pixels: many tiles of the persistent kernel, ragged last tiles."""
    rng = np.random.default_rng(20245)
    done = 0
    while done < 30:
        k = int(rng.choice([1, 3, 5, 7]))
        kh, kw = k, int(rng.choice([k, max(1, k - 2)]))
        C = int(rng.choice([32, 48, 64, 70, 96, 128, 160, 256, 300, 512, 1024]))
        F, B = int(rng.integers(1, 400)), int(rng.choice([1, 3, 8, 32, 64, 128, 256]))
        H, W = int(rng.integers(kh, 64)), int(rng.integers(kw, 64))
        pad = int(rng.integers(0, min(kh, kw) + 1)) if 1 < kh * kw <= 32 else 0
        stride = int(rng.integers(1, 4))
        L = wl.Layer("probe", C=C, H=H, W=W, F=F, kh=kh, kw=kw, pad=pad, stride=stride)
        M = B * L.Ho * L.Wo
        if M * F > 4e7 or B * C * H * W > 6e7 or M < 2000:
            continue
        closed_form_check(rng, B, C, H, W, F, kh, kw, pad, stride)
        done += 1


def limit_shapes():
    """Shapes on both sides of the limits that decide which kernel runs and how it is tiled."""
    cases = []
    for C in (224, 256, 288, 320):                                  # reductions around the persistent kernel's 36 k-steps
        cases.append((8, C, 20, 20, 130, 3, 3, 1, 1))
    for (kh, kw) in ((4, 8), (3, 11), (5, 7), (6, 6)):              # padded windows around 32 taps
        cases.append((4, 64, 24, 24, 70, kh, kw, 2, 1))
    for M in (16352, 16384, 16416):                                 # 511, 512, 513 blocks of 32 x 32
        cases.append((M // 16, 512, 4, 4, 32, 1, 1, 0, 1))
    for B in (63, 64, 65, 127, 128, 129, 255, 256, 257):            # block counts around the small-product limits, long reductions
        cases.append((B, 2304, 1, 1, 1000, 1, 1, 0, 1))
    for B in (500, 1024, 2048):
        cases.append((B, 4096, 1, 1, 1030, 1, 1, 0, 1))
    for (H, W) in ((16, 16), (16, 17), (23, 22), (32, 32)):         # pixel counts around whole tiles of 64 / 256 / 512
        for B in (1, 2, 31, 32, 33):
            cases.append((B, 64, H, W, 128, 3, 3, 1, 1))
    for F in (1, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257):   # filter counts around words and 128-filter tiles
        cases.append((16, 96, 18, 18, F, 3, 3, 1, 1))
    for pad in (0, 1, 2, 3):                                        # padding up to the kernel extent, strides
        for stride in (1, 2, 3):
            cases.append((16, 128, 21, 19, 100, 3, 3, pad, stride))
    return cases


def test_shapes_at_the_kernels_limits_whole_tensor():
    rng = np.random.default_rng(20246)
    for case in limit_shapes():
        closed_form_check(rng, *case)
