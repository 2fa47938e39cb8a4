"""GPU parity at the full sizes of the five configurations, in the launch shapes bench.py times.

The oracle cannot evaluate a whole layer at these sizes in seconds, so the fp32 outputs and
the integers s1 are checked on sampled outputs computed one by one (always including image
corners and borders and the last pixel / filter), while everything that is cheap on the
CPU is still checked in full: alpha/beta/K of every filter, every packed weight bit and
per-tap count, every packed activation bit.
"""
import numpy as np
import pytest
import torch

from oracle import layers as olay
from oracle import packing as opk
from paper_1804_02941_amd import binding as dab
from paper_1804_02941_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu


def sample_points(rng, B, Ho, Wo, F, count):
    pts = {(0, 0, 0, 0), (B - 1, Ho - 1, Wo - 1, F - 1), (0, 0, Wo - 1, F // 2), (B - 1, Ho - 1, 0, 0),
           (B // 2, Ho // 2, Wo // 2, F - 1), (0, Ho - 1, Wo // 2, 1 % F)}
    while len(pts) < count:
        pts.add((int(rng.integers(B)), int(rng.integers(Ho)), int(rng.integers(Wo)), int(rng.integers(F))))
    return sorted(pts)


def check_full_layer(L, x_nchw, W, tau, g, count=96, seed=0):
    """g = gu.gpu_layer(...) result (or equivalent dict) for this layer at full size."""
    W4 = W.reshape(L.F, L.C, L.kh, L.kw)
    e, differ = gu.check_estimate(W4, g["est"])
    E_ref, ecnt_ref = opk.pack_weights(e)
    assert np.array_equal(g["E"], E_ref) and np.array_equal(g["ecnt"], ecnt_ref)
    x4 = x_nchw if x_nchw.ndim == 4 else x_nchw[:, :, None, None]
    a = olay.binarize_activations(x4, tau)
    A_ref = opk.pack_activations(a)
    assert np.array_equal(g["A"].reshape(A_ref.shape), A_ref)
    B = x4.shape[0]
    pts = sample_points(np.random.default_rng(seed), B, L.Ho, L.Wo, L.F, count)
    alpha = g["est"]["alpha"].astype(np.float64)
    beta = g["est"]["beta"].astype(np.float64)
    Wt = olay.two_valued_filters(e, alpha, beta)
    pad, stride = (L.pad, L.pad), (L.stride, L.stride)
    y_ref = olay.conv2d_at(a, Wt, pad, stride, pts)
    s1_ref = olay.conv2d_at(a, e, pad, stride, pts)
    sA_ref = olay.conv2d_at(a, np.ones((1,) + e.shape[1:]), pad, stride, [(b, oy, ox, 0) for b, oy, ox, _ in pts])
    Y = g["Y"].reshape(B, L.Ho, L.Wo, L.F)
    S1 = g["s1"].reshape(B, L.Ho, L.Wo, L.F)
    for j, p in enumerate(pts):
        f = p[3]
        assert S1[p] == int(round(s1_ref[j])), f"s1 at {p}"
        bound = abs(alpha[f]) * abs(s1_ref[j]) + abs(beta[f]) * abs(sA_ref[j] - s1_ref[j])
        assert abs(float(Y[p]) - y_ref[j]) <= gu.Y_RTOL * max(abs(y_ref[j]), bound), f"Y at {p}"
    # a property that holds at any size: s1 and K have the same parity as the number of valid taps' e-bits,
    # and |s1| never exceeds the e-bits inside the window
    K = g["est"]["K"].astype(np.int64)
    assert np.all(np.abs(S1.astype(np.int64)) <= K)
    if L.pad == 0:
        assert np.all((S1.astype(np.int64) - K) % 2 == 0)
    return differ


def test_config2_full():
    L, x, w = wl.config2()
    tau = x.mean(axis=(0, 2, 3)).astype(np.float32)
    g = gu.gpu_layer(L, x, w, tau)
    check_full_layer(L, x, w, tau, g)


def test_config3_full_chain():
    """Batch 256, every layer's input produced by the previous GPU layer, as in the benchmark."""
    import bench
    states = bench.build_states(256, dab, torch, wl)
    for s in states:
        L = s.L
        x = s.X.cpu().numpy()
        x_nchw = np.ascontiguousarray(np.transpose(x, (0, 3, 1, 2))) if x.ndim == 4 else x
        tau = s.tau.cpu().numpy()
        W = s.W.cpu().numpy()
        g = gu.gpu_layer(L, x_nchw, W, tau)
        # the benchmark's own launch (no s1 output, preallocated buffers) gives the same Y
        y_bench = bench.run_layer(s, dab)
        torch.cuda.synchronize()
        assert torch.equal(y_bench.reshape(-1), g["Y_gpu"].reshape(-1))
        check_full_layer(L, x_nchw, W, tau, g, count=64)
    # the benchmark's step (grouped calls, weight sides on side streams) reproduces every layer bit for bit
    want = [s.Y.clone() for s in states]
    bits = [s.A.clone() for s in states]
    sched = bench.GroupedStep(states, dab, torch)
    graph = None
    for it in range(7):
        if it == 3:
            graph = sched.capture()          # the step as one HIP graph, replayed with eager work in between
        for s in states:
            s.Y.zero_()
            s.A.zero_()
            s.EW[0].zero_()
            s.est["alpha"].zero_()
        if graph is None:
            sched.step()
        else:
            graph.replay()
        torch.cuda.synchronize()
        for s, y, a in zip(states, want, bits):
            assert torch.equal(s.A, a), (it, s.L.name)
            assert torch.equal(s.Y, y), (it, s.L.name)


@pytest.mark.parametrize("stage", [0, 1, 2, 3])
def test_config4_full(stage):
    L, x, w = wl.config4(stage)
    g = gu.gpu_layer(L, x, w)
    check_full_layer(L, x, w, None, g, count=64, seed=stage)


@pytest.mark.parametrize("which", [0, 1])
def test_config5_full(which):
    L, x, w = wl.config5(which)
    g = gu.gpu_layer(L, x, w)
    differ = check_full_layer(L, x, w, None, g, count=128, seed=which)
    assert differ <= 8        # near-ties in D among 4096 long rows are rare


# ---------------------------------------------------------------- whole tensors at full size
def _whole_layer_case(name):
    if name == "config1":
        L, x, w = wl.config1()
        return L, x, w, None
    if name == "config2":
        L, x, w = wl.config2()
        return L, x, w, x.mean(axis=(0, 2, 3)).astype(np.float32)
    if name.startswith("config3/"):
        import bench
        states = bench.build_states(256, dab, torch, wl)
        s = {t.L.name: t for t in states}[name.split("/")[1]]
        x = s.X.cpu().numpy()
        x = np.ascontiguousarray(np.transpose(x, (0, 3, 1, 2))) if x.ndim == 4 else x
        return s.L, x, s.W.cpu().numpy(), s.tau.cpu().numpy()
    if name.startswith("config4/"):
        L, x, w = wl.config4(int(name.split("/")[1]))
        return L, x, w, None
    L, x, w = wl.config5(int(name.split("/")[1]))
    return L, x, w, None


@pytest.mark.parametrize("name", ["config1", "config2", "config3/conv6", "config3/fc7", "config4/2", "config4/3", "config5/1"])
def test_whole_tensor_against_the_oracle(name):
    """One layer of every configuration at full size, every output: the integers s1 exactly and the fp32
    outputs within the tolerance, against the oracle's whole-layer float64 convolution."""
    L, x, W, tau = _whole_layer_case(name)
    g = gu.gpu_layer(L, x, W, tau)
    W4 = W.reshape(L.F, L.C, L.kh, L.kw)
    e, differ = gu.check_estimate(W4, g["est"])
    x4 = x if x.ndim == 4 else x[:, :, None, None]
    a = olay.binarize_activations(x4, tau)
    pad, stride = (L.pad, L.pad), (L.stride, L.stride)
    # integers below 2^53 are exact in the oracle's float64 sums
    s1_ref = np.rint(olay.conv2d(a, e, pad, stride)).astype(np.int64)
    sA_ref = np.rint(olay.conv2d(a, np.ones((1,) + e.shape[1:]), pad, stride)).astype(np.int64)[..., 0]
    B = x4.shape[0]
    assert np.array_equal(g["s1"].reshape(s1_ref.shape), s1_ref), "integer s1 differs"
    alpha = g["est"]["alpha"].astype(np.float64)
    beta = g["est"]["beta"].astype(np.float64)
    y_ref = olay.layer_from_integer_terms(s1_ref, sA_ref, alpha, beta)
    bound = olay.magnitude_bound(s1_ref, sA_ref, alpha, beta)
    err = np.abs(g["Y"].reshape(y_ref.shape).astype(np.float64) - y_ref)
    assert np.all(err <= gu.Y_RTOL * np.maximum(np.abs(y_ref), bound)), (name, float(err.max()))
    # and the launch without the s1 output (the one the benchmark times) writes the same Y
    g2 = gu.gpu_layer(L, x, W, tau, want_s1=False)
    assert np.array_equal(g2["Y"], g["Y"])


def _structured_masks(L, rng):
    """Masks whose products have closed forms: every tap and channel; one channel at one tap; a range of
    channels at one tap; all channels along one row of taps."""
    e = np.zeros((L.F, L.C, L.kh, L.kw), dtype=np.uint8)
    spec = []
    for f in range(L.F):
        kind = f % 4
        ky, kx = int(rng.integers(L.kh)), int(rng.integers(L.kw))
        c0 = int(rng.integers(L.C))
        c1 = int(rng.integers(c0, L.C)) + 1
        if kind == 0:
            c0, c1, taps = 0, L.C, [(i, j) for i in range(L.kh) for j in range(L.kw)]
        elif kind == 1:
            c1, taps = c0 + 1, [(ky, kx)]
        elif kind == 2:
            taps = [(ky, kx)]
        else:
            c0, c1, taps = 0, L.C, [(ky, j) for j in range(L.kw)]
        for (i, j) in taps:
            e[f, c0:c1, i, j] = 1
        spec.append((c0, c1, taps))
    return e, spec


@pytest.mark.parametrize("name,batch", [("conv2", 256), ("conv4", 256), ("conv3_b32", 32), ("stage1", 64), ("stage4", 64),
                                        ("fc_9216", 1024)])
def test_whole_tensor_closed_forms(name, batch):
    """Every output of a full-size launch against values that need no convolution at all: with masks
    that select whole windows, single weights, channel ranges or tap rows, s1 is a difference of
    channel prefix sums of the activations, shifted and added; alpha = 1.5, beta = 0.5 make
    y = s1 + sA / 2 exact in fp32.  The expected tensor is built with numpy indexing only."""
    layers = {"conv2": wl.CFG3_LAYERS[0], "conv4": wl.CFG3_LAYERS[2], "conv3_b32": wl.CFG3_LAYERS[1],
              "stage1": wl.CFG4_LAYERS[0], "stage4": wl.CFG4_LAYERS[3], "fc_9216": wl.CFG5_LAYERS[0]}
    L = layers[name]
    import zlib
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    a = (rng.integers(0, 2, size=(batch, L.C, L.H, L.W), dtype=np.int8) * 2 - 1)
    e, spec = _structured_masks(L, rng)
    E_ref, _ = opk.pack_weights(e)
    A_ref = opk.pack_activations(a)
    A = gu.to_gpu(A_ref.view(np.int32))
    E = gu.to_gpu(E_ref.view(np.int32))
    alpha = torch.full((L.F,), 1.5, dtype=torch.float32, device="cuda:0")
    beta = torch.full((L.F,), 0.5, dtype=torch.float32, device="cuda:0")
    if L.is_fc:
        Y = dab.dab_binfc(A.reshape(batch, -1), E, alpha, beta, L.C)
    else:
        d = dab.dab_conv_desc(batch, L.C, L.H, L.W, L.F, L.kh, L.kw, L.pad, L.pad, L.stride, L.stride)
        Y = dab.dab_binconv2d(d, A.reshape(batch, L.H, L.W, -1), E, alpha, beta)
    torch.cuda.synchronize()
    Y = Y.cpu().numpy().reshape(batch, L.Ho, L.Wo, L.F)
    # channel prefix sums of the zero-padded activations
    p = L.pad
    cp = np.zeros((batch, L.C + 1, L.H + 2 * p, L.W + 2 * p), dtype=np.int32)
    np.cumsum(a, axis=1, dtype=np.int32, out=cp[:, 1:, p:p + L.H, p:p + L.W])
    s = L.stride

    def window_sum(plane, taps):
        out = np.zeros((batch, L.Ho, L.Wo), dtype=np.int32)
        for (i, j) in taps:
            out += plane[:, i:i + s * (L.Ho - 1) + 1:s, j:j + s * (L.Wo - 1) + 1:s]
        return out

    all_taps = [(i, j) for i in range(L.kh) for j in range(L.kw)]
    sA = window_sum(cp[:, L.C], all_taps)
    cache = {}
    for f, (c0, c1, taps) in enumerate(spec):
        key = (c0, c1, tuple(taps))
        if key not in cache:
            cache[key] = window_sum(cp[:, c1] - cp[:, c0], taps)
        want = cache[key].astype(np.float32) + 0.5 * sA.astype(np.float32)
        assert np.array_equal(Y[..., f], want), (name, f, spec[f][:2])
