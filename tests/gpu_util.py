"""Helpers for the GPU parity tests: run one layer through the C ABI and through the oracle."""
import numpy as np
import torch

from oracle import estimate as oest
from oracle import layers as olay
from oracle import packing as opk
from paper_1804_02941_amd import binding as dab

DEV = "cuda:0"
# fp32 epilogue: Y is compared with the float64 oracle to this relative tolerance, measured
# against max(|y|, |alpha||s1| + |beta||s2|) (the scale a two-term fp32 sum is accurate to).
Y_RTOL = 1e-5
# alpha and beta are single fp64 means rounded once to fp32.
AB_RTOL = 1e-6
# the score D is flat near its maximum; a split is accepted if its D is this close to the best
D_RTOL = 1e-12


def to_gpu(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(DEV)


def u32(t):
    """int32 tensor from the binding -> numpy uint32."""
    return t.cpu().numpy().view(np.uint32)


def gpu_estimate(W):
    """W numpy [F, ...] -> dict of numpy arrays from dab_estimate_alpha_beta."""
    F = W.shape[0]
    out = dab.dab_estimate_alpha_beta(to_gpu(W.reshape(F, -1)))
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in out.items()}, out


def check_estimate(W, got):
    """Compare the GPU estimate with the oracle, filter by filter.

    Returns the masks e implied by the GPU's split descriptors (the oracle's own when the
    splits agree), the number of filters whose split differs (near-ties only).
    """
    F = W.shape[0]
    W2 = W.reshape(F, -1)
    n = W2.shape[1]
    e = np.empty((F, n), dtype=np.uint8)
    differ = 0
    for f in range(F):
        r = oest.estimate_filter(W2[f])
        upper = int(got["alpha_is_upper"][f])
        K = int(got["K"][f])
        i_gpu = n - K if upper else K
        tv, ti = float(got["thr_val"][f]), int(got["thr_idx"][f])
        low = oest.lower_group_from_descriptor(W2[f], tv, ti)
        assert int(low.sum()) == i_gpu, f"filter {f}: descriptor gives {low.sum()} lower elements, K says {i_gpu}"
        assert 1 <= i_gpu <= n - 1
        if i_gpu != r["i_star"]:
            differ += 1
            d_gpu = oest.score_of_split(W2[f], i_gpu)
            assert d_gpu >= r["maxD"] * (1 - D_RTOL), f"filter {f}: split {i_gpu} vs {r['i_star']} is not a near-tie"
            # the descriptor must still describe the i_gpu smallest elements in stable order
            order = oest.stable_order(W2[f])
            ref_low = np.zeros(n, bool)
            ref_low[order[:i_gpu]] = True
            assert np.array_equal(low, ref_low)
            w64 = W2[f].astype(np.float64)
            mu_l, mu_u = w64[low].mean(), w64[~low].mean()
            want_upper = 1 if abs(mu_u) >= abs(mu_l) else 0
            a_ref, b_ref = (mu_u, mu_l) if want_upper else (mu_l, mu_u)
        else:
            assert (tv, ti) == (np.float32(r["thr_val"]), r["thr_idx"]), f"filter {f}: descriptor differs"
            want_upper, a_ref, b_ref = r["alpha_is_upper"], r["alpha"], r["beta"]
        if abs(abs(a_ref) - abs(b_ref)) > 1e-12 * abs(a_ref):   # labelling is decided by a clear margin
            assert upper == want_upper, f"filter {f}: labelling"
        else:
            a_ref, b_ref = (a_ref, b_ref) if upper == want_upper else (b_ref, a_ref)
        assert abs(got["alpha"][f] - a_ref) <= AB_RTOL * abs(a_ref) + 1e-30, f"filter {f}: alpha"
        assert abs(got["beta"][f] - b_ref) <= AB_RTOL * abs(b_ref) + 1e-30, f"filter {f}: beta"
        e[f] = (~low if upper else low)
    return e.reshape(W.shape), differ


def gpu_layer(L, x_nchw, W, tau=None, layout="nhwc", want_s1=True):
    """Full GPU path for one layer: estimate, pack weights, pack activations, binary product.

    Returns a dict with numpy copies of every intermediate.
    """
    est_np, est = gpu_estimate(W)
    W4 = W.reshape(L.F, L.C, L.kh, L.kw)
    E, ecnt = dab.dab_pack_weights(to_gpu(W4), est["thr_val"], est["thr_idx"], est["alpha_is_upper"])
    tau_t = to_gpu(tau) if tau is not None else None
    if x_nchw.ndim == 2:
        A = dab.dab_pack_activations(to_gpu(x_nchw), dab.DAB_LAYOUT_NHWC, tau_t)
    elif layout == "nhwc":
        A = dab.dab_pack_activations(to_gpu(np.transpose(x_nchw, (0, 2, 3, 1))), dab.DAB_LAYOUT_NHWC, tau_t)
    else:
        A = dab.dab_pack_activations(to_gpu(x_nchw), dab.DAB_LAYOUT_NCHW, tau_t)
    B = x_nchw.shape[0]
    if L.is_fc:
        res = dab.dab_binfc(A.reshape(B, -1), E, est["alpha"], est["beta"], L.C, want_s1=want_s1)
    else:
        d = dab.dab_conv_desc(B, L.C, L.H, L.W, L.F, L.kh, L.kw, L.pad, L.pad, L.stride, L.stride)
        res = dab.dab_binconv2d(d, A, E, est["alpha"], est["beta"], want_s1=want_s1)
    torch.cuda.synchronize()
    Y, s1 = res if want_s1 else (res, None)
    return dict(est=est_np, E=u32(E), ecnt=u32(ecnt), A=u32(A), Y=Y.cpu().numpy(),
                s1=None if s1 is None else s1.cpu().numpy(), Y_gpu=Y)


def check_layer(L, x_nchw, W, tau=None, layout="nhwc"):
    """Element-by-element parity of one layer against the oracle (small shapes)."""
    B = x_nchw.shape[0]
    g = gpu_layer(L, x_nchw, W, tau, layout)
    W4 = W.reshape(L.F, L.C, L.kh, L.kw)
    e, differ = check_estimate(W4, g["est"])
    # packed weights and counts, bit for bit
    E_ref, ecnt_ref = opk.pack_weights(e)
    assert np.array_equal(g["E"], E_ref), "packed weight bits differ"
    assert np.array_equal(g["ecnt"], ecnt_ref), "per-tap counts differ"
    # packed activations, bit for bit
    x4 = x_nchw if x_nchw.ndim == 4 else x_nchw[:, :, None, None]
    a = olay.binarize_activations(x4, tau)
    A_ref = opk.pack_activations(a)
    assert np.array_equal(g["A"].reshape(A_ref.shape), A_ref), "packed activation bits differ"
    # integers exactly, fp32 output within tolerance of the float64 layer
    pad, stride = (L.pad, L.pad), (L.stride, L.stride)
    s1_ref, sA_ref = olay.integer_terms(a, e, pad, stride)
    assert np.array_equal(g["s1"].reshape(s1_ref.shape), s1_ref), "integer s1 differs"
    alpha = g["est"]["alpha"].astype(np.float64)
    beta = g["est"]["beta"].astype(np.float64)
    Wt = olay.two_valued_filters(e, alpha, beta)
    y_ref = olay.conv2d(a, Wt, pad, stride)
    y_int = olay.layer_from_integer_terms(s1_ref, sA_ref, alpha, beta)
    bound = olay.magnitude_bound(s1_ref, sA_ref, alpha, beta)
    assert np.all(np.abs(y_ref - y_int) <= 1e-9 * np.maximum(bound, 1e-300) + 1e-12 * np.abs(Wt).reshape(L.F, -1).sum(1))
    err = np.abs(g["Y"].reshape(y_ref.shape).astype(np.float64) - y_ref)
    tol = Y_RTOL * np.maximum(np.abs(y_ref), bound)
    assert np.all(err <= tol), f"max err/tol = {np.max(err / np.maximum(tol, 1e-300))}"
    return dict(differ=differ, max_rel=float(np.max(err / np.maximum(np.maximum(np.abs(y_ref), bound), 1e-300))))
