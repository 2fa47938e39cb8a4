"""The grouped entry points: several layers' weight sides in one call (dab_binarize_weights_multi).

Every job's estimate is checked against the oracle filter by filter (as in test_gpu_parity.py) and its
packed mask and per-tap counts bit for bit against the oracle's packing of the mask the estimate
implies; the call with a previous split is checked against the oracle's restricted search."""
import numpy as np
import pytest
import torch

from oracle import packing as opk
from paper_1804_02941_amd import binding as dab
from paper_1804_02941_amd import workloads as wl

import gpu_util as gu
from test_gpu_parity import weight_rows
from test_gpu_training import check_bounded

pytestmark = pytest.mark.gpu

# (F, C, kh, kw, kind): short rows down to two weights, rows around the limits of the kernels, long
# rows including ones the value buckets hand over to the sort (few distinct values), filter counts
# that are not multiples of 64
JOBS = [(70, 45, 2, 3, "dupes"), (5, 3, 1, 1, "gauss"), (64, 64, 3, 3, "mixture"), (130, 100, 5, 5, "laplace"),
        (9, 256, 7, 7, "gauss"), (33, 5000, 1, 1, "dupes"), (40, 512, 1, 1, "mixture"), (3, 2, 1, 1, "onesided"),
        (17, 4608, 1, 1, "gauss"), (6, 4609, 1, 1, "mixture"), (4, 13312, 1, 1, "laplace"), (12, 256, 3, 3, "onesided")]


def make_items(rng, with_packing=True):
    items, Ws = [], []
    for (F, C, kh, kw, kind) in JOBS:
        W = weight_rows(rng, F, C * kh * kw, kind).reshape(F, C, kh, kw)
        if kind == "dupes":
            W[0] = 0.25                                           # a constant filter
        Ws.append(W)
        Wt = gu.to_gpu(W)
        items.append(dict(W=Wt, est=dab.estimate_outputs(F, Wt.device),
                          packed=dab.pack_weights_outputs(F, C, kh, kw, Wt.device) if with_packing else None))
    return items, Ws


def test_binarize_weights_multi_against_the_oracle():
    rng = np.random.default_rng(2024)
    items, Ws = make_items(rng)
    for it in items:                                              # every word must be written by the call
        it["packed"][0].fill_(-1)
        it["packed"][1].fill_(-1)
    dab.dab_binarize_weights_multi(dab.weight_jobs(items))
    torch.cuda.synchronize()
    for it, W in zip(items, Ws):
        got = {k: v.cpu().numpy() for k, v in it["est"].items()}
        e, differ = gu.check_estimate(W, got)
        assert differ <= 1
        E_ref, ecnt_ref = opk.pack_weights(e)
        assert np.array_equal(gu.u32(it["packed"][0]), E_ref), W.shape
        assert np.array_equal(gu.u32(it["packed"][1]), ecnt_ref), W.shape


def test_binarize_weights_multi_equals_separate_calls_and_runs_without_packing():
    rng = np.random.default_rng(2025)
    items, Ws = make_items(rng)
    dab.dab_binarize_weights_multi(dab.weight_jobs(items))
    bare, _ = make_items(np.random.default_rng(2025), with_packing=False)
    dab.dab_binarize_weights_multi(dab.weight_jobs(bare))
    torch.cuda.synchronize()
    for it, b, W in zip(items, bare, Ws):
        for k in it["est"]:
            assert torch.equal(it["est"][k], b["est"][k]), k       # packing changes nothing of the estimate
        # the packing of the separate call, fed this estimate
        E, ecnt = dab.dab_pack_weights(it["W"], it["est"]["thr_val"], it["est"]["thr_idx"], it["est"]["alpha_is_upper"])
        torch.cuda.synchronize()
        assert torch.equal(E, it["packed"][0]) and torch.equal(ecnt, it["packed"][1])


def test_binarize_weights_multi_with_previous_split():
    rng = np.random.default_rng(2026)
    shapes = [(24, 64, 3, 3), (10, 700, 3, 3), (16, 128, 5, 5)]
    items, W1 = [], []
    for (F, C, kh, kw) in shapes:
        n = C * kh * kw
        w0 = wl.skewed_mixture_weights(rng, rng, F, n, n)
        prev = dab.dab_estimate_alpha_beta(gu.to_gpu(w0))
        w1 = (w0 + 0.05 * np.float32(np.sqrt(2.0 / n)) * rng.standard_normal((F, n))).astype(np.float32)
        W1.append((w1, prev["K"].cpu().numpy(), prev["alpha_is_upper"].cpu().numpy()))
        Wt = gu.to_gpu(w1.reshape(F, C, kh, kw))
        items.append(dict(W=Wt, est=dab.estimate_outputs(F, Wt.device), packed=dab.pack_weights_outputs(F, C, kh, kw, Wt.device),
                          prev=(prev["K"], prev["alpha_is_upper"], max(2, n // 50))))
    dab.dab_binarize_weights_multi(dab.weight_jobs(items))
    torch.cuda.synchronize()
    for it, (w1, Kp, up), (F, C, kh, kw) in zip(items, W1, shapes):
        check_bounded(w1, {k: v.cpu().numpy() for k, v in it["est"].items()}, Kp, up, max(2, C * kh * kw // 50))


def test_binarize_weights_multi_errors():
    lib = dab.lib()
    rng = np.random.default_rng(1)
    items, _ = make_items(rng)
    jobs = dab.weight_jobs(items)
    assert lib.dab_binarize_weights_multi(None, 1, None, 0, None) == dab.DAB_ERR_NULL
    assert lib.dab_binarize_weights_multi(jobs, 0, None, 0, None) == dab.DAB_ERR_SHAPE
    assert lib.dab_binarize_weights_multi(jobs, 17, None, 0, None) == dab.DAB_ERR_UNSUPPORTED
    assert lib.dab_binarize_weights_multi_workspace_bytes(jobs, len(jobs)) > 0
    assert lib.dab_binarize_weights_multi(jobs, len(jobs), None, 0, None) == dab.DAB_ERR_WORKSPACE   # long rows need the flags
    assert lib.dab_binarize_weights_multi_workspace_bytes(jobs, 3) == 0                            # short rows only
    torch.cuda.synchronize()


# ---------------------------------------------------------------- weight side and activation packing in the same launches
# (B, C, H, W, with thresholds): channel counts on the aligned fast path and off it, one tensor smaller than a batch
PACK_SHAPES = [(7, 64, 9, 11, True), (3, 37, 5, 6, True), (16, 256, 6, 6, False), (5, 100, 4, 4, True), (33, 512, 1, 1, False),
               (2, 1024, 3, 3, True), (1, 64, 1, 1, False)]


def make_pack_items(rng):
    items = []
    for (B, C, H, W, thr) in PACK_SHAPES:
        x = rng.standard_normal((B, H, W, C)).astype(np.float32)
        X = gu.to_gpu(x if H * W > 1 else x.reshape(B, C))
        tau = gu.to_gpu(rng.standard_normal(C).astype(np.float32) * 0.3) if thr else None
        A = torch.full((B, H, W, dab.words_per_pixel(C)), -1, dtype=torch.int32, device=X.device)
        items.append((X, tau, A if H * W > 1 else A.reshape(B, -1)))
    return items


@pytest.mark.parametrize("subset", ["all", "short rows only", "long rows only"])
def test_prepare_layers_equals_the_two_separate_calls(subset):
    rng = np.random.default_rng(77)
    w_all, _ = make_items(rng)
    keep = {"all": lambda n: True, "short rows only": lambda n: n <= 2304, "long rows only": lambda n: n > 4608}[subset]
    w_items = [it for it in w_all if keep(it["W"][0].numel())]
    p_items = make_pack_items(rng)
    dab.dab_prepare_layers(dab.weight_jobs(w_items), dab.pack_jobs(p_items))
    torch.cuda.synchronize()
    # the same inputs through the two separate calls
    w_ref = [dict(W=it["W"], est=dab.estimate_outputs(it["W"].shape[0], it["W"].device),
                  packed=dab.pack_weights_outputs(*it["W"].shape, it["W"].device)) for it in w_items]
    p_ref = [(X, tau, torch.empty_like(A)) for (X, tau, A) in p_items]
    dab.dab_binarize_weights_multi(dab.weight_jobs(w_ref))
    dab.dab_pack_activations_multi(dab.pack_jobs(p_ref))
    torch.cuda.synchronize()
    for a, b in zip(w_items, w_ref):
        for k in a["est"]:
            assert torch.equal(a["est"][k], b["est"][k]), k
        assert torch.equal(a["packed"][0], b["packed"][0]) and torch.equal(a["packed"][1], b["packed"][1])
    for (_, _, A), (_, _, R), shape in zip(p_items, p_ref, PACK_SHAPES):
        assert torch.equal(A, R), shape


def test_prepare_layers_errors():
    lib = dab.lib()
    rng = np.random.default_rng(3)
    w_items, _ = make_items(rng)
    p_items = make_pack_items(rng)
    wj, pj = dab.weight_jobs(w_items), dab.pack_jobs(p_items)
    assert lib.dab_prepare_layers(None, 1, pj, 1, None, 0, None) == dab.DAB_ERR_NULL
    assert lib.dab_prepare_layers(wj, 1, None, 1, None, 0, None) == dab.DAB_ERR_NULL
    assert lib.dab_prepare_layers(wj, 0, pj, 1, None, 0, None) == dab.DAB_ERR_SHAPE
    assert lib.dab_prepare_layers(wj, len(wj), pj, 17, None, 0, None) == dab.DAB_ERR_UNSUPPORTED
    assert lib.dab_prepare_layers(wj, len(wj), pj, len(pj), None, 0, None) == dab.DAB_ERR_WORKSPACE   # long rows need the flags
    few = dab.weight_jobs([dict(W=gu.to_gpu(np.ones((2, 3, 1, 1), np.float32)), est=dab.estimate_outputs(2, "cuda:0"), packed=None)])
    assert lib.dab_prepare_layers(few, 1, pj, len(pj), None, 0, None) == dab.DAB_ERR_UNSUPPORTED    # fewer filters than tensors
    torch.cuda.synchronize()


def test_many_medium_rows_are_handed_to_the_sort_kernel():
    """From 1536 rows of 2305..4608 weights on, rows the buckets cannot finish are flagged for the sort kernel
    instead of being sorted in place; results are those of the separate calls, degenerate rows included."""
    rng = np.random.default_rng(99)
    F, n = 1600, 2400
    W = weight_rows(rng, F, n, "gauss")
    W[3] = 0.5                                                     # a constant row
    W[10::97] = np.round(W[10::97] * 8) / 8                        # rows with few distinct values
    W2 = weight_rows(rng, 40, 4608, "mixture")
    items = []
    for w, shape in ((W, (F, 800, 1, 3)), (W2, (40, 512, 3, 3))):
        Wt = gu.to_gpu(w.reshape(shape))
        items.append(dict(W=Wt, est=dab.estimate_outputs(shape[0], Wt.device), packed=dab.pack_weights_outputs(*shape, Wt.device)))
    jobs = dab.weight_jobs(items)
    assert dab.lib().dab_binarize_weights_multi_workspace_bytes(jobs, len(jobs)) > 0
    dab.dab_binarize_weights_multi(jobs)
    torch.cuda.synchronize()
    for it, w in zip(items, (W, W2)):
        ref = dab.dab_estimate_alpha_beta(it["W"].reshape(it["W"].shape[0], -1))
        E, ecnt = dab.dab_pack_weights(it["W"], ref["thr_val"], ref["thr_idx"], ref["alpha_is_upper"])
        torch.cuda.synchronize()
        for k in ref:
            assert torch.equal(it["est"][k], ref[k]), k
        assert torch.equal(E, it["packed"][0]) and torch.equal(ecnt, it["packed"][1])
    got = {k: v.cpu().numpy() for k, v in items[0]["est"].items()}
    gu.check_estimate(W[:64], {k: v[:64] for k, v in got.items()})
