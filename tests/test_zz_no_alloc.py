"""dab_estimate_alpha_beta_noalloc: the estimator with its scratch in the library's own device array.

Called through the C ABI (ctypes, raw pointers) and compared, bit for bit, with dab_estimate_alpha_beta
run with a caller's workspace, on two calls in a row of which the second is smaller: the array keeps
the first call's flags, and nothing of them may leak into the second result.
"""
import numpy as np
import pytest
import torch

from paper_1804_02941_amd import binding as dab

import gpu_util as gu

pytestmark = pytest.mark.gpu


def rows(rng, F, n):
    """Gaussian rows, with every third row made of few distinct values: the value buckets cannot finish
    those, so they are handed over through the flags to the sort kernel."""
    W = (rng.standard_normal((F, n)) * 0.05).astype(np.float32)
    W[::3] = (np.round(rng.standard_normal((len(W[::3]), n)) * 6) / 16).astype(np.float32)
    W[1] = 0.25                                               # a constant row
    return W


def noalloc(Wt):
    F, n = Wt.shape
    out = dab.estimate_outputs(F, Wt.device)
    rc = dab.lib().dab_estimate_alpha_beta_noalloc(
        Wt.data_ptr(), F, n, out["alpha"].data_ptr(), out["beta"].data_ptr(), out["K"].data_ptr(),
        out["thr_val"].data_ptr(), out["thr_idx"].data_ptr(), out["alpha_is_upper"].data_ptr(), None)
    assert rc == 0, dab.lib().dab_strerror(rc)
    return out


def test_noalloc_matches_workspace_entry_point_on_two_calls():
    lib = dab.lib()
    assert lib.dab_init() == 0
    rng = np.random.default_rng(77)
    for F, n in ((300, 6000), (41, 4500)):                    # second call smaller, in both sizes
        W = rows(rng, F, n)
        Wt = gu.to_gpu(W)
        ref = dab.dab_estimate_alpha_beta(Wt)                 # caller's workspace
        got = noalloc(Wt)
        torch.cuda.synchronize()
        for key in ref:
            assert torch.equal(ref[key], got[key]), f"F={F} n={n}: {key} differs"
        pick = np.concatenate([np.arange(6), rng.choice(F, size=6, replace=False)])
        gu.check_estimate(W[pick], {k: v.cpu().numpy()[pick] for k, v in got.items()})


def test_noalloc_short_rows_and_limits():
    lib = dab.lib()
    rng = np.random.default_rng(78)
    W = rows(rng, 50, 700)                                    # short rows: no flags involved
    Wt = gu.to_gpu(W)
    ref = dab.dab_estimate_alpha_beta(Wt)
    got = noalloc(Wt)
    torch.cuda.synchronize()
    for key in ref:
        assert torch.equal(ref[key], got[key])
    # beyond the array: a clear error, before anything is launched
    fake = 4096
    too_many = lib.dab_estimate_noalloc_max_filters() + 1
    assert lib.dab_estimate_alpha_beta_noalloc(fake, too_many, 5000, fake, fake, fake, fake, fake, fake, None) == 5
    assert lib.dab_estimate_alpha_beta_noalloc(None, 4, 5000, fake, fake, fake, fake, fake, fake, None) == 1
    assert lib.dab_estimate_alpha_beta_noalloc(fake, 4, 1, fake, fake, fake, fake, fake, fake, None) == 2
