"""Pins for the oracle's step between two binarized layers (pool, then sign)."""
import numpy as np
import torch

from oracle import layers as olay
from oracle import packing as opk


def test_max_pool_against_library_routine():
    rng = np.random.default_rng(5)
    for (H, W, kh, kw, sh, sw) in [(31, 31, 3, 3, 2, 2), (15, 15, 3, 3, 2, 2), (9, 7, 2, 3, 1, 2), (5, 5, 5, 5, 1, 1)]:
        y = rng.standard_normal((3, H, W, 6))
        ref = torch.nn.functional.max_pool2d(torch.from_numpy(y).permute(0, 3, 1, 2), (kh, kw), (sh, sw))
        got = olay.max_pool(y, kh, kw, sh, sw)
        assert np.array_equal(got, ref.permute(0, 2, 3, 1).numpy())


def test_sign_of_pooled_output_is_or_of_signs():
    """sign(max(y) - tau) = OR of sign(y - tau): what lets pooling run on packed bits."""
    rng = np.random.default_rng(6)
    y = np.round(rng.standard_normal((2, 11, 9, 40)) * 4) / 4        # many exact ties with the thresholds
    tau = np.round(rng.standard_normal(40) * 2) / 4
    pooled = olay.next_layer_input(y, tau, pool=(3, 3, 2, 2))        # definition: pool, then sign
    bits = opk.pack_activations(olay.next_layer_input(y, tau))       # sign first, packed
    B, H, W, Cw = bits.shape
    Ho, Wo = (H - 3) // 2 + 1, (W - 3) // 2 + 1
    ored = np.zeros((B, Ho, Wo, Cw), dtype=np.uint32)
    for ky in range(3):
        for kx in range(3):
            ored |= bits[:, ky:ky + (Ho - 1) * 2 + 1:2, kx:kx + (Wo - 1) * 2 + 1:2, :]
    assert np.array_equal(ored, opk.pack_activations(pooled))


def test_hand_example():
    # one channel, 3x3 window over a 3x4 image, stride 1: windows are columns 0..2 and 1..3
    y = np.array([[-1.0, -2.0, -3.0, 0.5], [-1.5, -0.25, -4.0, -5.0], [-2.0, -6.0, -7.0, -8.0]]).reshape(1, 3, 4, 1)
    a = olay.next_layer_input(y, np.array([0.0]), pool=(3, 3, 1, 1))
    assert a.shape == (1, 1, 1, 2) and a.reshape(-1).tolist() == [-1, 1]      # maxima -0.25 and 0.5
    a = olay.next_layer_input(y, np.array([-0.25]), pool=(3, 3, 1, 1))
    assert a.reshape(-1).tolist() == [1, 1]                                    # -0.25 >= -0.25
