"""Pins of the reference packers (CPU only): hand-typed words and round trips."""
import json
import os

import numpy as np

from oracle import packing as pk


def test_bit_order_golden(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "bit_order.json")))
    ga = g["activations"]
    a = -np.ones((1, ga["C"]), dtype=np.int8)
    a[0, ga["plus_one_channels"]] = 1
    words = pk.pack_activations(a)
    assert words.dtype == np.uint32 and words.shape == (1, 2)
    assert [int(w) for w in words[0]] == [int(s, 16) for s in ga["words"]]
    assert np.array_equal(pk.pack_activations(a[:, :, None, None])[0, 0, 0], words[0])

    gw = g["weights"]
    e = np.zeros((gw["F"], gw["C"], gw["kh"], gw["kw"]), dtype=np.uint8)
    for f, c, ky, kx in gw["ones"]:
        e[f, c, ky, kx] = 1
    E, ecnt = pk.pack_weights(e)
    assert E.shape == (gw["rows"], gw["columns"]) and E.dtype == np.uint32
    want = np.zeros_like(E)
    for key, val in gw["nonzero_words"].items():
        r, f = map(int, key.split(","))
        want[r, f] = int(val, 16)
    assert np.array_equal(E, want)
    assert ecnt.tolist() == gw["ecnt"]


def test_round_trip_and_tails():
    rng = np.random.default_rng(4)
    for C in (1, 31, 32, 33, 64, 100):
        a = np.where(rng.random((2, C, 3, 2)) < 0.5, 1, -1).astype(np.int8)
        A = pk.pack_activations(a)
        assert A.shape == (2, 3, 2, pk.words_per_pixel(C))
        assert np.array_equal(pk.unpack_activations(A, C), a)
        if C % 32:
            assert np.all(A[..., -1] >> np.uint32(C % 32) == 0)
        assert int(pk.popcount32(A).sum()) == int((a == 1).sum())


def test_popcount():
    xs = np.array([0, 1, 0x80000000, 0xFFFFFFFF, 0x12345678], dtype=np.uint32)
    assert pk.popcount32(xs).tolist() == [bin(int(x)).count("1") for x in xs]


def test_weight_layout_is_word_major():
    rng = np.random.default_rng(8)
    F, C, kh, kw = 70, 45, 2, 3
    e = (rng.random((F, C, kh, kw)) < 0.3).astype(np.uint8)
    E, ecnt = pk.pack_weights(e)
    Cw = 2
    assert E.shape == (kh * kw * Cw, 128) and np.all(E[:, F:] == 0)
    assert np.array_equal(ecnt, e.sum(axis=1).reshape(F, kh * kw))
    f, c, ky, kx = 69, 44, 1, 2
    assert (int(E[(ky * kw + kx) * Cw + 1, f]) >> (44 - 32)) & 1 == e[f, c, ky, kx]
    assert int(pk.popcount32(E).sum()) == int(e.sum())
