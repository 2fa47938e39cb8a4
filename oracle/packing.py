"""Oracle (test infrastructure): reference bit packers.

The paper (arXiv 1804.02941) stores one bit per weight plus two scalars per
filter (Section 4.4: only the binarized weights are kept for inference) and
assumes binary inputs (Section 4); it fixes no storage order.  The order below
is this repository's, stated once here and once in the C header, and the two
sides implement it independently:

Activations   uint32 [B][H][W][Cw], Cw = ceil(C/32).  Bit (c mod 32), counted
              from the least significant bit, of word (c div 32) of pixel
              (b,h,w) is 1 iff a[b,c,h,w] = +1.  Bits past C are 0.
              A fully-connected input is the case H = W = 1.
Weights       uint32 [R][Fp], R = kh*kw*Cw, Fp = 64*ceil(F/64).  Row
              r = (ky*kw + kx)*Cw + (c div 32), column f, bit (c mod 32) is
              e[f,c,ky,kx].  Bits past C and columns past F are 0.
Tap counts    uint32 [F][kh*kw]: ecnt[f][ky*kw+kx] = sum_c e[f,c,ky,kx].
"""
from __future__ import annotations

import numpy as np


def words_per_pixel(C: int) -> int:
    return (C + 31) // 32


def padded_filters(F: int) -> int:
    return 64 * ((F + 63) // 64)


def pack_activations(a_pm1: np.ndarray) -> np.ndarray:
    """[B,C,H,W] (or [B,C]) of +1/-1  ->  uint32 [B,H,W,Cw] (or [B,Cw])."""
    a = np.asarray(a_pm1)
    flat = a.ndim == 2
    if flat:
        a = a[:, :, None, None]
    B, C, H, W = a.shape
    Cw = words_per_pixel(C)
    out = np.zeros((B, H, W, Cw), dtype=np.uint32)
    for c in range(C):
        bit = (a[:, c, :, :] == 1).astype(np.uint32)
        out[:, :, :, c // 32] |= bit << np.uint32(c % 32)
    return out[:, 0, 0, :] if flat else out


def pack_weights(e: np.ndarray):
    """[F,C,kh,kw] (or [F,K]) of 0/1  ->  (uint32 [R,Fp], uint32 ecnt [F,kh*kw])."""
    e = np.asarray(e)
    if e.ndim == 2:
        e = e[:, :, None, None]
    F, C, kh, kw = e.shape
    Cw = words_per_pixel(C)
    Fp = padded_filters(F)
    E = np.zeros((kh * kw * Cw, Fp), dtype=np.uint32)
    ecnt = np.zeros((F, kh * kw), dtype=np.uint32)
    for ky in range(kh):
        for kx in range(kw):
            tap = ky * kw + kx
            for c in range(C):
                bit = (e[:, c, ky, kx] != 0).astype(np.uint32)
                E[tap * Cw + c // 32, :F] |= bit << np.uint32(c % 32)
                ecnt[:, tap] += bit
    return E, ecnt


def unpack_activations(A: np.ndarray, C: int) -> np.ndarray:
    """Inverse of pack_activations for a [B,H,W,Cw] array: +1/-1 as [B,C,H,W]."""
    A = np.asarray(A, dtype=np.uint32)
    B, H, W, _ = A.shape
    out = np.empty((B, C, H, W), dtype=np.int8)
    for c in range(C):
        out[:, c] = np.where((A[..., c // 32] >> np.uint32(c % 32)) & np.uint32(1), 1, -1)
    return out


def popcount32(x: np.ndarray) -> np.ndarray:
    """Number of set bits of every uint32 element (bit by bit)."""
    x = np.asarray(x, dtype=np.uint32)
    n = np.zeros(x.shape, dtype=np.int64)
    for k in range(32):
        n += (x >> np.uint32(k)) & np.uint32(1)
    return n
