"""ctypes binding of libdab_hip.so: argument marshalling only.

Every function here has the name of the C entry point it calls (see
``include/dab.h``) and does nothing but check tensor dtype / device /
contiguity, allocate the output tensors with ``torch.empty`` and pass raw
device pointers plus the current HIP stream.  All arithmetic of the path runs in
the HIP kernels.  There is no CPU fallback: if the library is not built, or a
tensor is not on the GPU, the call raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import c_char_p, c_float, c_int, c_int32, c_size_t, c_void_p

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libdab_hip.so")

DAB_OK = 0
DAB_ERR_NULL, DAB_ERR_SHAPE, DAB_ERR_ALIGN, DAB_ERR_WORKSPACE, DAB_ERR_UNSUPPORTED, DAB_ERR_HIP = 1, 2, 3, 4, 5, 6
DAB_LAYOUT_NHWC = 0
DAB_LAYOUT_NCHW = 1


class DabError(RuntimeError):
    def __init__(self, name, status, text):
        super().__init__(f"{name} failed: status {status} ({text})")
        self.status = status


class dab_conv_desc(ctypes.Structure):
    _fields_ = [(k, c_int32) for k in
                ("B", "C", "H", "W", "F", "kh", "kw", "pad_h", "pad_w", "stride_h", "stride_w")]

    @property
    def Ho(self):
        return (self.H + 2 * self.pad_h - self.kh) // self.stride_h + 1

    @property
    def Wo(self):
        return (self.W + 2 * self.pad_w - self.kw) // self.stride_w + 1


_SIGNATURES = {
    "dab_strerror": (c_char_p, [c_int]),
    "dab_last_hip_error": (c_int, []),
    "dab_init": (c_int, []),
    "dab_probe_popcount": (c_int, [c_int, c_int, c_int, c_void_p, c_void_p, ctypes.POINTER(ctypes.c_int64),
                                   ctypes.POINTER(c_int32), c_void_p]),
    "dab_estimate_alpha_beta": (c_int, [c_void_p, c_int32, c_int32, c_void_p, c_void_p, c_void_p, c_void_p,
                                        c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]),
    "dab_estimate_alpha_beta_bounded": (c_int, [c_void_p, c_int32, c_int32, c_void_p, c_void_p, c_int32, c_void_p,
                                                c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t,
                                                c_void_p]),
    "dab_estimate_sign_split": (c_int, [c_void_p, c_int32, c_int32, c_void_p, c_void_p, c_void_p, c_void_p,
                                        c_void_p, c_void_p, c_void_p]),
    "dab_estimate_alpha_beta_noalloc": (c_int, [c_void_p, c_int32, c_int32, c_void_p, c_void_p, c_void_p, c_void_p,
                                                c_void_p, c_void_p, c_void_p]),
    "dab_estimate_noalloc_max_filters": (c_int32, []),
    "dab_estimate_workspace_bytes": (c_size_t, [c_int32, c_int32]),
    "dab_estimate_max_n": (c_int32, []),
    "dab_pack_weights": (c_int, [c_void_p, c_int32, c_int32, c_int32, c_int32, c_void_p, c_void_p, c_void_p,
                                 c_void_p, c_void_p, c_void_p]),
    "dab_pack_activations": (c_int, [c_void_p, c_int32, c_int32, c_int32, c_int32, c_int32, c_void_p, c_void_p,
                                     c_void_p]),
    "dab_pack_activations_multi": (c_int, [c_void_p, c_int32, c_void_p]),
    "dab_binarize_weights_multi": (c_int, [c_void_p, c_int32, c_void_p, c_size_t, c_void_p]),
    "dab_binarize_weights_multi_workspace_bytes": (c_size_t, [c_void_p, c_int32]),
    "dab_prepare_layers": (c_int, [c_void_p, c_int32, c_void_p, c_int32, c_void_p, c_size_t, c_void_p]),
    "dab_binconv2d": (c_int, [ctypes.POINTER(dab_conv_desc), c_void_p, c_void_p, c_void_p, c_void_p,
                              c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]),
    "dab_binconv2d_workspace_bytes": (c_size_t, [ctypes.POINTER(dab_conv_desc)]),
    "dab_binfc": (c_int, [c_int32, c_int32, c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                          c_void_p, c_void_p, c_size_t, c_void_p]),
    "dab_binfc_workspace_bytes": (c_size_t, [c_int32, c_int32, c_int32]),
    "dab_binconv2d_bits": (c_int, [ctypes.POINTER(dab_conv_desc), c_void_p, c_void_p, c_void_p, c_void_p,
                                   c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]),
    "dab_binfc_bits": (c_int, [c_int32, c_int32, c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                               c_void_p, c_void_p, c_size_t, c_void_p]),
    "dab_pool_bits": (c_int, [c_void_p, c_int32, c_int32, c_int32, c_int32, c_int32, c_int32, c_int32, c_int32,
                              c_void_p, c_void_p]),
    "dab_wbin_conv2d_workspace_bytes": (c_size_t, [ctypes.POINTER(dab_conv_desc)]),
    "dab_wbin_fc_workspace_bytes": (c_size_t, [c_int32, c_int32, c_int32]),
    "dab_wbin_conv2d": (c_int, [ctypes.POINTER(dab_conv_desc), c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                c_void_p, c_size_t, c_void_p]),
    "dab_wbin_fc": (c_int, [c_int32, c_int32, c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                            c_size_t, c_void_p]),
    "dab_mean_center_clamp": (c_int, [c_void_p, c_int32, c_int32, c_int32, c_int32, c_float, c_float, c_void_p,
                                      c_void_p]),
    "dab_binarized_weights": (c_int, [c_void_p, c_int32, c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                      c_void_p, c_void_p]),
    "dab_weight_gradient": (c_int, [c_void_p, c_int32, c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                    c_void_p]),
}

_lib = None


def lib() -> ctypes.CDLL:
    """The loaded shared library (opened on first use; raises if it was never built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_1804_02941_amd.build` first")
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def _check(name, status):
    if status != DAB_OK:
        raise DabError(name, status, lib().dab_strerror(status).decode())


def _ptr(t, dtype, name):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name}: expected a tensor on the GPU")
    if t.dtype != dtype:
        raise TypeError(f"{name}: expected {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name}: tensor must be contiguous")
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def words_per_pixel(C):
    return (C + 31) // 32


def padded_filters(F):
    return 64 * ((F + 63) // 64)


def _workspace(nbytes, dev, ws):
    """A caller-supplied workspace tensor if it is large enough, else a fresh one (None when none is needed)."""
    if nbytes == 0:
        return None
    if ws is not None and ws.numel() * ws.element_size() >= nbytes:
        return ws
    return torch.empty(nbytes, dtype=torch.uint8, device=dev)


def estimate_outputs(F, dev):
    """Empty output tensors of dab_estimate_alpha_beta for F filters."""
    return dict(
        alpha=torch.empty(F, dtype=torch.float32, device=dev), beta=torch.empty(F, dtype=torch.float32, device=dev),
        K=torch.empty(F, dtype=torch.int32, device=dev), thr_val=torch.empty(F, dtype=torch.float32, device=dev),
        thr_idx=torch.empty(F, dtype=torch.int32, device=dev),
        alpha_is_upper=torch.empty(F, dtype=torch.uint8, device=dev))


def dab_estimate_alpha_beta(W, out=None, ws=None):
    """W [F, n] fp32 -> dict(alpha, beta, K, thr_val, thr_idx, alpha_is_upper), each [F].

    out: a dict from estimate_outputs() to write into instead of fresh tensors."""
    F, n = W.shape
    dev = W.device
    if out is None:
        out = estimate_outputs(F, dev)
    nbytes = lib().dab_estimate_workspace_bytes(F, n)
    ws = _workspace(nbytes, dev, ws)
    _check("dab_estimate_alpha_beta", lib().dab_estimate_alpha_beta(
        _ptr(W, torch.float32, "W"), F, n, out["alpha"].data_ptr(), out["beta"].data_ptr(), out["K"].data_ptr(),
        out["thr_val"].data_ptr(), out["thr_idx"].data_ptr(), out["alpha_is_upper"].data_ptr(),
        ws.data_ptr() if ws is not None else None, nbytes, _stream()))
    return out


def dab_estimate_alpha_beta_noalloc(W, out):
    """dab_estimate_alpha_beta into the tensors of `out` (from estimate_outputs()), with the hand-over flags in
    the library's own device array: the call allocates nothing."""
    F, n = W.shape
    _check("dab_estimate_alpha_beta_noalloc", lib().dab_estimate_alpha_beta_noalloc(
        _ptr(W, torch.float32, "W"), F, n, out["alpha"].data_ptr(), out["beta"].data_ptr(), out["K"].data_ptr(),
        out["thr_val"].data_ptr(), out["thr_idx"].data_ptr(), out["alpha_is_upper"].data_ptr(), _stream()))
    return out


def dab_estimate_sign_split(W, out=None):
    """W [F, n] fp32 -> the same dict as dab_estimate_alpha_beta for e = [w >= 0], alpha = mean|w|, beta = -alpha."""
    F, n = W.shape
    if out is None:
        out = estimate_outputs(F, W.device)
    _check("dab_estimate_sign_split", lib().dab_estimate_sign_split(
        _ptr(W, torch.float32, "W"), F, n, out["alpha"].data_ptr(), out["beta"].data_ptr(), out["K"].data_ptr(),
        out["thr_val"].data_ptr(), out["thr_idx"].data_ptr(), out["alpha_is_upper"].data_ptr(), _stream()))
    return out


def pack_weights_outputs(F, C, kh, kw, dev):
    """Empty (E_packed, ecnt) of dab_pack_weights."""
    R, Fp = kh * kw * words_per_pixel(C), padded_filters(F)
    return (torch.empty((R, Fp), dtype=torch.int32, device=dev),
            torch.empty((F, kh * kw), dtype=torch.int32, device=dev))


def dab_pack_weights(W, thr_val, thr_idx, alpha_is_upper, out=None):
    """W [F, C, kh, kw] fp32 + split descriptor -> (E_packed uint32-as-int32 [R, Fp], ecnt int32 [F, kh*kw]).

    out: an (E_packed, ecnt) pair from pack_weights_outputs() to write into."""
    F, C, kh, kw = W.shape
    E, ecnt = out if out is not None else pack_weights_outputs(F, C, kh, kw, W.device)
    _check("dab_pack_weights", lib().dab_pack_weights(
        _ptr(W, torch.float32, "W"), F, C, kh, kw, _ptr(thr_val, torch.float32, "thr_val"),
        _ptr(thr_idx, torch.int32, "thr_idx"), _ptr(alpha_is_upper, torch.uint8, "alpha_is_upper"),
        _ptr(E, torch.int32, "E_packed"), _ptr(ecnt, torch.int32, "ecnt"), _stream()))
    return E, ecnt


def dab_pack_activations(X, layout=DAB_LAYOUT_NHWC, tau=None, out=None):
    """X fp32 NHWC [B,H,W,C] (or NCHW [B,C,H,W]; a 2-D [B,C] is H=W=1) -> int32 [B,H,W,Cw]."""
    if X.dim() == 2:
        B, C = X.shape
        H = W = 1
    elif layout == DAB_LAYOUT_NHWC:
        B, H, W, C = X.shape
    else:
        B, C, H, W = X.shape
    A = out if out is not None else torch.empty((B, H, W, words_per_pixel(C)), dtype=torch.int32, device=X.device)
    _check("dab_pack_activations", lib().dab_pack_activations(
        _ptr(X, torch.float32, "X"), layout, B, C, H, W, _ptr(tau, torch.float32, "tau"),
        _ptr(A, torch.int32, "A_packed"), _stream()))
    return A


def dab_init():
    """One-time set-up of the current device (every entry point does it on first use as well)."""
    _check("dab_init", lib().dab_init())


def dab_probe_popcount(pair, iters, grid, out, clocks):
    """One launch of the popcount-rate probe; returns (lane-popcounts issued, constant-rate clock in kHz)."""
    ops, khz = ctypes.c_int64(0), c_int32(0)
    _check("dab_probe_popcount", lib().dab_probe_popcount(
        int(bool(pair)), iters, grid, _ptr(out, torch.int32, "out"), _ptr(clocks, torch.int64, "clocks"),
        ctypes.byref(ops), ctypes.byref(khz), _stream()))
    return ops.value, khz.value


class dab_weight_job(ctypes.Structure):
    _fields_ = [("W", c_void_p), ("F", c_int32), ("C", c_int32), ("kh", c_int32), ("kw", c_int32),
                ("alpha", c_void_p), ("beta", c_void_p), ("K", c_void_p), ("thr_val", c_void_p), ("thr_idx", c_void_p),
                ("alpha_is_upper", c_void_p), ("E_packed", c_void_p), ("ecnt", c_void_p),
                ("K_prev", c_void_p), ("alpha_is_upper_prev", c_void_p), ("max_change", c_int32)]


def weight_jobs(items):
    """A host array of dab_weight_job from dicts(W=[F,C,kh,kw], est=estimate_outputs(), packed=(E, ecnt) or None,
    prev=(K_prev, alpha_is_upper_prev, max_change) or None); built once, reused per call."""
    arr = (dab_weight_job * len(items))()
    for k, it in enumerate(items):
        W, est = it["W"], it["est"]
        F, C, kh, kw = W.shape
        E, ecnt = it.get("packed") or (None, None)
        Kp, up, mc = it.get("prev") or (None, None, 0)
        arr[k] = dab_weight_job(
            _ptr(W, torch.float32, "W"), F, C, kh, kw, _ptr(est["alpha"], torch.float32, "alpha"),
            _ptr(est["beta"], torch.float32, "beta"), _ptr(est["K"], torch.int32, "K"),
            _ptr(est["thr_val"], torch.float32, "thr_val"), _ptr(est["thr_idx"], torch.int32, "thr_idx"),
            _ptr(est["alpha_is_upper"], torch.uint8, "alpha_is_upper"), _ptr(E, torch.int32, "E_packed"),
            _ptr(ecnt, torch.int32, "ecnt"), _ptr(Kp, torch.int32, "K_prev"), _ptr(up, torch.uint8, "alpha_is_upper_prev"), mc)
    return arr


def dab_binarize_weights_multi(jobs, ws=None):
    """Estimation and weight packing of every job of weight_jobs() in two or three launches."""
    nbytes = lib().dab_binarize_weights_multi_workspace_bytes(jobs, len(jobs))
    if nbytes and (ws is None or ws.numel() * ws.element_size() < nbytes):
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    _check("dab_binarize_weights_multi", lib().dab_binarize_weights_multi(
        jobs, len(jobs), ws.data_ptr() if nbytes else None, nbytes, _stream()))


class dab_pack_job(ctypes.Structure):
    _fields_ = [("X", c_void_p), ("tau", c_void_p), ("A_packed", c_void_p),
                ("B", c_int32), ("C", c_int32), ("H", c_int32), ("W", c_int32)]


def pack_jobs(items):
    """A host array of dab_pack_job from (X NHWC or [B,C], tau or None, A_packed) triples (built once, reused per call)."""
    arr = (dab_pack_job * len(items))()
    for k, (X, tau, A) in enumerate(items):
        if X.dim() == 2:
            B, C = X.shape
            H = W = 1
        else:
            B, H, W, C = X.shape
        arr[k] = dab_pack_job(_ptr(X, torch.float32, "X"), _ptr(tau, torch.float32, "tau"), _ptr(A, torch.int32, "A_packed"),
                              B, C, H, W)
    return arr


def dab_pack_activations_multi(jobs):
    """dab_pack_activations for every job of pack_jobs() in one launch."""
    _check("dab_pack_activations_multi", lib().dab_pack_activations_multi(jobs, len(jobs), _stream()))


def dab_prepare_layers(wjobs, pjobs, ws=None):
    """dab_binarize_weights_multi(wjobs) and dab_pack_activations_multi(pjobs) in the same launches."""
    nbytes = lib().dab_binarize_weights_multi_workspace_bytes(wjobs, len(wjobs))
    if nbytes and (ws is None or ws.numel() * ws.element_size() < nbytes):
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    _check("dab_prepare_layers", lib().dab_prepare_layers(
        wjobs, len(wjobs), pjobs, len(pjobs), ws.data_ptr() if nbytes else None, nbytes, _stream()))


def dab_binconv2d(desc, A_packed, E_packed, alpha, beta, want_s1=False, out=None, ws=None):
    """Binarized convolution; returns Y fp32 [B,Ho,Wo,F] (and int32 s1 of the same shape if asked)."""
    dev = A_packed.device
    shape = (desc.B, desc.Ho, desc.Wo, desc.F)
    Y = out if out is not None else torch.empty(shape, dtype=torch.float32, device=dev)
    s1 = torch.empty(shape, dtype=torch.int32, device=dev) if want_s1 else None
    nbytes = lib().dab_binconv2d_workspace_bytes(ctypes.byref(desc))
    ws = _workspace(nbytes, dev, ws)
    _check("dab_binconv2d", lib().dab_binconv2d(
        ctypes.byref(desc), _ptr(A_packed, torch.int32, "A_packed"), _ptr(E_packed, torch.int32, "E_packed"),
        _ptr(alpha, torch.float32, "alpha"), _ptr(beta, torch.float32, "beta"),
        _ptr(Y, torch.float32, "Y"), s1.data_ptr() if want_s1 else None,
        ws.data_ptr() if ws is not None else None, nbytes, _stream()))
    return (Y, s1) if want_s1 else Y


def dab_binfc(A_packed, E_packed, alpha, beta, Kin, want_s1=False, out=None, ws=None):
    """Binarized fully-connected layer; A_packed [B, Kw], returns Y fp32 [B, F]."""
    dev = A_packed.device
    B = A_packed.shape[0]
    F = alpha.shape[0]
    Y = out if out is not None else torch.empty((B, F), dtype=torch.float32, device=dev)
    s1 = torch.empty((B, F), dtype=torch.int32, device=dev) if want_s1 else None
    nbytes = lib().dab_binfc_workspace_bytes(B, Kin, F)
    ws = _workspace(nbytes, dev, ws)
    _check("dab_binfc", lib().dab_binfc(
        B, Kin, F, _ptr(A_packed, torch.int32, "A_packed"), _ptr(E_packed, torch.int32, "E_packed"),
        _ptr(alpha, torch.float32, "alpha"), _ptr(beta, torch.float32, "beta"),
        _ptr(Y, torch.float32, "Y"), s1.data_ptr() if want_s1 else None,
        ws.data_ptr() if ws is not None else None, nbytes, _stream()))
    return (Y, s1) if want_s1 else Y


def dab_binconv2d_bits(desc, A_packed, E_packed, alpha, beta, tau_out=None, out=None, ws=None):
    """Binarized convolution with the re-binarizing epilogue; returns int32 [B,Ho,Wo,ceil(F/32)]."""
    dev = A_packed.device
    shape = (desc.B, desc.Ho, desc.Wo, words_per_pixel(desc.F))
    A_next = out if out is not None else torch.empty(shape, dtype=torch.int32, device=dev)
    nbytes = lib().dab_binconv2d_workspace_bytes(ctypes.byref(desc))
    ws = _workspace(nbytes, dev, ws)
    _check("dab_binconv2d_bits", lib().dab_binconv2d_bits(
        ctypes.byref(desc), _ptr(A_packed, torch.int32, "A_packed"), _ptr(E_packed, torch.int32, "E_packed"),
        _ptr(alpha, torch.float32, "alpha"), _ptr(beta, torch.float32, "beta"), _ptr(tau_out, torch.float32, "tau_out"),
        _ptr(A_next, torch.int32, "A_next"), ws.data_ptr() if ws is not None else None, nbytes, _stream()))
    return A_next


def dab_binfc_bits(A_packed, E_packed, alpha, beta, Kin, tau_out=None, out=None, ws=None):
    """Binarized fully-connected layer with the re-binarizing epilogue; returns int32 [B, ceil(F/32)]."""
    dev = A_packed.device
    B, F = A_packed.shape[0], alpha.shape[0]
    A_next = out if out is not None else torch.empty((B, words_per_pixel(F)), dtype=torch.int32, device=dev)
    nbytes = lib().dab_binfc_workspace_bytes(B, Kin, F)
    ws = _workspace(nbytes, dev, ws)
    _check("dab_binfc_bits", lib().dab_binfc_bits(
        B, Kin, F, _ptr(A_packed, torch.int32, "A_packed"), _ptr(E_packed, torch.int32, "E_packed"),
        _ptr(alpha, torch.float32, "alpha"), _ptr(beta, torch.float32, "beta"), _ptr(tau_out, torch.float32, "tau_out"),
        _ptr(A_next, torch.int32, "A_next"), ws.data_ptr() if ws is not None else None, nbytes, _stream()))
    return A_next


def dab_pool_bits(A_packed, C, kh, kw, stride_h, stride_w, out=None):
    """OR-pooling of packed signs: int32 [B,H,W,Cw] -> [B,Ho,Wo,Cw] (windows inside the image)."""
    B, H, W, Cw = A_packed.shape
    Ho, Wo = (H - kh) // stride_h + 1, (W - kw) // stride_w + 1
    A_pooled = out if out is not None else torch.empty((B, max(Ho, 0), max(Wo, 0), Cw), dtype=torch.int32,
                                                        device=A_packed.device)
    _check("dab_pool_bits", lib().dab_pool_bits(
        _ptr(A_packed, torch.int32, "A_packed"), B, C, H, W, kh, kw, stride_h, stride_w,
        _ptr(A_pooled, torch.int32, "A_pooled"), _stream()))
    return A_pooled


DAB_CENTER_FILTER, DAB_CENTER_CHANNEL = 0, 1


def dab_mean_center_clamp(W, axis=DAB_CENTER_FILTER, lo=-1.0, hi=1.0, out=None):
    """MeanCenter + Clamp of W[F,C,kh,kw] (fp32); out may be W itself."""
    F, C = W.shape[0], W.shape[1]
    T = W.shape[2] * W.shape[3]
    W_out = out if out is not None else torch.empty_like(W)
    _check("dab_mean_center_clamp", lib().dab_mean_center_clamp(
        _ptr(W, torch.float32, "W"), F, C, T, axis, lo, hi, _ptr(W_out, torch.float32, "W_out"), _stream()))
    return W_out


def dab_binarized_weights(W, alpha, beta, thr_val, thr_idx, alpha_is_upper, out=None):
    """W~ = alpha e + beta (1 - e) as fp32 [F,n] from W[F,n] and the estimator's outputs."""
    F, n = W.shape
    Wt = out if out is not None else torch.empty_like(W)
    _check("dab_binarized_weights", lib().dab_binarized_weights(
        _ptr(W, torch.float32, "W"), F, n, _ptr(alpha, torch.float32, "alpha"), _ptr(beta, torch.float32, "beta"),
        _ptr(thr_val, torch.float32, "thr_val"), _ptr(thr_idx, torch.int32, "thr_idx"),
        _ptr(alpha_is_upper, torch.uint8, "alpha_is_upper"), _ptr(Wt, torch.float32, "W_tilde"), _stream()))
    return Wt


def dab_weight_gradient(W, thr_val, thr_idx, alpha_is_upper, upstream=None, out=None):
    """Theorem 4's element-wise factor G~ for W[F,n] (times `upstream` when given)."""
    F, n = W.shape
    G = out if out is not None else torch.empty_like(W)
    up = None if upstream is None else _ptr(upstream, torch.float32, "upstream")
    _check("dab_weight_gradient", lib().dab_weight_gradient(
        _ptr(W, torch.float32, "W"), F, n, _ptr(thr_val, torch.float32, "thr_val"),
        _ptr(thr_idx, torch.int32, "thr_idx"), _ptr(alpha_is_upper, torch.uint8, "alpha_is_upper"), up,
        _ptr(G, torch.float32, "G_out"), _stream()))
    return G


def dab_estimate_alpha_beta_bounded(W, K_prev, alpha_is_upper_prev, max_change, out=None, ws=None):
    """dab_estimate_alpha_beta with the split at most `max_change` elements from the previous one
    (K_prev int32 [F], alpha_is_upper_prev uint8 [F]: the previous call's outputs; `out` may hold them)."""
    F, n = W.shape
    o = out if out is not None else estimate_outputs(F, W.device)
    nbytes = lib().dab_estimate_workspace_bytes(F, n)
    ws = _workspace(nbytes, W.device, ws)
    _check("dab_estimate_alpha_beta_bounded", lib().dab_estimate_alpha_beta_bounded(
        _ptr(W, torch.float32, "W"), F, n, _ptr(K_prev, torch.int32, "K_prev"),
        _ptr(alpha_is_upper_prev, torch.uint8, "alpha_is_upper_prev"), max_change,
        _ptr(o["alpha"], torch.float32, "alpha"), _ptr(o["beta"], torch.float32, "beta"), _ptr(o["K"], torch.int32, "K"),
        _ptr(o["thr_val"], torch.float32, "thr_val"), _ptr(o["thr_idx"], torch.int32, "thr_idx"),
        _ptr(o["alpha_is_upper"], torch.uint8, "alpha_is_upper"), ws.data_ptr() if ws is not None else None, nbytes,
        _stream()))
    return o


def dab_wbin_conv2d(desc, X, E_packed, alpha, beta, out=None, ws=None):
    """Weights-only binarized convolution: X fp32 NHWC [B,H,W,C] -> Y fp32 [B,Ho,Wo,F]."""
    dev = X.device
    Y = out if out is not None else torch.empty((desc.B, desc.Ho, desc.Wo, desc.F), dtype=torch.float32, device=dev)
    nbytes = lib().dab_wbin_conv2d_workspace_bytes(ctypes.byref(desc))
    ws = _workspace(nbytes, dev, ws)
    _check("dab_wbin_conv2d", lib().dab_wbin_conv2d(
        ctypes.byref(desc), _ptr(X, torch.float32, "X"), _ptr(E_packed, torch.int32, "E_packed"),
        _ptr(alpha, torch.float32, "alpha"), _ptr(beta, torch.float32, "beta"), _ptr(Y, torch.float32, "Y"),
        ws.data_ptr() if ws is not None else None, nbytes, _stream()))
    return Y


def dab_wbin_fc(X, E_packed, alpha, beta, out=None, ws=None):
    """Weights-only binarized fully-connected layer: X fp32 [B,Kin] -> Y fp32 [B,F]."""
    dev = X.device
    B, Kin = X.shape
    F = alpha.shape[0]
    Y = out if out is not None else torch.empty((B, F), dtype=torch.float32, device=dev)
    nbytes = lib().dab_wbin_fc_workspace_bytes(B, Kin, F)
    ws = _workspace(nbytes, dev, ws)
    _check("dab_wbin_fc", lib().dab_wbin_fc(
        B, Kin, F, _ptr(X, torch.float32, "X"), _ptr(E_packed, torch.int32, "E_packed"),
        _ptr(alpha, torch.float32, "alpha"), _ptr(beta, torch.float32, "beta"), _ptr(Y, torch.float32, "Y"),
        ws.data_ptr() if ws is not None else None, nbytes, _stream()))
    return Y
