"""The C-ABI library: it loads, exports every symbol the header declares, and validates on the host."""
import ctypes
import os
import re

import pytest

from paper_1804_02941_amd import binding, build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    return binding.lib()


def declared_symbols():
    text = "".join(open(os.path.join(ROOT, "include", f)).read()
                   for f in sorted(os.listdir(os.path.join(ROOT, "include"))) if f.endswith(".h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dab_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = declared_symbols()
    assert {"dab_pack_weights", "dab_estimate_alpha_beta", "dab_pack_activations", "dab_binconv2d", "dab_binfc"} <= set(names)
    for name in names:
        assert hasattr(lib, name), f"{name} is declared in include/ but not exported"
    # and the binding covers every one of them
    assert set(names) == set(binding._SIGNATURES)


def test_status_text(lib):
    assert lib.dab_strerror(0) == b"ok"
    for s in range(1, 7):
        assert len(lib.dab_strerror(s)) > 3
    assert lib.dab_strerror(99) == b"unknown status"
    assert lib.dab_last_hip_error() == 0


def test_host_side_validation_needs_no_gpu(lib):
    """NULL / shape errors are reported before any HIP call, so they are testable without a device."""
    assert lib.dab_pack_activations(None, 0, 1, 1, 1, 1, None, None, None) == 1
    assert lib.dab_estimate_alpha_beta(None, 1, 2, None, None, None, None, None, None, None, 0, None) == 1
    assert lib.dab_pack_weights(None, 1, 1, 1, 1, None, None, None, None, None, None) == 1
    assert lib.dab_binconv2d(None, None, None, None, None, None, None, None, 0, None) == 1
    assert lib.dab_binfc(1, 2, 1, None, None, None, None, None, None, None, 0, None) == 1
    fake = ctypes.c_void_p(4096)       # never dereferenced: shape checks come first
    assert lib.dab_estimate_alpha_beta(fake, 1, 1, fake, fake, fake, fake, fake, fake, None, 0, None) == 2
    assert lib.dab_estimate_alpha_beta(fake, 0, 5, fake, fake, fake, fake, fake, fake, None, 0, None) == 2
    assert lib.dab_estimate_alpha_beta(fake, 1, lib.dab_estimate_max_n() + 1, fake, fake, fake, fake, fake, fake, None, 0, None) == 5
    assert lib.dab_pack_weights(fake, 1, 1, 1, 1, fake, fake, fake, fake, fake, None) == 2
    assert lib.dab_binfc(0, 64, 1, fake, fake, fake, fake, fake, None, None, 0, None) == 2
    assert lib.dab_binfc(1, 64, 1, fake, ctypes.c_void_p(4100), fake, fake, fake, None, None, 0, None) == 3
    assert lib.dab_binfc(8192, 9216, 512, fake, fake, fake, fake, fake, None, None, 0, None) == 4   # workspace missing
    d = binding.dab_conv_desc(1, 8, 4, 4, 2, 5, 5, 0, 0, 1, 1)      # window larger than the image
    assert lib.dab_binconv2d(ctypes.byref(d), fake, fake, fake, fake, fake, None, None, 0, None) == 2
    d = binding.dab_conv_desc(1, 8, 4, 4, 2, 3, 3, 0, 0, 0, 1)      # zero stride
    assert lib.dab_binconv2d(ctypes.byref(d), fake, fake, fake, fake, fake, None, None, 0, None) == 2
    assert lib.dab_estimate_workspace_bytes(4, 100) == 0
    assert lib.dab_binfc_workspace_bytes(4, 100, 4) == 0            # small layers run from the bits alone
    assert lib.dab_binfc_workspace_bytes(2048, 64, 512) == 0        # and so do all whose filter bits fit in LDS
    assert lib.dab_binfc_workspace_bytes(8192, 9216, 512) > 0       # a long reduction over many rows expands its operands
    assert lib.dab_binfc_workspace_bytes(0, 100, 4) == 0


def test_bench_refuses_more_than_one_gpu():
    """One GPU only: bench.py --gpus 2 exits with a message and a non-zero status before touching a GPU."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert p.returncode == 2
    assert "one GPU" in p.stderr
