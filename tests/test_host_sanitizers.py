"""The library's host code (geometry checks, planners, workspace sizes, argument validation) built with
AddressSanitizer and UBSan (host side of the hipcc compile only) and driven over random layer
geometries by tests/host/fuzz_plans.cpp, which also checks the invariants the kernels rely on.
No GPU is needed: every entry point ends before its first launch here."""
import os
import subprocess

import pytest

from paper_1804_02941_amd import build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def fuzz(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("host") / "fuzz_plans")
    flags = [f for f in build.FLAGS if f not in ("-shared", "-fPIC") and not f.startswith("-Rpass")]
    cmd = [os.environ.get("HIPCC", "/opt/rocm/bin/hipcc"), *flags, "-g",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-I", os.path.join(ROOT, "include"), "-I", build.CSRC,
           *[os.path.join(build.CSRC, s) for s in build.SOURCES],
           os.path.join(ROOT, "tests", "host", "fuzz_plans.cpp"), "-o", exe]
    p = subprocess.run(cmd, capture_output=True, text=True)
    assert p.returncode == 0, p.stdout[-3000:] + p.stderr[-3000:]
    return exe


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_geometries_through_the_host_code(fuzz, seed):
    p = subprocess.run([fuzz, "100000", str(seed)], capture_output=True, text=True, timeout=600)
    assert p.returncode == 0, p.stdout[-2000:] + p.stderr[-4000:]
    assert "geometries checked" in p.stdout
