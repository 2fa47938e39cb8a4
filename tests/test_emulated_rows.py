"""The estimator's per-row device functions on the CPU under sanitizers.

tests/emu/ compiles paper_1804_02941_amd/csrc/estimate_rows.h for the host, one OS thread per GPU
thread, workgroup barriers as pthread barriers and wavefront operations as exchanges between
barriers of the wavefront's 64 threads.  ThreadSanitizer then reports any LDS word that two threads
touch (one of them writing) without a barrier between them, AddressSanitizer / UBSan any LDS index
out of bounds, MemorySanitizer (LDS marked uninitialised before every workgroup) any read of an LDS
word or register that nothing wrote.  Every case also checks the results against a plain sort.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EMU = os.path.join(ROOT, "tests", "emu")
CSRC = os.path.join(ROOT, "paper_1804_02941_amd", "csrc")
CLANG = "/opt/rocm/llvm/bin/clang++"
CASES = ["sort64x3", "sort256x7", "sort512x7", "sort1024x7", "sort1024x13", "bucket256x9", "bucket512x9", "bucket512x26"]


def build(tmp, name, compiler, flags):
    exe = os.path.join(tmp, name)
    cmd = [compiler, "-std=c++17", "-O1", "-g", "-pthread", *flags, "-I", EMU, "-I", CSRC,
           os.path.join(EMU, "emulate_rows.cpp"), "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    return exe


@pytest.fixture(scope="module")
def builds(tmp_path_factory):
    tmp = str(tmp_path_factory.mktemp("emu"))
    out = {"tsan": build(tmp, "emu_tsan", "g++", ["-fsanitize=thread"]),
           "asan": build(tmp, "emu_asan", "g++", ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"])}
    if os.path.exists(CLANG):
        out["msan"] = build(tmp, "emu_msan", CLANG, ["-fsanitize=memory", "-DEMU_POISON_LDS"])
    return out


def run(exe, case, seed=1, env=None):
    e = dict(os.environ, TSAN_OPTIONS="halt_on_error=0 exitcode=66")
    e.update(env or {})
    return subprocess.run([exe, case, str(seed)], capture_output=True, text=True, env=e, timeout=900)


@pytest.mark.parametrize("case", CASES)
def test_no_data_race_between_barriers(builds, case):
    for seed in (1, 2):
        p = run(builds["tsan"], case, seed)
        assert "ThreadSanitizer" not in p.stderr, p.stderr[-3000:]
        assert p.returncode == 0, p.stdout[-2000:] + p.stderr[-2000:]
        assert "WRONG" not in p.stdout


@pytest.mark.parametrize("case", CASES)
def test_no_access_out_of_bounds(builds, case):
    p = run(builds["asan"], case)
    assert p.returncode == 0, p.stdout[-2000:] + p.stderr[-3000:]


@pytest.mark.parametrize("case", CASES)
def test_no_read_of_unwritten_memory(builds, case):
    if "msan" not in builds:
        pytest.skip("no clang with MemorySanitizer here")
    p = run(builds["msan"], case)
    assert "MemorySanitizer" not in p.stderr and p.returncode == 0, p.stdout[-2000:] + p.stderr[-3000:]
    assert "LDS section marked uninitialised" in p.stdout


def test_the_checker_sees_a_missing_barrier(builds):
    """With one workgroup barrier skipped by every thread the race report must appear."""
    p = run(builds["tsan"], "sort64x3", env={"EMU_SKIP_BARRIER": "3"})
    assert "ThreadSanitizer: data race" in p.stderr and p.returncode != 0
