"""Static checks over the gfx950 ISA of the kernels that use inline assembly (no GPU needed).

    python -m paper_1804_02941_amd.isa_checks            # compiles csrc/direct.hip and csrc/binconv.hip with -S and checks them

Two things the compiler does for its own instructions but not for inline assembly:

1. loads_in_flight: the activation loads of the persistent product kernel are inline-assembly buffer loads
   with hand-placed `s_waitcnt vmcnt(N)`.  No instruction may read or write the destination registers of
   such a load while it can still be pending on some path.  Loads complete in order, so after vmcnt(N) at
   most the N youngest memory operations are pending; the check is a dataflow analysis over the kernel's
   control-flow graph with the queue of pending loads as the state.
2. scalar_read_hazards: on this ISA a vector instruction needs two wait states (a vector-memory instruction
   five) before it reads a scalar register that a vector instruction (compare, readlane, readfirstlane) has
   written.  The packed-sign epilogue's `v_writelane_b32` in inline assembly once read a ballot register one
   instruction behind the compare that wrote it and took its previous content.
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
import tempfile

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")


def compile_to_isa(source: str, out: str, extra=()) -> None:
    """hipcc -S of one translation unit of csrc/ for gfx950 (the flags of build.py that shape the code)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fno-gpu-rdc", "-ffp-contract=off",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           *extra, "-S", "--cuda-device-only", os.path.join(CSRC, source), "-o", out]
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc -S failed:\n" + proc.stdout)


def kernels(text: str):
    """[(mangled name, lines of the kernel)] of an ISA listing."""
    lines = text.split("\n")
    out = []
    for s, l in enumerate(lines):
        if re.match(r"^_ZN3dab\w+:", l):
            e = next((i for i in range(s, len(lines)) if lines[i].strip().startswith(".Lfunc_end")), len(lines) - 1)
            out.append((l.split(":")[0], lines[s:e]))
    return out


def _instructions(lines):
    """[(line index, text, inside inline assembly)], {label: instruction index}"""
    insns, labels, in_asm = [], {}, False
    for i, l in enumerate(lines):
        t = l.strip()
        if "ASMSTART" in t:
            in_asm = True
        if "ASMEND" in t:
            in_asm = False
        m = re.match(r"^(\.LBB\d+_\d+):", l)
        if m:
            labels[m.group(1)] = len(insns)
        if not t or t.startswith(";") or t.startswith(".") or t.endswith(":"):
            continue
        insns.append((i, t.split(";")[0].strip(), in_asm))
    return insns, labels


def _vregs(text):
    out = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b", text):
        if m.group(1) is not None:
            out.update(range(int(m.group(1)), int(m.group(2)) + 1))
        else:
            out.add(int(m.group(3)))
    return frozenset(out)


def _sregs(text):
    out = set()
    for m in re.finditer(r"\bs\[(\d+):(\d+)\]|\bs(\d+)\b|\bvcc\b", text):
        if m.group(1) is not None:
            out.update(range(int(m.group(1)), int(m.group(2)) + 1))
        elif m.group(3) is not None:
            out.add(int(m.group(3)))
        else:
            out.add("vcc")
    return out


def loads_in_flight(lines, max_states=2_000_000):
    """Violations [(line, text, line of the load)] of one kernel: an instruction that touches the destination of an
    inline-assembly load that may still be pending.  Memory operations the compiler generated are not tracked
    (they can only make a wait longer than assumed here)."""
    insns, labels = _instructions(lines)
    n = len(insns)
    succ = [[] for _ in range(n)]
    for k, (_, t, _) in enumerate(insns):
        op = t.split()[0]
        if op == "s_endpgm":
            continue
        if op == "s_branch":
            succ[k].append(labels[t.split()[1]])
            continue
        m = re.match(r"s_cbranch_\w+\s+(\.LBB\d+_\d+)", t)
        if m:
            succ[k].append(labels[m.group(1)])
        if k + 1 < n:
            succ[k].append(k + 1)
    seen = [set() for _ in range(n)]
    work, bad, steps = [(0, ())], {}, 0
    while work:
        k, st = work.pop()
        if st in seen[k]:
            continue
        seen[k].add(st)
        steps += 1
        if steps > max_states:
            raise RuntimeError("too many states")
        i, t, in_asm = insns[k]
        op = t.split()[0]
        m = re.match(r"s_waitcnt.*vmcnt\((\d+)\)", t)
        new = st
        if m:
            c = int(m.group(1))
            new = () if c == 0 else (st[len(st) - c:] if c < len(st) else st)
        else:
            r = _vregs(t)
            for (li, pr) in st:
                if (r & pr) and li != i:
                    bad[(i, li)] = t
            if in_asm and (op.startswith("buffer_load") or op.startswith("global_load")):
                dst = _vregs(t.split(",")[0])
                for (li, pr) in st:
                    if li == i and dst & pr:
                        bad[(i, li)] = t + "   [issued again while pending]"
                new = (st + ((i, dst),))[-64:]
        for s2 in succ[k]:
            if new not in seen[s2]:
                work.append((s2, new))
    return [(i, t, li) for (i, li), t in sorted(bad.items())]


def scalar_read_hazards(lines):
    """Violations [(line, text, writer text)] of one kernel: an inline-assembly instruction that reads a scalar
    register fewer than two (vector instruction) or five (vector-memory instruction) wait states behind the
    vector instruction that wrote it.  Straight-line distance; s_nop N counts as N + 1."""
    insns, _ = _instructions(lines)
    hist, bad = [], []                                      # (text, scalar registers written by a vector instruction)
    for (i, t, in_asm) in insns:
        op = t.split()[0]
        parts = [p.strip() for p in t[len(op):].split(",")]
        if op == "s_nop":
            hist += [("s_nop", set())] * (int(parts[0], 0) + 1)
            continue
        # (the asm strings of this library hold "s_nop N" and the instruction on separate lines, so both are seen)
        written = set()
        if op.startswith("v_readfirstlane") or op.startswith("v_readlane") or (op.startswith("v_cmp") and "_e64" in op):
            written = _sregs(parts[0])
        elif op.startswith("v_cmp"):
            written = {"vcc"}
        if in_asm and not op.startswith("s_"):
            is_mem = op.startswith("buffer_") or op.startswith("global_") or op.startswith("flat_")
            reads = set()
            for p in (parts if (is_mem and "store" in op) else parts[1:]):
                reads |= _sregs(p)
            need = 5 if is_mem else 2
            for (wt, w) in hist[-need:]:
                if w & reads:
                    bad.append((i, t, wt))
        hist.append((t, written))
    return bad


def reads_before_any_write(lines):
    """Violations [(instruction index, text, registers)] of one kernel: a vector register read that is not written
    on every path from the kernel's entry (v0, the work-item id, is set at entry).  A partial write (under any EXEC
    or DPP mask) counts as a write, so only registers wholly unwritten on some path are reported; a DPP
    instruction whose row or bank mask is not all ones or that has no bound_ctrl, v_writelane and the
    multiply-accumulate forms read their destination's old value."""
    insns, labels = _instructions(lines)
    n = len(insns)
    succ = [[] for _ in range(n)]
    for k, (_, t, _) in enumerate(insns):
        op = t.split()[0]
        if op == "s_endpgm":
            continue
        if op == "s_branch":
            succ[k].append(labels[t.split()[1]])
            continue
        m = re.match(r"s_cbranch_\w+\s+(\.LBB\d+_\d+)", t)
        if m:
            succ[k].append(labels[m.group(1)])
        if k + 1 < n:
            succ[k].append(k + 1)

    def reads_writes(t):
        op = t.split()[0]
        parts = [p.strip() for p in t[len(op):].split(",")]
        reads, writes = set(), set()
        memory = op.startswith(("ds_", "buffer_", "global_", "flat_", "scratch_"))
        if not (op.startswith("v_") or memory):
            return reads, writes
        no_result = ("store" in op or op.startswith("ds_write") or
                     (op.startswith("ds_") and not op.startswith("ds_read") and "rtn" not in op and "permute" not in op))
        if op.startswith(("v_cmp", "v_readfirstlane", "v_readlane")):
            for q in parts[1:]:
                reads |= _vregs(q)
        elif no_result:
            for q in parts:
                reads |= _vregs(q)
        else:
            writes |= _vregs(parts[0])
            for q in parts[1:]:
                reads |= _vregs(q)
            dpp = "_dpp" in op or "row_" in t or "quad_perm" in t
            keeps_old = dpp and (("row_mask" in t and "row_mask:0xf" not in t) or ("bank_mask" in t and "bank_mask:0xf" not in t)
                                 or "bound_ctrl" not in t)
            if keeps_old or op.startswith(("v_writelane", "v_mac", "v_fmac")):
                reads |= _vregs(parts[0])
        return reads, writes

    defined = [None] * n
    defined[0] = frozenset({0})
    work, seen_bad = [0], {}
    while work:
        k = work.pop()
        r, w = reads_writes(insns[k][1])
        if r - defined[k]:
            seen_bad[k] = r
        out = defined[k] | frozenset(w)
        for s2 in succ[k]:
            new = out if defined[s2] is None else defined[s2] & out
            if new != defined[s2]:
                defined[s2] = new
                work.append(s2)
    return [(k, insns[k][1], sorted(r - defined[k])) for k, r in sorted(seen_bad.items()) if r - defined[k]]


def check_estimators_without_the_reserved_register(verbose=True):
    """The sort kernels as they are allocated without DAB_RESERVE_VGPRS (57-64 registers: the allocation whose
    results were wrong on the GPU): no register read before any write; returns the number of violations."""
    total = 0
    with tempfile.TemporaryDirectory() as tmp:
        isa = os.path.join(tmp, "estimate.s")
        compile_to_isa("estimate.hip", isa, ["-DDAB_NO_RESERVE_VGPRS"])
        for name, lines in kernels(open(isa).read()):
            if "estimate_kernel" not in name:
                continue
            v = reads_before_any_write(lines)
            total += len(v)
            if verbose and v:
                print(name)
                for item in v[:8]:
                    print("   ", item)
    if verbose:
        print("reads before any write:", total)
    return total


def check_sources(verbose=True):
    """Compiles the two translation units with inline assembly and runs both checks; returns the number of violations."""
    total = 0
    with tempfile.TemporaryDirectory() as tmp:
        for src in ("direct.hip", "binconv.hip"):
            isa = os.path.join(tmp, src + ".s")
            compile_to_isa(src, isa)
            for name, lines in kernels(open(isa).read()):
                v = scalar_read_hazards(lines)
                if "binconv_direct_kernel" in name:
                    v += loads_in_flight(lines)
                total += len(v)
                if verbose and v:
                    print(name)
                    for item in v[:8]:
                        print("   line", item[0], ":", item[1], "|", item[2])
    if verbose:
        print("violations:", total)
    return total


if __name__ == "__main__":
    sys.exit(1 if check_sources() + check_estimators_without_the_reserved_register() else 0)
