"""The prefill kernel counts outstanding loads by hand: the wait before a stage barrier, vmcnt(N), leaves the N
youngest loads in flight, which is right only if every X request (a load that writes LDS directly) is older than at
least N ordinary loads.  The compiler is free to order instructions that no scheduling barrier separates, so this
test compiles the kernel to assembly and checks the order that came out, for every tile size and both formats.
It runs on the CPU: hipcc cross-compiles for gfx950 without a GPU."""
import importlib.util
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2604_15272_amd")


def _build_module():
    spec = importlib.util.spec_from_file_location("_prism_build_for_test", os.path.join(PKG, "build.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def hand_written_waits(asm_text):
    """{kernel symbol: [(N of a hand-written 's_waitcnt vmcnt(N) lgkmcnt(0)', ordinary loads since the last
    load-to-LDS request, or None if there was no request yet)]} in program order."""
    out, name, in_asm, since = {}, None, False, None
    for line in asm_text.split("\n"):
        m = re.match(r"^(_ZN5prism14prefill_kernel\S+):", line)
        if m:
            name, in_asm, since = m.group(1), False, None
            out[name] = []
            continue
        if name is None:
            continue
        if "s_endpgm" in line:
            name = None
        elif "#ASMSTART" in line:
            in_asm = True
        elif "#ASMEND" in line:
            in_asm = False
        elif re.search(r"\b(buffer|global)_load", line):
            if re.search(r"\blds\b", line):
                since = 0
            elif since is not None:
                since += 1
        elif in_asm:
            w = re.search(r"s_waitcnt vmcnt\((\d+)\) lgkmcnt\(0\)", line)
            if w:
                out[name].append((int(w.group(1)), since))
    return out


def test_checker_sees_a_request_that_is_too_young():
    asm = "\n".join(["_ZN5prism14prefill_kernelIxEEv:", " buffer_load_dwordx4 v1, s[0:3], 0 offen lds",
                     " buffer_load_dwordx4 v[2:5], v1, s[0:3], 0 offen", " buffer_load_dword v9, s[0:3], 0 offen lds",
                     " buffer_load_dwordx4 v[2:5], v1, s[0:3], 0 offen", ";;#ASMSTART",
                     " s_waitcnt vmcnt(2) lgkmcnt(0)", ";;#ASMEND", " s_waitcnt vmcnt(0) lgkmcnt(0)", " s_endpgm"])
    assert hand_written_waits(asm) == {"_ZN5prism14prefill_kernelIxEEv": [(2, 1)]}


def _check_compiled_kernel(tmp_path):
    b = _build_module()
    # No skip without a compiler: the library cannot be built without it either, and a silently skipped guard is how a
    # toolchain update would bring the race back unnoticed.
    hipcc = b.hipcc_path()
    flags = [f for f in b.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    out = str(tmp_path / "prefill.s")
    cmd = [hipcc] + flags + ["-S", "--cuda-device-only", "-I", os.path.join(ROOT, "include"), "-I",
                             os.path.join(PKG, "csrc"), os.path.join(PKG, "csrc", "prefill_kernel.hip"), "-o", out]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    waits = hand_written_waits(open(out).read())
    assert len(waits) == 16, sorted(waits)  # 8 tiles x 2 storage formats
    for name, seq in waits.items():
        in_loop = [(n, since) for n, since in seq if n > 0]
        assert len(in_loop) >= 2, (name, seq)  # the K loop is unrolled twice, one stage barrier per step
        for n, since in seq:
            assert n == 0 or (since is not None and since >= n), (name, seq)


def test_every_x_request_is_older_than_the_loads_the_barrier_leaves_in_flight(tmp_path):
    _check_compiled_kernel(tmp_path)


@pytest.mark.gpu
def test_wait_counts_hold_for_the_compiler_on_the_gpu_box(tmp_path):
    """The same check in the GPU tier: the compiler that is installed where the kernels run."""
    _check_compiled_kernel(tmp_path)
