"""The fp16 softmax kernels take a lane's maximum over its eight values with packed fp16 maxima.  A bit cast written
directly on a vector element once compiled to a maximum over the first dword only (no packed instruction at all,
and results that were right unless exp(x - max) overflowed).  This test compiles the kernels to assembly on the CPU
and checks that the fp16 instantiations contain the packed maxima; the numerical check is the GPU test with
planted maxima."""
import importlib.util
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2604_15272_amd")


def _functions(asm_text, prefix):
    out, name = {}, None
    for line in asm_text.split("\n"):
        m = re.match(r"^(_ZN5prism\S+):", line)
        if m:
            name = m.group(1) if m.group(1).startswith(prefix) else None
            if name:
                out[name] = []
        elif name is not None:
            out[name].append(line)
            if ".amdhsa_kernel" in line:
                name = None
    return out


@pytest.mark.parametrize("source,prefix", [("softmax_kernel.hip", "_ZN5prism19softmax_rows_kernel"),
                                           ("softmax_split_kernel.hip", "_ZN5prism")])
def test_fp16_instantiations_use_packed_maxima_over_all_four_dwords(tmp_path, source, prefix):
    spec = importlib.util.spec_from_file_location("_prism_build_for_test", os.path.join(PKG, "build.py"))
    b = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(b)
    try:
        hipcc = b.hipcc_path()
    except RuntimeError:
        pytest.skip("no hipcc here")
    flags = [f for f in b.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    out = str(tmp_path / "k.s")
    cmd = [hipcc] + flags + ["-S", "--cuda-device-only", "-I", os.path.join(ROOT, "include"), "-I",
                             os.path.join(PKG, "csrc"), os.path.join(PKG, "csrc", source), "-o", out]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    fns = {n: body for n, body in _functions(open(out).read(), prefix).items() if "F16" in n}
    assert fns, "no fp16 instantiation found"
    for name, body in fns.items():
        packed = sum(1 for l in body if "v_pk_max_f16" in l)
        # three packed maxima reduce four dwords to one (the compiler adds more to canonicalise inputs)
        assert packed >= 3, (name, packed)
