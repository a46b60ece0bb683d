"""The nontemporal hint has to reach the machine code.

Written as `if (nt) nontemporal store else plain store`, the compiler merges the two stores (they differ in
nothing but the hint) and drops it, silently: every result stays the same, only the cache behaviour changes.
These tests compile two translation units to gfx950 assembly (no GPU needed) and look at the store
instructions of the kernels that are meant to carry the hint.
"""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_1810_08297_amd", "csrc")

pytestmark = pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not found")


def _assembly(source, tmp_path):
    out = os.path.join(tmp_path, os.path.splitext(source)[0] + ".s")
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-S", "--cuda-device-only",
           "-o", out, os.path.join(CSRC, source)]
    subprocess.run(cmd, check=True, capture_output=True)
    with open(out) as f:
        return f.read()


def _kernel_body(asm, symbol):
    start = asm.index("\n" + symbol + ":")
    end = asm.index(".Lfunc_end", start)
    return asm[start:end]


def _vector_stores(body):
    stores = re.findall(r"^\s*global_store_dwordx4 .*$", body, flags=re.M)
    hinted = [s for s in stores if re.search(r"\bnt\b", s)]
    return len(stores) - len(hinted), len(hinted)


def test_forward_kernel_holds_both_store_forms(tmp_path):
    """branchy5's forward kernel writes 1 output + 5 planes per lane: each of the six stores exists plainly and with
    the hint (the block picks one form), both with a scalar base and a 32-bit lane offset."""
    asm = _assembly("ops_misc.hip", str(tmp_path))
    body = _kernel_body(asm, "_ZN2bd16fwd_tiled_kernelINS_10OpBranchy5EfLi4ELb1ELb1ELb0EEEvNS_14FwdTiledParamsE")
    plain, hinted = _vector_stores(body)
    assert plain == 6 and hinted == 6, (plain, hinted)
    assert all(re.search(r"s\[\d+:\d+\]", s) for s in re.findall(r"^\s*global_store_dwordx4 .*$", body, flags=re.M))


def test_backward_kernels_take_the_hint_as_a_template_parameter(tmp_path):
    """The kernel compiled for branchy5's mix of gradients writes its two full-shape gradients per row step (edge and
    interior path): with the hint in the form built for it, plainly in the other."""
    asm = _assembly("bwd_kernels.hip", str(tmp_path))
    base = "_ZN2bd14bwd_sig_kernelIfLi4ELi1ELi2ELi1ELi1ELi1ELm0ELm0ELi1ELb1ELb%dEEEvNS_14BwdTiledParamsE"
    plain, hinted = _vector_stores(_kernel_body(asm, base % 1))
    assert hinted >= 2, (plain, hinted)  # (the blocks at a ragged row end keep plain stores)
    plain, hinted = _vector_stores(_kernel_body(asm, base % 0))
    assert plain >= 2 and hinted == 0, (plain, hinted)
