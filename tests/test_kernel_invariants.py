"""Properties of the compiled kernels that their speed or correctness counts on (no GPU needed).

1. What the 64-channel fp32 3x3 kernel's waits count on.

Without the add link the kernel issues the next tile's first two slab loads ahead of a tile's output stores and then
waits BY COUNT (vmcnt(45) / vmcnt(44): all but the other slab, the 32 stores and the 12 loads of the next patch).
That is only right if every wavefront really issues 32 stores and 12 patch loads per tile, whatever its lanes'
predicates: fewer operations after the slab than the wait allows to be outstanding and the slab may still be in
flight when it is read.  The compiler is free to branch around a store whose lanes are all off, to merge stores, or
to drop loads; this test fails the build of the library's sources if it ever does.

2. No wait for all vector-memory operations between two stores of an epilogue.  Every store of these epilogues sits
in a branch of its own; with a load still pending when such a branch is entered (a bias or addend value loaded inside
the epilogue) the compiler puts `s_waitcnt vmcnt(0)` in front of every store, and every store then waits for the one
before it to be written.  The kernels load those values ahead and state the wait once; this checks that it stays so.
"""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_1805_00907_amd", "csrc")
HIPCC = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


def _kernel_body(asm, mangled_piece):
    """Instructions and block labels of one kernel, in program text order."""
    m = re.search(r"^_ZN\S*" + mangled_piece + r"\S*:.*?\n(.*?)\.Lfunc_end", asm, re.S | re.M)
    assert m, mangled_piece
    lines = []
    for ln in m.group(1).splitlines():
        ln = ln.split(";")[0].strip()
        if ln and (ln.startswith(".LBB") or not ln.startswith(".")):
            lines.append(ln)
    return lines


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not installed")
def test_k3c64_f32_issues_a_fixed_number_of_memory_operations_per_tile(tmp_path):
    out = tmp_path / "k3c64.s"
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-I", CSRC, "-I", os.path.join(ROOT, "include"), "-S", "--cuda-device-only",
           "-o", str(out), os.path.join(CSRC, "conv_k3c64_f32.hip")]
    subprocess.run(cmd, check=True, capture_output=True)
    body = _kernel_body(out.read_text(), "conv_k3c64_f32_kernelILb0E")       # the kernel without the add link
    stores = [i for i, ln in enumerate(body) if ln.startswith("buffer_store_dword")]
    assert len(stores) == 32, len(stores)                                    # one epilogue, 2 x 16 results per lane
    assert not any(ln.startswith(("global_store", "flat_store", "buffer_store_dwordx")) for ln in body)
    # nothing skips a store: a store under a lane predicate would sit between a branch on the exec mask and that
    # branch's (forward) target
    labels = {ln[:-1]: i for i, ln in enumerate(body) if ln.endswith(":")}
    for i, ln in enumerate(body):
        m = re.match(r"s_cbranch_exec(?:z|nz) (\S+)$", ln)
        if m and labels.get(m.group(1), -1) > i:
            skipped = [j for j in stores if i < j < labels[m.group(1)]]
            assert not skipped, (ln, len(skipped))
    # the patch fetch: twelve 16-byte loads at each of its two call sites (before the tile loop, inside it)
    patch_loads = [ln for ln in body if re.match(r"buffer_load_dwordx4 v\[", ln)]
    assert len(patch_loads) == 24, len(patch_loads)
    # the waits themselves: gfx9 encodes vmcnt in bits 3:0 and 15:14
    waits = set()
    for ln in body:
        m = re.match(r"s_waitcnt vmcnt\((\d+)\)$", ln)
        if m:
            waits.add(int(m.group(1)))
    assert {45, 44, 33, 32, 13, 12, 1, 0} <= waits, sorted(waits)


def _compile(tmp_path, name):
    out = tmp_path / (name + ".s")
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-I", CSRC, "-I", os.path.join(ROOT, "include"), "-S", "--cuda-device-only",
           "-o", str(out), os.path.join(CSRC, name + ".hip")]
    subprocess.run(cmd, check=True, capture_output=True)
    return out.read_text()


def _stores_that_wait(body):
    stores = [i for i, ln in enumerate(body) if re.match(r"(global|buffer|flat)_store", ln)]
    waits = 0
    for a, b in zip(stores, stores[1:]):
        if any(ln.startswith("s_waitcnt") and "vmcnt(0)" in ln for ln in body[a + 1:b]):
            waits += 1
    return len(stores), waits


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not installed")
@pytest.mark.parametrize("source,kernel,n_stores", [
    ("conv_k3v_f32", "conv_k3v_f32_kernelILb0ELi7E", 112),          # 64 (squares) + 48 (strips of three blocks)
    ("conv_k3v_f32", "conv_k3v_f32_kernelILb0ELi8E", 128),
    ("igemm_f32_p3", "igemm_f32_p3_kernelILi2ELb0ELb0ELi3E", 32),
    ("igemm_f32_p3", "igemm_f32_p3_kernelILi2ELb1ELb1ELi3E", 32),
])
def test_no_epilogue_store_waits_for_the_one_before_it(tmp_path, source, kernel, n_stores):
    body = _kernel_body(_compile(tmp_path, source), kernel)
    stores, waiting = _stores_that_wait(body)
    assert stores == n_stores, stores
    assert waiting <= 2, waiting        # (the contraction over planes waits once per 32-channel column, by design)
