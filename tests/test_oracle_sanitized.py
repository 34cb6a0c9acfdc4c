"""The oracle's C source rebuilt with the host sanitizers and run against every pin (no GPU).

Two builds in a temporary directory: UndefinedBehaviorSanitizer with -fno-sanitize-recover (signed
overflow, shifts out of range, misaligned or out-of-bounds indexing the compiler can see, float-to-int
casts that do not fit) and AddressSanitizer (heap accesses outside the numpy buffers the wrappers
pass).  Each runs in a child process, because a finding aborts the process and ASan's runtime has to
be loaded before the interpreter starts.
"""
import os
import subprocess
import sys
import textwrap

import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(os.path.dirname(oracle.__file__), "glow_oracle.c")

CHILD = textwrap.dedent("""
    import sys
    sys.path.insert(0, {root!r})
    sys.path.insert(0, {tests!r})
    import oracle
    from oracle_pins import ALL_PINS
    with oracle.use_library({so!r}):
        for pin in ALL_PINS:
            pin()
            print("ok", pin.__name__, flush=True)
    print("ALL_PINS_PASSED", len(ALL_PINS))
""")


def _gcc_file(name):
    out = subprocess.run(["gcc", "-print-file-name=" + name], capture_output=True, text=True).stdout.strip()
    return out if os.path.isabs(out) and os.path.exists(out) else None


def _run_pins(so, env_extra):
    env = dict(os.environ)
    env.update(env_extra)
    env["OMP_NUM_THREADS"] = "2"
    code = CHILD.format(root=ROOT, tests=os.path.join(ROOT, "tests"), so=so)
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, env=env, timeout=900)
    assert r.returncode == 0 and "ALL_PINS_PASSED" in r.stdout, (r.stdout[-2000:], r.stderr[-4000:])


def test_pins_under_ubsan(tmp_path):
    so = str(tmp_path / "liboracle_ubsan.so")
    subprocess.run(["gcc", "-std=c11", "-O1", "-g", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                    "-fsanitize=undefined,float-cast-overflow", "-fno-sanitize-recover=all", "-o", so, SRC, "-lm"],
                   check=True)
    _run_pins(so, {"UBSAN_OPTIONS": "halt_on_error=1:print_stacktrace=1"})


def test_pins_under_asan(tmp_path):
    asan = _gcc_file("libasan.so")
    if asan is None:
        pytest.skip("gcc has no libasan.so here")
    so = str(tmp_path / "liboracle_asan.so")
    subprocess.run(["gcc", "-std=c11", "-O1", "-g", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                    "-fsanitize=address", "-fno-omit-frame-pointer", "-o", so, SRC, "-lm"], check=True)
    # the interpreter itself is not instrumented: leaks it reports are not the oracle's
    _run_pins(so, {"LD_PRELOAD": asan, "ASAN_OPTIONS": "detect_leaks=0:abort_on_error=1"})
