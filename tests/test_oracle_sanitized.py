"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only, host code only).

``oracle/chai_oracle.c`` is rebuilt with ``-fsanitize=address,undefined`` and every pin is run against that
build in a child interpreter (the sanitizer runtime has to be loaded before anything else, hence the child with
the runtime preloaded in front of whatever the environment already preloads).  An out-of-bounds read, a misaligned
access, a signed overflow in an index computation or a use-after-free inside the oracle ends the child with a
report; so does a failing pin.
"""
import os
import subprocess
import sys

import pytest

from oracle import chai_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(os.path.dirname(O.__file__), "chai_oracle.c")

CHILD = r"""
import sys
sys.path.insert(0, {root!r}); sys.path.insert(0, {tests!r})
import oracle_pins as P
from oracle import chai_oracle as O
with O.use_library({so!r}):
    for pin in P.ALL_PINS:
        pin()
        print("ok", pin.__name__, flush=True)
print("ALL PINS PASSED UNDER THE SANITIZERS", flush=True)
"""


def _runtime(name):
    path = subprocess.run(["gcc", "-print-file-name=" + name], capture_output=True, text=True, check=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def test_all_pins_pass_under_asan_and_ubsan(tmp_path):
    asan = _runtime("libasan.so")
    if asan is None:
        pytest.skip("gcc has no AddressSanitizer runtime here")
    so = tmp_path / "libchai_oracle_san.so"
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
                    "-shared", "-fPIC", SRC, "-o", str(so), "-lm"], check=True)
    env = dict(os.environ)
    env["LD_PRELOAD"] = ":".join(p for p in (asan, env.get("LD_PRELOAD", "")) if p)
    # the interpreter and numpy are not instrumented: their own leaks and link order are not the subject
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0:exitcode=97"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    code = CHILD.format(root=ROOT, tests=os.path.join(ROOT, "tests"), so=str(so))
    res = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, timeout=1200)
    tail = (res.stdout[-2000:] + "\n" + res.stderr[-4000:])
    assert res.returncode == 0, tail
    assert "ALL PINS PASSED UNDER THE SANITIZERS" in res.stdout, tail
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, tail
