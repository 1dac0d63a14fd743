"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer: its source is compiled once
more with -fsanitize=address,undefined and the oracle's own pins (PSH construction and lookup,
hash2col / col2hash, the convolution and pooling operators) run against that build in a child
process.  Host code only; nothing here touches a GPU."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _libasan():
    try:
        path = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    except (OSError, subprocess.CalledProcessError):
        return None
    return path if os.path.isabs(path) and os.path.exists(path) else None


@pytest.mark.skipif(_libasan() is None, reason="gcc has no libasan.so here")
def test_oracle_pins_under_asan_ubsan(tmp_path):
    sys.path.insert(0, ROOT)
    from oracle import oracle as O
    lib = str(tmp_path / "liboracle_asan.so")
    O.build(force=True, out=lib, extra_flags=("-O1", "-g", "-fno-omit-frame-pointer",
                                              "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"))
    env = dict(os.environ)
    # the sanitizer runtime must come first among the preloaded libraries; whatever is already
    # preloaded stays
    env["LD_PRELOAD"] = ":".join(x for x in (_libasan(), env.get("LD_PRELOAD", "")) if x)
    # python itself is not instrumented: its arenas would all be reported as leaks
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=86"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1"
    env["HCH_ORACLE_LIB"] = lib
    env["OMP_NUM_THREADS"] = "4"
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider",
                          os.path.join(ROOT, "tests", "test_oracle_psh.py"),
                          os.path.join(ROOT, "tests", "test_oracle_ops.py")],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=1500)
    tail = (run.stdout + run.stderr)[-4000:]
    assert run.returncode == 0, tail
    assert "ERROR: AddressSanitizer" not in tail and "runtime error:" not in run.stdout + run.stderr, tail
