"""Host-only sanitizer leg: the oracle compiled with AddressSanitizer and UndefinedBehaviorSanitizer runs the
pin tests in a subprocess (the ASan runtime has to be the first library of the process, so it is put in
front of whatever LD_PRELOAD already names).  No GPU code is involved."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _gcc_file(name):
    out = subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True).stdout.strip()
    return out if os.path.isabs(out) and os.path.exists(out) else None


def _run_pins_under_sanitizers(tmp_path, edit=None):
    tree = str(tmp_path / "tree")
    os.makedirs(os.path.join(tree, "tests"))
    shutil.copytree(os.path.join(ROOT, "oracle"), os.path.join(tree, "oracle"),
                    ignore=shutil.ignore_patterns("*.so", "__pycache__"))
    shutil.copytree(os.path.join(ROOT, "tests", "golden"), os.path.join(tree, "tests", "golden"))
    for name in ("test_oracle_pins.py", "conftest.py"):
        shutil.copy(os.path.join(ROOT, "tests", name), os.path.join(tree, "tests", name))
    shutil.copy(os.path.join(ROOT, "vla_inputs.py"), tree)
    if edit is not None:
        src = os.path.join(tree, "oracle", "vla_oracle.c")
        text = open(src).read()
        assert text.count(edit[0]) == 1
        open(src, "w").write(text.replace(edit[0], edit[1]))
    # no OpenMP: one thread keeps the sanitizer reports readable and the run deterministic
    subprocess.run(["gcc", "-std=c11", "-O1", "-g", "-fPIC", "-shared", "-fno-omit-frame-pointer",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-Wall", "-Wextra",
                    "-ffp-contract=off", os.path.join(tree, "oracle", "vla_oracle.c"), "-o",
                    os.path.join(tree, "oracle", "libvla_oracle.so"), "-lm"], check=True)
    preload = " ".join(x for x in (_gcc_file("libasan.so"), os.environ.get("LD_PRELOAD", "")) if x)
    env = dict(os.environ, PYTHONPATH=tree, PYTHONDONTWRITEBYTECODE="1", LD_PRELOAD=preload,
               # the interpreter itself is not leak-clean; heap errors in the oracle still abort
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=1:halt_on_error=1",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-s", "-p", "no:cacheprovider",
                        os.path.join(tree, "tests", "test_oracle_pins.py")],
                       cwd=tree, env=env, capture_output=True, text=True, timeout=900)
    return r


needs_asan = pytest.mark.skipif(_gcc_file("libasan.so") is None, reason="gcc ships no ASan runtime here")


@needs_asan
def test_pins_pass_on_the_oracle_built_with_asan_and_ubsan(tmp_path):
    r = _run_pins_under_sanitizers(tmp_path)
    assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-3000:])
    assert "AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-3000:]


@needs_asan
def test_the_sanitizer_leg_reports_a_planted_heap_overflow(tmp_path):
    """The leg is live: a work vector allocated one element short in the temporary copy is reported."""
    r = _run_pins_under_sanitizers(
        tmp_path, ("double* z = (double*)malloc(sizeof(double) * dk);",
                   "double* z = (double*)malloc(sizeof(double) * (dk - 1));"))
    assert r.returncode != 0
    assert "heap-buffer-overflow" in r.stderr, r.stderr[-3000:]
