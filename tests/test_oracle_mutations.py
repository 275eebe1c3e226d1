"""Mutation check of the oracle pins (CPU only).

Each case plants one plausible mistake in a temporary copy of oracle/vla_oracle.c (a wrong sign, a dropped
term, a pre- instead of post-update operand, a shifted schedule, ...), rebuilds that copy and runs the pin tests
against it in a subprocess: at least one pin must fail.  The planted mistakes live in the oracle only; nothing
here touches the GPU path.
"""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# name -> list of (text in vla_oracle.c, replacement)
MUTANTS = {
    "rank-1 update of A with the wrong sign": [("-= z[i] * z[j] / delta", "+= z[i] * z[j] / delta")],
    "rank-1 update of A without delta": [("-= z[i] * z[j] / delta", "-= z[i] * z[j]")],
    "delta without the 1": [("double delta_raw = 1.0 + dot(u, z, dk);", "double delta_raw = dot(u, z, dk);")],
    "z from the key instead of the penalty direction": [("matvec(A, u, z, dk, dk);", "matvec(A, kh, z, dk, dk);")],
    "write direction from the pre-update A": [
        ("matvec(A, u, z, dk, dk);", "matvec(A, u, z, dk, dk); matvec(A, kh, a, dk, dk);"),
        ("    matvec(A, kh, a, dk, dk);\n    double an", "    double an")],
    "write direction not normalised": [("a[j] = a[j] / aden;", "a[j] = a[j];")],
    "key not normalised": [("kh[j] = kt[j] / kden;", "kh[j] = kt[j];")],
    "additive eps in the key norm": [("double kden = kn > eps ? kn : eps;", "double kden = kn + eps;")],
    "residual with the wrong sign": [("e[i] = vt[i] - dot(", "e[i] = vt[i] + dot(")],
    "residual against q": [("e[i] = vt[i] - dot(S + (size_t)i * dk, kh, dk)",
                            "e[i] = vt[i] - dot(S + (size_t)i * dk, qt, dk)")],
    "S written along the key": [("+= e[i] * a[j]", "+= e[i] * kh[j]")],
    "S update transposed": [("S[(size_t)i * dk + j] += e[i] * a[j]", "S[(size_t)i * dk + j] += e[i % dv] * a[j]"),
                            ("e[i] = vt[i] - dot(S + (size_t)i * dk, kh, dk)",
                             "e[i] = vt[i] - dot(S + (size_t)((i + 1) % dv) * dk, kh, dk)")],
    "read-out before the write": [
        ("    matvec(S, qt, o + (size_t)t * dv, dv, dk);\n", ""),
        ("    for (int i = 0; i < dv; ++i) e[i] = vt[i]", "    matvec(S, qt, o + (size_t)t * dv, dv, dk);\n"
         "    for (int i = 0; i < dv; ++i) e[i] = vt[i]")],
    "refresh one step late": [("(step_offset + t + 1) % refresh_period == 0", "(step_offset + t) % refresh_period == 0")],
    "refresh ignores the step offset": [("(step_offset + t + 1) % refresh_period == 0", "(t + 1) % refresh_period == 0")],
    "refresh counts the offset twice": [("(step_offset + t + 1) % refresh_period == 0",
                                         "(2 * step_offset + t + 1) % refresh_period == 0")],
    "refresh after the write direction": [
        ("    if (refresh_period > 0 && (step_offset + t + 1) % refresh_period == 0)\n"
         "      for (int i = 0; i < dk; ++i) A[(size_t)i * dk + i] += refresh_eta;\n", ""),
        ("    /* residual against the pre-update S",
         "    if (refresh_period > 0 && (step_offset + t + 1) % refresh_period == 0)\n"
         "      for (int i = 0; i < dk; ++i) A[(size_t)i * dk + i] += refresh_eta;\n"
         "    /* residual against the pre-update S")],
    "key sum of the normalised keys": [("zkey[j] += kt[j];", "zkey[j] += kh[j];")],
    "read-out denominator from the previous key sum": [
        ("    for (int j = 0; j < dk; ++j) zkey[j] += kt[j];\n", ""),
        ("      for (int i = 0; i < dv; ++i) o[(size_t)t * dv + i] /= den;\n    }\n",
         "      for (int i = 0; i < dv; ++i) o[(size_t)t * dv + i] /= den;\n    }\n"
         "    for (int j = 0; j < dk; ++j) zkey[j] += kt[j];\n")],
    "supplied u not scaled": [("u[j] = u_scale * (ut[j] / uden);", "u[j] = ut[j] / uden;")],
    "ELU branch at the wrong sign": [("kf[j] = feature_map ? (kr > 0.0 ? kr + 1.0 : exp(kr)) : kr;",
                                      "kf[j] = feature_map ? (kr < 0.0 ? kr + 1.0 : exp(kr)) : kr;")],
}


def _run_pins(tree):
    env = dict(os.environ, PYTHONPATH=tree, PYTHONDONTWRITEBYTECODE="1")
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                           os.path.join(tree, "tests", "test_oracle_pins.py")],
                          cwd=tree, env=env, capture_output=True, text=True, timeout=600)


def _make_tree(tmp_path, edits):
    tree = str(tmp_path / "tree")
    os.makedirs(os.path.join(tree, "tests"))
    shutil.copytree(os.path.join(ROOT, "oracle"), os.path.join(tree, "oracle"),
                    ignore=shutil.ignore_patterns("*.so", "__pycache__"))
    shutil.copytree(os.path.join(ROOT, "tests", "golden"), os.path.join(tree, "tests", "golden"))
    for name in ("test_oracle_pins.py", "conftest.py"):
        shutil.copy(os.path.join(ROOT, "tests", name), os.path.join(tree, "tests", name))
    shutil.copy(os.path.join(ROOT, "vla_inputs.py"), tree)
    src = os.path.join(tree, "oracle", "vla_oracle.c")
    text = open(src).read()
    for old, new in edits:
        assert text.count(old) == 1, f"edit does not apply exactly once: {old!r}"
        text = text.replace(old, new)
    open(src, "w").write(text)
    subprocess.run([sys.executable, os.path.join(tree, "oracle", "build_oracle.py")], check=True,
                   capture_output=True, cwd=tree)
    return tree


def test_unmodified_copy_passes_every_pin(tmp_path):
    """The harness itself: the same temporary tree without an edit is green."""
    r = _run_pins(_make_tree(tmp_path, []))
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_fails_a_pin(name, tmp_path):
    r = _run_pins(_make_tree(tmp_path, MUTANTS[name]))
    assert r.returncode == 1, f"no pin caught: {name}\n{r.stdout[-1500:]}"
    assert " failed" in r.stdout
