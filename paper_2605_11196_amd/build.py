"""Compile the HIP sources under csrc/ into paper_2605_11196_amd/libvla.so for gfx950.

hipcc cross-compiles without a GPU.  Packed-FP32 instruction selection is switched
off for all device code (the -packed-fp32-ops target feature).  Every source is
compiled to an object of its own (in parallel) and the objects are linked; a plain
call compiles everything, `--incremental` skips objects newer than their source
and every header.
"""
import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
OUT = os.path.join(HERE, "libvla.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def headers():
    return sorted(glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(HERE, "..", "include", "*.h")))


def object_path(src):
    return os.path.join(OBJ, os.path.splitext(os.path.basename(src))[0] + ".o")


def compile_one(src, verbose=False, extra=()):
    """One translation unit to its object; returns what the compiler printed (remarks included)."""
    cmd = [HIPCC] + FLAGS + list(extra) + ["-c", src, "-o", object_path(src)]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise subprocess.CalledProcessError(r.returncode, cmd)
    return r.stdout + r.stderr


def build(verbose: bool = False, extra=(), incremental: bool = False, jobs: int = 8) -> str:
    os.makedirs(OBJ, exist_ok=True)
    srcs = sources()
    todo = srcs
    if incremental:
        newest_header = max(os.path.getmtime(h) for h in headers())
        todo = [s for s in srcs if not os.path.exists(object_path(s)) or
                os.path.getmtime(object_path(s)) < max(os.path.getmtime(s), newest_header)]
    with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(todo) or 1))) as pool:
        for out in pool.map(lambda s: compile_one(s, verbose, extra), todo):
            if verbose and out.strip():
                # the host pass does not know the device-only target feature: harmless, not repeated here
                lines = [l for l in out.splitlines() if "packed-fp32-ops" not in l]
                if lines:
                    print("\n".join(lines), flush=True)
    link = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + [object_path(s) for s in srcs] + ["-o", OUT]
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.run(link, check=True)
    return OUT


def resource_usage(src, extra=()):
    """The compiler's own resource report for every kernel of one source (device pass only, nothing is
    written next to the library): {demangled kernel name: {"VGPRs": n, "AGPRs": n, "ScratchSize": bytes per
    lane, "VGPRSpill": n, "SGPRSpill": n, "Occupancy": waves per SIMD, "LDSSize": bytes, ...}}."""
    import re
    import tempfile

    with tempfile.TemporaryDirectory() as tmp:
        cmd = [HIPCC] + FLAGS + list(extra) + ["--cuda-device-only", "-Rpass-analysis=kernel-resource-usage",
                                               "-c", src, "-o", os.path.join(tmp, "dev.o")]
        r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise subprocess.CalledProcessError(r.returncode, cmd)
    out, cur = {}, None
    keys = {"TotalSGPRs": "SGPRs", "VGPRs": "VGPRs", "AGPRs": "AGPRs", "ScratchSize [bytes/lane]": "ScratchSize",
            "Occupancy [waves/SIMD]": "Occupancy", "SGPRs Spill": "SGPRSpill", "VGPRs Spill": "VGPRSpill",
            "LDS Size [bytes/block]": "LDSSize"}
    for line in (r.stdout + r.stderr).splitlines():
        m = re.search(r"remark: (?:\S+: )?\s*Function Name: (\S+)", line)
        if m:
            cur = out.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark: (?:\S+: )?\s*([A-Za-z][A-Za-z /\[\]]*?): (\d+)", line)
        if m and cur is not None and m.group(1).strip() in keys:
            cur[keys[m.group(1).strip()]] = int(m.group(2))
    names = list(out)
    if names:
        dem = subprocess.run(["c++filt"] + names, capture_output=True, text=True).stdout.split("\n")
        out = {d.strip() or n: out[n] for n, d in zip(names, dem)}
    return out


if __name__ == "__main__":
    args = sys.argv[1:]
    inc = "--incremental" in args
    print(build(verbose=True, extra=[a for a in args if a != "--incremental"], incremental=inc))
