"""CPU-only checks of the C ABI: the library loads, exports what include/vla.h declares, and
rejects bad arguments on the host before anything is launched (no GPU needed)."""
import ctypes
import os
import re

import pytest

import paper_2605_11196_amd as vla
from paper_2605_11196_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "vla.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vla_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = vla.load_library()
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


def test_version_and_status_strings():
    assert vla.version() >= 100
    assert vla.status_string(0) == "VLA_OK"
    assert vla.status_string(1) == "VLA_ERR_INVALID_ARG"
    assert vla.status_string(2) == "VLA_ERR_UNSUPPORTED"
    assert vla.status_string(3) == "VLA_ERR_WORKSPACE"
    assert vla.status_string(4) == "VLA_ERR_HIP"
    assert vla.status_string(99) == "VLA_ERR_UNKNOWN"


def test_default_opts():
    o = binding.VlaOpts()
    vla.load_library().vla_default_opts(ctypes.byref(o))
    assert abs(o.lambda0 - 0.1) < 1e-7 and abs(o.eps - 1e-4) < 1e-10 and o.mode == vla.MODE_AUTO
    assert o.u is None and o.u_scale == 1.0 and o.refresh_period == 0 and abs(o.refresh_eta - 1e-3) < 1e-9
    assert o.step_offset == 0 and o.normalise_output == 0 and o.feature_map == 0
    assert o.zkey0 is None and o.zkey_T is None


def test_opts_struct_layout_matches_the_header():
    """ctypes mirror of vla_opts: field order and count as declared in include/vla.h."""
    text = open(os.path.join(ROOT, "include", "vla.h")).read()
    body = re.search(r"typedef struct vla_opts \{(.*?)\} vla_opts;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    names = re.findall(r"(\w+)\s*;", body)
    assert names == [f[0] for f in binding.VlaOpts._fields_]


def test_options_run_on_the_block_kernel_or_the_scan_family():
    assert vla.resolve_mode(2, 2, 64, 128, 128, vla.VLA_BF16) == vla.MODE_CHUNKED
    for d, want in ((128, vla.MODE_CHUNKED), (64, vla.MODE_CHUNKED), (32, vla.MODE_CHUNKED),
                    (96, vla.MODE_CHUNKED), (16, vla.MODE_CHUNKED)):
        assert vla.resolve_mode(2, 2, 64, d, d, vla.VLA_BF16, refresh_period=20) == want
    # few heads on a long sequence: the time-parallel mode carries every option but the identity refresh
    assert vla.resolve_mode(1, 4, 65536, 64, 64, vla.VLA_BF16, normalise_output=1) == vla.MODE_TIME_PARALLEL
    assert vla.resolve_mode(1, 16, 131072, 64, 64, vla.VLA_BF16, u=FAKE, normalise_output=1,
                            feature_map=1) == vla.MODE_TIME_PARALLEL
    assert vla.resolve_mode(1, 4, 65536, 64, 64, vla.VLA_BF16, normalise_output=1,
                            refresh_period=20) == vla.MODE_CHUNKED
    assert vla.resolve_mode(1, 4, 65536, 96, 96, vla.VLA_BF16, normalise_output=1) == vla.MODE_TIME_PARALLEL
    assert vla.resolve_mode(1, 4, 65536, 16, 16, vla.VLA_BF16, normalise_output=1) == vla.MODE_CHUNKED
    assert vla.resolve_mode(2, 2, 64, 128, 128, vla.VLA_BF16, mode=vla.MODE_CHUNKED, normalise_output=1) == vla.MODE_CHUNKED
    assert vla.resolve_mode(2, 2, 64, 128, 128, vla.VLA_BF16, mode=vla.MODE_SCAN, normalise_output=1) == vla.MODE_SCAN
    for mode in (vla.MODE_TWO_PHASE, vla.MODE_TIME_PARALLEL):
        assert vla.resolve_mode(2, 2, 64, 128, 128, vla.VLA_BF16, mode=mode, normalise_output=1) == mode
        assert vla.resolve_mode(2, 2, 64, 128, 128, vla.VLA_BF16, mode=mode, u=FAKE, u_scale=0.5) == mode
        assert vla.resolve_mode(2, 2, 64, 128, 128, vla.VLA_BF16, mode=mode, refresh_period=20) == -1
        assert vla.resolve_mode(2, 2, 64, 128, 128, vla.VLA_BF16, mode=mode, feature_map=1) == mode
    # the feature map alone keeps the plain routing
    assert vla.resolve_mode(1, 16, 131072, 64, 64, vla.VLA_BF16, feature_map=1) == vla.MODE_TIME_PARALLEL
    assert vla.resolve_mode(64, 32, 8192, 128, 128, vla.VLA_BF16, feature_map=1) == vla.MODE_CHUNKED
    assert vla.resolve_mode(2, 2, 64, 96, 96, vla.VLA_BF16, mode=vla.MODE_CHUNKED, normalise_output=1) == vla.MODE_CHUNKED
    assert vla.resolve_mode(2, 2, 64, 16, 16, vla.VLA_BF16, mode=vla.MODE_CHUNKED, normalise_output=1) == vla.MODE_CHUNKED
    # d = 96 has every mode; d = 16 has no segment modes
    assert vla.resolve_mode(2, 2, 64, 96, 96, vla.VLA_BF16) == vla.MODE_CHUNKED
    assert vla.resolve_mode(1, 4, 65536, 96, 96, vla.VLA_BF16, feature_map=1) == vla.MODE_TIME_PARALLEL
    assert vla.resolve_mode(2, 2, 64, 96, 96, vla.VLA_BF16, mode=vla.MODE_TIME_PARALLEL) == vla.MODE_TIME_PARALLEL
    assert vla.resolve_mode(2, 2, 64, 96, 96, vla.VLA_BF16, mode=vla.MODE_TWO_PHASE) == vla.MODE_TWO_PHASE
    assert vla.resolve_mode(2, 2, 64, 16, 16, vla.VLA_BF16, mode=vla.MODE_TIME_PARALLEL) == -1
    assert vla.resolve_mode(2, 2, 64, 16, 16, vla.VLA_BF16) == vla.MODE_CHUNKED     # plain block kernel at d = 16
    assert vla.resolve_mode(2, 2, 64, 16, 16, vla.VLA_BF16, refresh_period=5) == vla.MODE_CHUNKED


FAKE = 0x10000  # a 16-byte aligned non-null address; never dereferenced on these paths


def call(**kw):
    a = dict(q=FAKE, k=FAKE + 0x1000, v=FAKE + 0x2000, S0=0, A0=0, o=FAKE + 0x3000, S_T=0, A_T=0,
             B=1, H=1, T=8, d_k=16, d_v=16, io_dtype=vla.VLA_F32)
    opt = dict(lambda0=None, eps=None, mode=None, workspace=0, workspace_bytes=0)
    for key, val in kw.items():
        (a if key in a else opt)[key] = val
    return vla.vla_forward_raw(a["q"], a["k"], a["v"], a["S0"], a["A0"], a["o"], a["S_T"], a["A_T"],
                               a["B"], a["H"], a["T"], a["d_k"], a["d_v"], a["io_dtype"], **opt)


@pytest.mark.parametrize("kw,status", [
    (dict(B=0), 1), (dict(H=-1), 1), (dict(T=-1), 1), (dict(d_k=0, d_v=0), 1),
    (dict(io_dtype=7), 1), (dict(mode=9), 1), (dict(lambda0=0.0), 1), (dict(eps=-1.0), 1),
    (dict(refresh_period=-1), 1), (dict(step_offset=-5), 1), (dict(step_offset=2**31 - 20, refresh_period=4), 1), (dict(u=FAKE + 2), 1), (dict(zkey_T=FAKE + 4), 1),
    (dict(mode=3, d_k=64, d_v=64, refresh_period=3), 2), (dict(mode=4, d_k=64, d_v=64, normalise_output=1, refresh_period=5), 2),
    (dict(mode=3, d_k=16, d_v=16), 2),
    (dict(q=0), 1), (dict(o=0), 1), (dict(q=FAKE + 4), 1), (dict(S0=FAKE + 8), 1),
    (dict(o=FAKE), 1),                       # o aliases q
    (dict(o=FAKE + 0x100), 1),               # o starts inside q (512 bytes at FAKE)
    (dict(o=FAKE + 0x1000 - 0x100), 1),      # o ends inside k
    (dict(u=FAKE + 0x3000 - 0x100), 1),      # the penalty directions end inside o
    (dict(zkey0=FAKE + 0x3000 + 0x1f0, normalise_output=1), 1),   # the carried key sum starts inside o
    (dict(S0=FAKE + 0x5000, S_T=FAKE + 0x5100), 1),   # S_T may be S0 itself, not a shifted copy of it
    (dict(A0=FAKE + 0x5000, A_T=FAKE + 0x4f00), 1),
    (dict(A_T=FAKE + 0x3100), 1),            # a state output inside o
    (dict(S_T=FAKE + 0x6000, A_T=FAKE + 0x6200), 1),  # the two state outputs inside each other
    (dict(zkey0=FAKE + 0x7000, zkey_T=FAKE + 0x7010, normalise_output=1), 1),
    (dict(mode=3, d_k=64, d_v=64, workspace=FAKE + 0x2800, workspace_bytes=1 << 20), 1),   # workspace over v and o
    (dict(d_k=48, d_v=48), 2), (dict(d_k=16, d_v=48), 2), (dict(d_k=96, d_v=48), 2), (dict(d_k=256, d_v=256), 2),
    (dict(d_k=16, d_v=32, mode=3), 2), (dict(d_k=64, d_v=128, refresh_period=4, mode=3), 2),   # rectangular heads:
    (dict(d_k=96, d_v=64, mode=4, refresh_period=4), 2), (dict(d_k=16, d_v=128, mode=4, normalise_output=1), 2),   # no refresh in the
    (dict(d_k=16, d_v=64, mode=4), 2), (dict(d_k=64, d_v=48, mode=3), 2),   # segment modes, none of them at d_k = 16, sizes outside the set
])
def test_host_side_validation_returns_status_without_launch(kw, status):
    assert call(**kw) == status


def decode_call(**kw):
    a = dict(q=FAKE, k=FAKE + 0x1000, v=FAKE + 0x2000, S=FAKE + 0x4000, A=FAKE + 0x8000, o=FAKE + 0x3000,
             B=1, H=1, d_k=16, d_v=16, io_dtype=vla.VLA_F32)
    opt = {}
    for key, val in kw.items():
        (a if key in a else opt)[key] = val
    return vla.vla_decode_step_raw(a["q"], a["k"], a["v"], a["S"], a["A"], a["o"], a["B"], a["H"],
                                   a["d_k"], a["d_v"], a["io_dtype"], **opt)


@pytest.mark.parametrize("kw,status", [
    (dict(B=0), 1), (dict(io_dtype=3), 1), (dict(eps=0.0), 1),
    (dict(S=0), 1), (dict(A=0), 1), (dict(o=0), 1), (dict(k=0), 1),     # the state is required here
    (dict(A=FAKE + 0x8004), 1), (dict(o=FAKE + 0x1000), 1),             # misaligned; o aliases k
    (dict(o=FAKE + 0x1000 + 0x20), 1), (dict(A=FAKE + 0x4100), 1),      # o inside k; A inside S (1024 bytes)
    (dict(o=FAKE + 0x4000 + 0x3f0), 1), (dict(u=FAKE + 0x3000 - 0x10), 1),   # o inside S; u ends inside o
    (dict(d_k=48, d_v=48), 2), (dict(d_k=96, d_v=48, normalise_output=1), 2),
    (dict(d_k=32, d_v=24, refresh_period=2), 2), (dict(d_k=8, d_v=32, feature_map=1), 2),   # sizes outside the set
    (dict(u=FAKE + 2), 1), (dict(zkey_T=FAKE + 4), 1), (dict(refresh_period=-2), 1),   # option arguments are checked too
])
def test_decode_step_host_side_validation(kw, status):
    assert decode_call(**kw) == status


def test_zero_tokens_without_state_outputs_is_ok_and_launches_nothing():
    assert call(T=0, q=0, k=0, v=0, o=0) == 0


def test_workspace_query_and_mode_resolution():
    assert vla.vla_forward_workspace_bytes(1, 1, 8, 16, 16, vla.VLA_F32, mode=vla.MODE_SCAN) == 0
    assert vla.vla_forward_workspace_bytes(0, 1, 8, 16, 16, vla.VLA_F32) == 0
    assert vla.resolve_mode(1, 1, 8, 16, 16, vla.VLA_F32, mode=vla.MODE_SCAN) == vla.MODE_SCAN
    assert vla.resolve_mode(1, 1, 8, 48, 48, vla.VLA_F32) == -1
    assert vla.resolve_mode(64, 32, 8192, 128, 128, vla.VLA_BF16) == vla.MODE_CHUNKED
    assert vla.resolve_mode(1, 16, 131072, 64, 64, vla.VLA_BF16) == vla.MODE_TIME_PARALLEL
    assert vla.resolve_mode(1, 16, 512, 64, 64, vla.VLA_BF16) == vla.MODE_TIME_PARALLEL   # few heads: from T = 512
    assert vla.resolve_mode(1, 16, 500, 64, 64, vla.VLA_BF16) == vla.MODE_CHUNKED
    assert vla.resolve_mode(1, 128, 512, 64, 64, vla.VLA_BF16) == vla.MODE_CHUNKED
    assert vla.resolve_mode(1, 128, 1024, 64, 64, vla.VLA_BF16) == vla.MODE_TIME_PARALLEL
    assert vla.resolve_mode(1, 16, 131072, 96, 96, vla.VLA_BF16) == vla.MODE_TIME_PARALLEL
    assert vla.resolve_mode(1, 16, 131072, 16, 16, vla.VLA_BF16) == vla.MODE_CHUNKED   # no segment modes at d = 16
    # value heads of another size than the key heads: the same routing by the key head size (few heads on a
    # long sequence -> time-parallel), every mode; no segment modes at d_k = 16
    assert vla.resolve_mode(4, 4, 4096, 64, 128, vla.VLA_BF16) == vla.MODE_TIME_PARALLEL
    assert vla.resolve_mode(64, 32, 4096, 64, 128, vla.VLA_BF16) == vla.MODE_CHUNKED
    assert vla.resolve_mode(4, 4, 4096, 64, 128, vla.VLA_BF16, mode=vla.MODE_SCAN) == vla.MODE_SCAN
    assert vla.resolve_mode(4, 4, 4096, 64, 128, vla.VLA_BF16, mode=vla.MODE_TIME_PARALLEL) == vla.MODE_TIME_PARALLEL
    assert vla.resolve_mode(4, 4, 4096, 128, 16, vla.VLA_BF16, mode=vla.MODE_TWO_PHASE) == vla.MODE_TWO_PHASE
    assert vla.resolve_mode(4, 4, 4096, 16, 32, vla.VLA_BF16) == vla.MODE_CHUNKED
    assert vla.resolve_mode(4, 4, 4096, 16, 32, vla.VLA_BF16, mode=vla.MODE_TIME_PARALLEL) == -1
    # every pair of head sizes runs on the block kernels (the waves of a head share out the row tiles of S, evenly
    # or in turn), with or without options
    assert vla.resolve_mode(4, 4, 4096, 16, 64, vla.VLA_BF16) == vla.MODE_CHUNKED
    assert vla.resolve_mode(64, 32, 4096, 32, 128, vla.VLA_BF16) == vla.MODE_CHUNKED
    assert vla.resolve_mode(64, 32, 4096, 64, 96, vla.VLA_BF16, feature_map=1) == vla.MODE_CHUNKED
    assert vla.resolve_mode(64, 32, 4096, 128, 32, vla.VLA_BF16) == vla.MODE_CHUNKED
    assert vla.resolve_mode(64, 32, 4096, 96, 64, vla.VLA_BF16) == vla.MODE_CHUNKED
    assert vla.resolve_mode(64, 32, 4096, 64, 16, vla.VLA_BF16) == vla.MODE_CHUNKED
    assert vla.resolve_mode(64, 32, 4096, 32, 128, vla.VLA_BF16, normalise_output=1) == vla.MODE_CHUNKED
    assert vla.resolve_mode(4, 4, 4096, 32, 128, vla.VLA_BF16, u=FAKE, refresh_period=20) == vla.MODE_CHUNKED
    assert vla.resolve_mode(4, 4, 4096, 32, 128, vla.VLA_BF16, mode=vla.MODE_CHUNKED, normalise_output=1) == vla.MODE_CHUNKED
    assert vla.resolve_mode(4, 4, 4096, 32, 128, vla.VLA_BF16, normalise_output=1) == vla.MODE_TIME_PARALLEL
    assert vla.resolve_mode(4, 4, 4096, 32, 128, vla.VLA_BF16, mode=vla.MODE_TIME_PARALLEL, normalise_output=1) == vla.MODE_TIME_PARALLEL
    assert vla.resolve_mode(4, 4, 4096, 32, 128, vla.VLA_BF16, mode=vla.MODE_TIME_PARALLEL, refresh_period=5) == -1
    assert vla.resolve_mode(4, 4, 4096, 32, 48, vla.VLA_BF16) == -1


def test_time_parallel_workspace_follows_the_segment_plan():
    """Workspace = the two-phase region (per 16-token block: 16 reciprocal key norms, W [d][16], Z and -NQ^T
    [16][16], 16 write strengths and 16 read-out denominators) + per (head, segment) one float64 and four
    float32 d x d matrices (Gram, A start, P, Q, S start) and one float64 and one float32 d-vector (key sums);
    one segment needs nothing beyond the two-phase region."""
    B, H, T, d = 1, 16, 8192, 64
    two = vla.vla_forward_workspace_bytes(B, H, T, d, d, vla.VLA_BF16, mode=vla.MODE_TWO_PHASE)
    nblk = T // 16
    assert two == B * H * nblk * (16 + 16 * d + 544) * 4
    tp = lambda s: vla.vla_forward_workspace_bytes(B, H, T, d, d, vla.VLA_BF16,
                                                   mode=vla.MODE_TIME_PARALLEL, segments=s)
    assert tp(1) == two
    for s in (2, 8, 64):
        assert tp(s) == two + B * H * s * (d * d * 6 + d * 3) * 4
    # 512 blocks in 100 segments: ceil(512/100) = 6 blocks each -> 86 non-empty segments
    assert tp(100) == two + B * H * 86 * (d * d * 6 + d * 3) * 4
    # never more segments than blocks, never more than 256
    assert vla.vla_forward_workspace_bytes(1, 1, 64, d, d, vla.VLA_F32, mode=vla.MODE_TIME_PARALLEL,
                                           segments=99) == 4 * (16 + 16 * d + 544) * 4 + 4 * (d * d * 6 + d * 3) * 4
    big = vla.vla_forward_workspace_bytes(1, 1, 16 * 4096, d, d, vla.VLA_F32,
                                          mode=vla.MODE_TIME_PARALLEL, segments=100000)
    assert big == 4096 * (16 + 16 * d + 544) * 4 + 256 * (d * d * 6 + d * 3) * 4
    # the library's own choice: about 1024 (head, segment) pairs, segments of at least 16 blocks
    auto = tp(0)
    assert auto == two + B * H * 32 * (d * d * 6 + d * 3) * 4    # 512 blocks / 16 = 32 < 1024 / 16 heads = 64
    # with a separate penalty direction or the normalised read-out at d = 64: about 768 pairs, 32 blocks
    for (T2, want) in ((131072, 48), (16384, 32), (4096, 16)):
        two2 = vla.vla_forward_workspace_bytes(B, H, T2, d, d, vla.VLA_BF16, mode=vla.MODE_TWO_PHASE,
                                               normalise_output=1)
        got = vla.vla_forward_workspace_bytes(B, H, T2, d, d, vla.VLA_BF16, mode=vla.MODE_TIME_PARALLEL,
                                              normalise_output=1)
        assert got == two2 + B * H * want * (d * d * 6 + d * 3) * 4, T2
    # whole rounds of 256 pairs: 24 heads x 16 segments would be a round and a half; two rounds = 21 segments
    # asked for, 256 blocks in segments of ceil(256 / 21) = 13 blocks -> 20 segments
    two24 = vla.vla_forward_workspace_bytes(1, 24, 4096, d, d, vla.VLA_BF16, mode=vla.MODE_TWO_PHASE)
    got = vla.vla_forward_workspace_bytes(1, 24, 4096, d, d, vla.VLA_BF16, mode=vla.MODE_TIME_PARALLEL)
    assert got == two24 + 24 * 20 * (d * d * 6 + d * 3) * 4
    # value heads of another size: per (head, segment) Gram (float64), A start and P stay d x d, Q and the S start
    # are d_v x d
    two_r = vla.vla_forward_workspace_bytes(B, H, T, d, 128, vla.VLA_BF16, mode=vla.MODE_TWO_PHASE)
    assert two_r == two
    got = vla.vla_forward_workspace_bytes(B, H, T, d, 128, vla.VLA_BF16, mode=vla.MODE_TIME_PARALLEL, segments=8)
    assert got == two + B * H * 8 * (d * d * 4 + 2 * 128 * d + d * 3) * 4
    # from d = 96: about 512 pairs, segments of at least 32 blocks
    for (T2, want) in ((8192, 16), (32768, 32), (131072, 32)):
        two2 = vla.vla_forward_workspace_bytes(B, H, T2, 128, 128, vla.VLA_BF16, mode=vla.MODE_TWO_PHASE)
        got = vla.vla_forward_workspace_bytes(B, H, T2, 128, 128, vla.VLA_BF16, mode=vla.MODE_TIME_PARALLEL)
        assert got == two2 + B * H * want * (128 * 128 * 6 + 128 * 3) * 4, T2


def test_torch_front_end_refuses_cpu_tensors():
    import torch

    x = torch.zeros(1, 1, 4, 16)
    with pytest.raises(ValueError):
        vla.vla_forward(x, x, x)


def test_device_image_exports_the_static_workspace_symbol():
    """vla_forward_static finds its array through hipGetSymbolAddress, which looks the name up in the device
    code object: the array has to be a global, defined symbol of 64 MiB there (a file-scope static that the
    compiler kept local would only show as a failure on the GPU)."""
    import shutil
    import subprocess
    import tempfile

    readelf = "/opt/rocm/llvm/bin/llvm-readelf"
    bundler = "/opt/rocm/llvm/bin/clang-offload-bundler"
    if not (os.path.exists(readelf) and os.path.exists(bundler) and shutil.which("objcopy")):
        pytest.skip("binutils / ROCm LLVM tools not present")
    with tempfile.TemporaryDirectory() as tmp:
        fat = os.path.join(tmp, "fatbin")
        subprocess.run(["objcopy", "-O", "binary", "--only-section=.hip_fatbin", vla.lib_path(), fat], check=True)
        blob = open(fat, "rb").read()
        magic = b"__CLANG_OFFLOAD_BUNDLE__"
        starts = [i for i in range(len(blob)) if blob.startswith(magic, i)]
        assert starts
        found = []
        for n, (a, b) in enumerate(zip(starts, starts[1:] + [len(blob)])):
            piece, elf = os.path.join(tmp, f"b{n}"), os.path.join(tmp, f"b{n}.elf")
            open(piece, "wb").write(blob[a:b])
            subprocess.run([bundler, "--unbundle", "--type=o", f"--input={piece}",
                            "--targets=hipv4-amdgcn-amd-amdhsa--gfx950", f"--output={elf}"], check=True,
                           capture_output=True)
            syms = subprocess.run([readelf, "-sW", elf], capture_output=True, text=True).stdout
            found += [l.split() for l in syms.splitlines() if l.strip().endswith("scratch") or "7scratch" in l]
    assert found, "no scratch symbol in any device code object"
    assert any(f[2] == str(64 << 20) and f[3] == "OBJECT" and f[4] == "GLOBAL" and f[6] != "UND" for f in found), found
