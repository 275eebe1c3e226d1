"""GPU parity for the optional lines of Algorithm 1 (separate penalty direction u, periodic identity
refresh, normalised read-out with the running key sum, ELU+1 feature map): the general scan kernel and the
general block kernel through the C ABI against the fp64 oracle, same error metric and tolerances as the main
parity tests."""
import numpy as np
import pytest

import oracle
import vla_inputs
from parity_utils import TOL, slab_rel_err, to_np

pytestmark = pytest.mark.gpu


SCAN, BLOCK = 1, 2


def modes_for(d):
    return [SCAN, BLOCK]


def run_both(q, k, v, *, dtype="f32", u=None, S0=None, A0=None, zkey0=None, mode=None, segments=None, **opt):
    import torch

    import paper_2605_11196_amd as vla

    if dtype == "bf16":
        q, k, v = (vla_inputs.round_to_bf16(x) for x in (q, k, v))
        u = None if u is None else vla_inputs.round_to_bf16(u)
    ref = oracle.forward(q, k, v, S0, A0, u=u, zkey0=zkey0, **opt)
    dev = torch.device("cuda:0")
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    t = lambda x, dt=tdt: None if x is None else torch.from_numpy(np.ascontiguousarray(x)).to(dev).to(dt)
    o, S_T, A_T, zk = vla.vla_forward(t(q), t(k), t(v), t(S0, torch.float32), t(A0, torch.float32),
                                       u=t(u), zkey0=t(zkey0, torch.float32), return_zkey=True, mode=mode,
                                       lambda0=opt.get("lambda0"), eps=opt.get("eps"),
                                       u_scale=opt.get("u_scale"), refresh_period=opt.get("refresh_period"),
                                       refresh_eta=opt.get("refresh_eta"), step_offset=opt.get("step_offset"),
                                       normalise_output=opt.get("normalise_output"),
                                       feature_map=opt.get("feature_map"), segments=segments)
    torch.cuda.synchronize()
    got = dict(o=to_np(o), S_T=to_np(S_T), A_T=to_np(A_T), zkey_T=to_np(zk))
    return got, ref


def assert_close(got, ref, tol):
    errs = dict(o=slab_rel_err(got["o"], ref["o"], 2), S=slab_rel_err(got["S_T"], ref["S_T"], 2),
                A=slab_rel_err(got["A_T"], ref["A_T"], 2), z=slab_rel_err(got["zkey_T"], ref["zkey_T"], 1))
    assert all(np.isfinite(x).all() for x in got.values())
    assert max(errs.values()) <= tol, errs
    return errs


OPTION_SETS = {
    "supplied_u": dict(with_u=True),
    "supplied_u_scaled": dict(with_u=True, u_scale=0.125),
    "refresh": dict(refresh_period=20, refresh_eta=1e-3),
    "normalised": dict(normalise_output=True, positive=True),
    "feature_map": dict(feature_map=True),
    "algorithm1": dict(with_u=True, u_scale=0.125, refresh_period=20, refresh_eta=1e-3,
                       normalise_output=True, feature_map=True),
    "only_key_sum": dict(want_zkey_only=True),
}


@pytest.mark.parametrize("name", list(OPTION_SETS))
@pytest.mark.parametrize("d,T,dtype", [(16, 70, "f32"), (64, 130, "f32"), (128, 45, "f32"), (96, 58, "f32"), (32, 97, "bf16"),
                                       (128, 64, "bf16")])
def test_option_parity(name, d, T, dtype):
    cfg = dict(OPTION_SETS[name])
    rng = np.random.default_rng(900 + d + T)
    q, k, v = vla_inputs.gaussian_qkv(2, 2, T, d, seed=700 + d + T)
    if cfg.pop("positive", False):      # a meaningful denominator needs non-negative features
        q, k = np.abs(q) + 0.05, np.abs(k) + 0.05
    u = rng.standard_normal(q.shape).astype(np.float32) if cfg.pop("with_u", False) else None
    cfg.pop("want_zkey_only", None)
    for mode in modes_for(d):
        got, ref = run_both(q, k, v, dtype=dtype, u=u, lambda0=0.1, mode=mode, **cfg)
        print(name, d, T, dtype, mode, assert_close(got, ref, TOL[dtype]))


@pytest.mark.parametrize("mode", [SCAN, BLOCK])
def test_split_sequence_with_every_option_carries_state(mode):
    """[0,T1) then [T1,T) with S, A, the key sum and the refresh phase carried == one call."""
    d, T, T1 = 64, 101, 37
    rng = np.random.default_rng(5)
    q, k, v = vla_inputs.gaussian_qkv(1, 3, T, d, seed=55)
    u = rng.standard_normal(q.shape).astype(np.float32)
    opt = dict(lambda0=0.1, u_scale=0.125, refresh_period=8, refresh_eta=1e-2, normalise_output=True,
               feature_map=True, mode=mode)
    full, ref = run_both(q, k, v, u=u, **opt)
    assert_close(full, ref, 1e-4)
    a, _ = run_both(q[:, :, :T1], k[:, :, :T1], v[:, :, :T1], u=u[:, :, :T1], **opt)
    b, _ = run_both(q[:, :, T1:], k[:, :, T1:], v[:, :, T1:], u=u[:, :, T1:], S0=a["S_T"], A0=a["A_T"],
                    zkey0=a["zkey_T"], step_offset=T1, **opt)
    joined = dict(o=np.concatenate([a["o"], b["o"]], axis=2), S_T=b["S_T"], A_T=b["A_T"], zkey_T=b["zkey_T"])
    assert_close(joined, ref, 1e-4)


@pytest.mark.parametrize("period", [1, 2, 5, 16, 17, 33])
@pytest.mark.parametrize("offset", [0, 3])
def test_block_kernel_takes_refresh_steps_anywhere_inside_a_block(period, offset):
    """Refresh steps fall anywhere inside the 16-token blocks: periods below, at and above the block length
    (several refreshes per block, one, or none), with a carried phase."""
    d, T = 32, 77
    q, k, v = vla_inputs.gaussian_qkv(1, 2, T, d, seed=300 + period)
    opt = dict(lambda0=0.1, refresh_period=period, refresh_eta=5e-3, step_offset=offset)
    got, ref = run_both(q, k, v, mode=BLOCK, **opt)
    print(period, offset, assert_close(got, ref, 1e-4))


@pytest.mark.parametrize("d", [32, 64, 128])
def test_block_kernel_options_on_zero_keys_and_tiny_directions(d):
    """Zero keys (no write, the read still happens), zero and tiny penalty directions (no A update for a zero
    u; a tiny one is normalised like any other), and a sequence shorter than a block."""
    T = 23
    rng = np.random.default_rng(d)
    q, k, v = vla_inputs.gaussian_qkv(2, 2, T, d, seed=40 + d)
    u = rng.standard_normal(q.shape).astype(np.float32)
    k[:, :, 3] = 0.0
    k[:, :, 17:19] = 0.0
    u[:, :, 5] = 0.0
    u[:, :, 9] *= 1e-7
    opt = dict(lambda0=0.1, u_scale=d ** -0.5, refresh_period=7, refresh_eta=1e-3)
    got, ref = run_both(q, k, v, u=u, mode=BLOCK, **opt)
    print(d, assert_close(got, ref, 1e-4))
    got, ref = run_both(q[:, :, :5], k[:, :, :5], v[:, :, :5], u=u[:, :, :5], mode=BLOCK, **opt)
    print(d, "T=5", assert_close(got, ref, 1e-4))


def test_block_kernel_with_options_holds_the_tolerance_on_a_long_sequence():
    d, T = 64, 6000
    rng = np.random.default_rng(11)
    q, k, v = vla_inputs.gaussian_qkv(1, 2, T, d, seed=77)
    u = rng.standard_normal(q.shape).astype(np.float32)
    opt = dict(lambda0=0.1, u_scale=0.125, refresh_period=20, refresh_eta=1e-3, normalise_output=True,
               feature_map=True)
    got, ref = run_both(q, k, v, u=u, mode=BLOCK, **opt)
    print(assert_close(got, ref, 1e-4))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("d,T,mode,segments", [(64, 2100, 4, 5), (128, 1100, 4, 3), (32, 700, 4, 4), (64, 300, 3, None),
                                               (128, 130, 3, None), (128, 257, 2, None)])
def test_feature_map_alone_runs_on_every_block_mode(d, T, mode, segments, dtype):
    """ELU+1 on q and k with no other option: plain block kernel, two-phase and time-parallel modes (the Gram
    sums behind the segment boundaries are then sums over the mapped keys)."""
    import torch

    import paper_2605_11196_amd as vla

    q, k, v = vla_inputs.gaussian_qkv(1, 3, T, d, seed=d + T)
    if dtype == "bf16":
        q, k, v = (vla_inputs.round_to_bf16(x) for x in (q, k, v))
    ref = oracle.forward(q, k, v, lambda0=0.1, feature_map=True)
    dev = torch.device("cuda:0")
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    t = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to(dev).to(tdt)
    o, S_T, A_T = vla.vla_forward(t(q), t(k), t(v), lambda0=0.1, feature_map=True, mode=mode, segments=segments)
    torch.cuda.synchronize()
    errs = dict(o=slab_rel_err(to_np(o), ref["o"], 2), S=slab_rel_err(to_np(S_T), ref["S_T"], 2),
                A=slab_rel_err(to_np(A_T), ref["A_T"], 2))
    print(d, T, mode, dtype, errs)
    assert max(errs.values()) <= TOL[dtype], errs


def test_refresh_is_refused_by_the_segment_modes_and_taken_by_the_block_kernel():
    import torch

    import paper_2605_11196_amd as vla

    dev = torch.device("cuda:0")
    x = torch.randn(1, 1, 32, 64, device=dev)
    for mode in (vla.MODE_TWO_PHASE, vla.MODE_TIME_PARALLEL):
        with pytest.raises(vla.VlaError) as e:
            vla.vla_forward(x, x, x, mode=mode, refresh_period=4)
        assert e.value.status == 2
    for mode in (None, vla.MODE_CHUNKED, vla.MODE_SCAN):
        o, _, _ = vla.vla_forward(x, x, x, mode=mode, refresh_period=4)
        torch.cuda.synchronize()
        assert torch.isfinite(o).all()


@pytest.mark.parametrize("d", [32, 128])
def test_block_kernel_with_options_is_deterministic_and_replays_in_a_hip_graph(d):
    """Same bits on every run (no atomics, fixed reduction orders); a captured call replays like the eager one
    on new inputs; S, A and the key sum may be updated in place."""
    import torch

    import paper_2605_11196_amd as vla

    B, H, T = 2, 3, 150
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(3)
    q, k, v, u = (torch.randn(B, H, T, d, device=dev, generator=gen) for _ in range(4))
    o = torch.empty_like(q)
    S = torch.empty(B, H, d, d, device=dev)
    A = torch.empty(B, H, d, d, device=dev)
    zk = torch.empty(B, H, d, device=dev)
    opt = dict(u=u.data_ptr(), u_scale=0.25, refresh_period=20, refresh_eta=1e-3, normalise_output=1,
               feature_map=1, zkey_T=zk.data_ptr(), mode=BLOCK)

    def call(stream):
        rc = vla.vla_forward_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), 0, 0, o.data_ptr(), S.data_ptr(),
                                 A.data_ptr(), B, H, T, d, d, vla.VLA_F32, stream=stream.cuda_stream, **opt)
        assert rc == 0

    side = torch.cuda.Stream(dev)
    side.wait_stream(torch.cuda.current_stream(dev))
    with torch.cuda.stream(side):
        call(side)
    side.synchronize()
    first = [x.clone() for x in (o, S, A, zk)]
    with torch.cuda.stream(side):
        call(side)
    side.synchronize()
    for a, b in zip(first, (o, S, A, zk)):
        assert torch.equal(a, b)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        call(torch.cuda.current_stream(dev))
    for rep in range(3):
        for x in (q, k, v, u):
            x.copy_(torch.randn(B, H, T, d, device=dev, generator=gen))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [x.clone() for x in (o, S, A, zk)]
        call(torch.cuda.current_stream(dev))
        torch.cuda.synchronize()
        for g, e in zip(got, (o, S, A, zk)):
            assert torch.equal(g, e), rep

    # state carried in place: S_T = S0, A_T = A0, zkey_T = zkey0 (second half of a split sequence)
    T1 = 70
    sl = lambda x, a, b: x[:, :, a:b].contiguous()
    parts = [(sl(q, 0, T1), sl(k, 0, T1), sl(v, 0, T1), sl(u, 0, T1)), (sl(q, T1, T), sl(k, T1, T), sl(v, T1, T), sl(u, T1, T))]
    call(torch.cuda.current_stream(dev))
    torch.cuda.synchronize()
    want = [x.clone() for x in (o, S, A, zk)]
    S2 = torch.zeros(B, H, d, d, device=dev)
    A2 = (torch.eye(d, device=dev) * 10.0).repeat(B, H, 1, 1).contiguous()
    z2 = torch.zeros(B, H, d, device=dev)
    outs = []
    off = 0
    for qq, kk, vv, uu in parts:
        oo = torch.empty_like(qq)
        rc = vla.vla_forward_raw(qq.data_ptr(), kk.data_ptr(), vv.data_ptr(), S2.data_ptr(), A2.data_ptr(),
                                 oo.data_ptr(), S2.data_ptr(), A2.data_ptr(), B, H, qq.shape[2], d, d, vla.VLA_F32,
                                 **dict(opt, u=uu.data_ptr(), zkey0=z2.data_ptr(), zkey_T=z2.data_ptr(),
                                        step_offset=off))
        assert rc == 0
        off += qq.shape[2]
        outs.append(oo)
    torch.cuda.synchronize()
    rel = lambda a, b: float((a - b).abs().max() / b.abs().max())
    assert rel(torch.cat(outs, dim=2), want[0]) < 1e-4
    assert rel(S2, want[1]) < 1e-4 and rel(A2, want[2]) < 1e-4 and rel(z2, want[3]) < 1e-5


@pytest.mark.parametrize("d,B,H", [(32, 5, 210), (64, 3, 100)])
def test_feature_map_with_many_small_heads(d, B, H):
    """The block kernel that shares a workgroup between several heads carries the feature map too."""
    q, k, v = vla_inputs.gaussian_qkv(B, H, 27, d, seed=4000 + d)
    got, ref = run_both(q, k, v, lambda0=0.1, feature_map=True, mode=BLOCK)
    errs = dict(o=slab_rel_err(got["o"], ref["o"], 2), S=slab_rel_err(got["S_T"], ref["S_T"], 2),
                A=slab_rel_err(got["A_T"], ref["A_T"], 2))
    print(d, B * H, errs)
    assert max(errs.values()) <= 1e-4, errs


# ---------------------------------------------------------------- the options inside the segment modes
TWO_PHASE, TIME_PARALLEL = 3, 4
SEGMENT_OPTION_SETS = {k: v for k, v in OPTION_SETS.items() if "refresh_period" not in v}
SEGMENT_OPTION_SETS["paper_head"] = dict(with_u=True, u_scale=0.125, normalise_output=True, feature_map=True)


@pytest.mark.parametrize("name", list(SEGMENT_OPTION_SETS))
@pytest.mark.parametrize("d,T,segments,dtype", [(64, 330, 5, "f32"), (32, 200, 13, "f32"), (128, 150, 3, "f32"),
                                                (64, 1000, 0, "bf16"), (128, 97, 2, "bf16"), (96, 210, 4, "f32"),
                                                (96, 90, 3, "bf16")])
def test_options_in_the_two_phase_and_time_parallel_modes(name, d, T, segments, dtype):
    """A separate penalty direction (the Gram sums at the segment boundaries are then over u, eq. (penalty)), the
    normalised read-out (every segment starts from the prefix sum of the keys before it, eq. (output)) and the
    feature map, in both segment modes, ragged last blocks and short last segments included."""
    cfg = dict(SEGMENT_OPTION_SETS[name])
    rng = np.random.default_rng(300 + d + T)
    q, k, v = vla_inputs.gaussian_qkv(2, 3, T, d, seed=1700 + d + T)
    if cfg.pop("positive", False):
        q, k = np.abs(q) + 0.05, np.abs(k) + 0.05
    u = rng.standard_normal(q.shape).astype(np.float32) if cfg.pop("with_u", False) else None
    cfg.pop("want_zkey_only", None)
    for mode in (TWO_PHASE, TIME_PARALLEL):
        got, ref = run_both(q, k, v, dtype=dtype, u=u, lambda0=0.1, mode=mode,
                            segments=segments if mode == TIME_PARALLEL else None, **cfg)
        print(name, d, T, dtype, mode, assert_close(got, ref, TOL[dtype]))


@pytest.mark.parametrize("d", [32, 64, 96, 128])
def test_time_parallel_with_options_carries_state_between_calls(d):
    """[0,T1) then [T1,T) in the time-parallel mode with S, A and the key sum carried == one oracle run; the
    second call starts from a non-trivial A0 (inverted in float64 at the boundaries), S0 and key sum."""
    T, T1 = 500, 212
    rng = np.random.default_rng(8 + d)
    q, k, v = vla_inputs.gaussian_qkv(1, 4, T, d, seed=91 + d)
    u = rng.standard_normal(q.shape).astype(np.float32)
    opt = dict(lambda0=0.1, u_scale=d ** -0.5, normalise_output=True, feature_map=True, mode=TIME_PARALLEL)
    ref = oracle.forward(q, k, v, u=u, lambda0=0.1, u_scale=d ** -0.5, normalise_output=True, feature_map=True)
    a, _ = run_both(q[:, :, :T1], k[:, :, :T1], v[:, :, :T1], u=u[:, :, :T1], segments=4, **opt)
    b, _ = run_both(q[:, :, T1:], k[:, :, T1:], v[:, :, T1:], u=u[:, :, T1:], S0=a["S_T"], A0=a["A_T"],
                    zkey0=a["zkey_T"], segments=6, **opt)
    joined = dict(o=np.concatenate([a["o"], b["o"]], axis=2), S_T=b["S_T"], A_T=b["A_T"], zkey_T=b["zkey_T"])
    print(d, assert_close(joined, ref, 1e-4))


@pytest.mark.parametrize("d,T,segments", [(64, 250, 8), (32, 300, 8), (128, 150, 8)])
def test_options_with_many_head_segment_pairs(d, T, segments):
    """256 (head, segment) pairs: the S recurrence runs in the kernels that share a block's operands through
    LDS, which carry the read-out denominators as well."""
    rng = np.random.default_rng(d)
    q, k, v = vla_inputs.gaussian_qkv(4, 8, T, d, seed=2200 + d)
    u = rng.standard_normal(q.shape).astype(np.float32)
    z0 = np.abs(rng.standard_normal((4, 8, d))).astype(np.float32)
    for dtype in ("f32", "bf16"):
        got, ref = run_both(q, k, v, dtype=dtype, u=u, zkey0=z0, lambda0=0.1, u_scale=0.25, normalise_output=True,
                            feature_map=True, mode=TIME_PARALLEL, segments=segments)
        print(d, dtype, assert_close(got, ref, TOL[dtype]))


def test_auto_sends_a_few_head_call_with_the_papers_options_to_the_time_parallel_mode():
    import paper_2605_11196_amd as vla

    assert vla.resolve_mode(1, 16, 131072, 64, 64, vla.VLA_BF16, u=0x10000, normalise_output=1,
                            feature_map=1) == vla.MODE_TIME_PARALLEL
    d, T = 32, 4096
    rng = np.random.default_rng(3)
    q, k, v = vla_inputs.gaussian_qkv(1, 4, T, d, seed=31)
    u = rng.standard_normal(q.shape).astype(np.float32)
    got, ref = run_both(q, k, v, dtype="bf16", u=u, lambda0=0.1, u_scale=d ** -0.5, normalise_output=True,
                        feature_map=True)       # mode AUTO
    print(assert_close(got, ref, TOL["bf16"]))
