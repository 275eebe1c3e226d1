"""GPU parity of the time-parallel mode: segments of the sequence run concurrently from boundary states
(A from the explicit inverse of Section 3.2 in float64, S from composed per-segment affine maps of
eq. (s-update)); the result must match the sequential fp64 oracle to the same tolerance as every other mode.
"""
import numpy as np
import pytest

import oracle
import vla_inputs
from parity_utils import TOL, check_parity, gpu_forward, slab_rel_err

pytestmark = pytest.mark.gpu

TP = 4  # VLA_MODE_TIME_PARALLEL


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("d,T,segments", [
    (64, 1000, 5),      # ragged: 63 blocks in segments of 13, the last one short, last block 8 tokens
    (32, 200, 256),     # more segments asked for than blocks: one block per segment
    (128, 513, 2),      # second segment ends in a one-token block
    (128, 300, 7),
    (96, 700, 6),       # three waves per head, keys staged by 6 threads of 16 elements; Gram sums and the
    (96, 47, 3),        # boundary inverse run in the d = 128 layout with the extra columns held at zero
    (64, 4096, 0),      # the library's own choice (16 segments for 6 heads)
    (32, 2048, 0),
    (64, 16, 4),        # a single block: degenerates to one segment
])
def test_segments_match_the_sequential_oracle(d, T, segments, dtype):
    q, k, v = vla_inputs.gaussian_qkv(2, 3, T, d, seed=900 + d + T)
    errs, _, _ = check_parity(q, k, v, dtype=dtype, lambda0=0.1, mode=TP, segments=segments)
    print(d, T, segments, dtype, errs)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("d,T,segments", [(64, 250, 8), (32, 300, 8), (128, 150, 8), (64, 16 * 9, 9), (96, 200, 8)])
def test_many_head_segment_pairs_take_the_shared_operand_kernels(d, T, segments, dtype):
    """32 heads x 8 segments = 256 (head, segment) pairs: from there on the S recurrence runs with one
    workgroup per pair and the block operands staged once through LDS (ragged last block, one- and
    two-block segments, the three-stage ring wrapping round)."""
    q, k, v = vla_inputs.gaussian_qkv(4, 8, T, d, seed=1200 + d + T)
    S0 = np.random.default_rng(d).standard_normal((4, 8, d, d)).astype(np.float32)
    errs, _, _ = check_parity(q, k, v, S0, None, dtype=dtype, lambda0=0.1, mode=TP, segments=segments)
    print(d, T, segments, dtype, errs)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("d,T,segments", [(64, 300, 8), (32, 277, 8), (64, 16 * 8 + 1, 8), (32, 16 * 16, 8)])
def test_chip_filling_pair_counts_form_the_maps_inside_the_a_scan(d, T, segments, dtype):
    """96 heads x 8 segments = 768 (head, segment) pairs: from there on (d <= 64, no options) the A scan forms the
    per-segment affine maps of S itself, one block behind (two- and three-block segments, a ragged last block, a
    one-token last segment, a given S0 and A0)."""
    q, k, v = vla_inputs.gaussian_qkv(6, 16, T, d, seed=1250 + d + T)
    rng = np.random.default_rng(d + T)
    S0 = rng.standard_normal((6, 16, d, d)).astype(np.float32)
    R = rng.standard_normal((6, 16, d, d)) / np.sqrt(d)
    A0 = (np.eye(d) * 2.0 + R @ np.swapaxes(R, -1, -2)).astype(np.float32)   # symmetric positive definite
    A0 = (A0 + np.swapaxes(A0, -1, -2)) / 2
    errs, _, _ = check_parity(q, k, v, S0, A0, dtype=dtype, lambda0=0.1, mode=TP, segments=segments)
    print(d, T, segments, dtype, errs)


@pytest.mark.parametrize("d,T", [(64, 100), (128, 33), (32, 200), (96, 70)])
def test_two_phase_with_many_heads_takes_the_shared_operand_kernel(d, T):
    q, k, v = vla_inputs.gaussian_qkv(16, 16, T, d, seed=1300 + d)
    check_parity(q, k, v, lambda0=0.1, mode=3)


@pytest.mark.parametrize("d", [32, 64, 96, 128])
def test_given_initial_state_enters_the_boundary_inverse(d):
    """A non-trivial symmetric positive definite A0 and a non-zero S0 (the state after T1 tokens, from
    the oracle) must be carried through the boundary computation: A0 is inverted in float64 there."""
    T, T1 = 700, 123
    q, k, v = vla_inputs.gaussian_qkv(1, 4, T, d, seed=77 + d)
    full = oracle.forward(q, k, v, lambda0=0.1)
    head = oracle.forward(q[:, :, :T1], k[:, :, :T1], v[:, :, :T1], lambda0=0.1)
    o, S_T, A_T = gpu_forward(q[:, :, T1:], k[:, :, T1:], v[:, :, T1:], head["S_T"], head["A_T"],
                              mode=TP, segments=6)
    errs = dict(o=slab_rel_err(o, full["o"][:, :, T1:], 2), S=slab_rel_err(S_T, full["S_T"], 2),
                A=slab_rel_err(A_T, full["A_T"], 2))
    assert max(errs.values()) <= TOL["f32"], errs


def test_recall_workload_with_zero_and_repeated_directions():
    """Mostly all-zero tokens and few distinct keys: the Gram sums are low-rank, so the boundary matrix
    lambda0 I + G has many eigenvalues equal to lambda0."""
    c = vla_inputs.CONFIGS["recall"]
    q, k, v, _ = vla_inputs.recall_task(4, c["H"], c["T"], c["d"], c["seed"], c["n_pairs"])
    check_parity(q, k, v, lambda0=c["lambda0"], mode=TP, segments=8)


def test_result_is_deterministic():
    """Every reduction has a fixed order (Gram partials summed in wave order, no floating-point atomics): two
    calls on the same inputs agree bit for bit, for the per-wave and for the shared-operand S kernels."""
    import torch

    import paper_2605_11196_amd as vla

    dev = torch.device("cuda:0")
    for heads, T, seg in ((3, 777, 5), (64, 333, 4)):
        q, k, v = (torch.from_numpy(x).to(dev) for x in vla_inputs.gaussian_qkv(1, heads, T, 64, seed=T))
        a = vla.vla_forward(q, k, v, mode=TP, segments=seg)
        b = vla.vla_forward(q, k, v, mode=TP, segments=seg)
        torch.cuda.synchronize()
        for x, y in zip(a, b):
            assert torch.equal(x, y)


def test_segment_count_only_changes_rounding():
    d, T = 64, 1536
    q, k, v = vla_inputs.gaussian_qkv(1, 2, T, d, seed=31)
    ref = gpu_forward(q, k, v, mode=3)
    for segments in (2, 3, 16, 96):
        got = gpu_forward(q, k, v, mode=TP, segments=segments)
        for x, y, nd in zip(got, ref, (2, 2, 2)):
            assert slab_rel_err(x, y, nd) <= 2e-5, segments


@pytest.mark.parametrize("heads", [3, 64])
def test_state_outputs_may_alias_inputs_or_be_null(heads):
    """S_T / A_T written over S0 / A0 (the boundary kernels have read them by then) and left out altogether;
    few heads take the per-wave S kernels, 64 heads x 4 segments the shared-operand ones."""
    import torch

    import paper_2605_11196_amd as vla

    d, T, seg = 64, 200, 4
    dev = torch.device("cuda:0")
    q, k, v = (torch.from_numpy(x).to(dev) for x in vla_inputs.gaussian_qkv(1, heads, T, d, seed=400))
    S0 = torch.randn((1, heads, d, d), device=dev)
    A0 = torch.eye(d, device=dev).expand(1, heads, d, d).contiguous() * 2.0
    o_ref, S_ref, A_ref = vla.vla_forward(q, k, v, S0, A0, mode=TP, segments=seg)
    S_al, A_al = S0.clone(), A0.clone()
    o = torch.empty_like(q)
    need = vla.vla_forward_workspace_bytes(1, heads, T, d, d, vla.VLA_F32, mode=TP, segments=seg)
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    st = torch.cuda.current_stream().cuda_stream
    args = (1, heads, T, d, d, vla.VLA_F32)
    kw = dict(mode=TP, segments=seg, workspace=ws.data_ptr(), workspace_bytes=need, stream=st)
    rc = vla.vla_forward_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), S_al.data_ptr(), A_al.data_ptr(),
                             o.data_ptr(), S_al.data_ptr(), A_al.data_ptr(), *args, **kw)
    assert rc == 0
    o2 = torch.empty_like(q)
    rc = vla.vla_forward_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), S0.data_ptr(), A0.data_ptr(),
                             o2.data_ptr(), 0, 0, *args, **kw)
    assert rc == 0
    torch.cuda.synchronize()
    assert torch.equal(o, o_ref) and torch.equal(S_al, S_ref) and torch.equal(A_al, A_ref)
    assert torch.equal(o2, o_ref)
    ref = oracle.forward(q.cpu().numpy(), k.cpu().numpy(), v.cpu().numpy(), S0.cpu().numpy(), A0.cpu().numpy())
    assert slab_rel_err(o.cpu().numpy(), ref["o"], 2) <= TOL["f32"]
    assert slab_rel_err(S_al.cpu().numpy(), ref["S_T"], 2) <= TOL["f32"]
    assert slab_rel_err(A_al.cpu().numpy(), ref["A_T"], 2) <= TOL["f32"]


def test_workspace_and_option_checks():
    import torch

    import paper_2605_11196_amd as vla

    B, H, T, d = 1, 2, 2048, 64
    need_tp = vla.vla_forward_workspace_bytes(B, H, T, d, d, vla.VLA_F32, mode=TP, segments=4)
    need_2p = vla.vla_forward_workspace_bytes(B, H, T, d, d, vla.VLA_F32, mode=vla.MODE_TWO_PHASE)
    assert need_tp > need_2p > 0
    # AUTO for few heads and a long sequence is this mode and asks for its workspace
    assert vla.resolve_mode(B, H, T, d, d, vla.VLA_F32) == TP
    assert vla.vla_forward_workspace_bytes(B, H, T, d, d, vla.VLA_F32) >= need_2p
    dev = torch.device("cuda:0")
    q = torch.randn(B, H, T, d, device=dev)
    o = torch.empty_like(q)
    ws = torch.empty(need_tp, dtype=torch.uint8, device=dev)
    args = (q.data_ptr(), q.data_ptr(), q.data_ptr(), 0, 0, o.data_ptr(), 0, 0, B, H, T, d, d, vla.VLA_F32)
    # too small a workspace for an explicitly requested mode is an error, nothing is launched
    rc = vla.vla_forward_raw(*args, mode=TP, segments=4, workspace=ws.data_ptr(), workspace_bytes=need_tp - 16)
    assert vla.status_string(rc) == "VLA_ERR_WORKSPACE"
    rc = vla.vla_forward_raw(*args, mode=TP, segments=4, workspace=ws.data_ptr(), workspace_bytes=need_tp)
    assert rc == 0
    # the options of Algorithm 1 break A_t = M_t^{-1} (refresh) or u = k^: refused
    rc = vla.vla_forward_raw(*args, mode=TP, segments=4, workspace=ws.data_ptr(), workspace_bytes=need_tp,
                             refresh_period=20)
    assert vla.status_string(rc) == "VLA_ERR_UNSUPPORTED"
    rc = vla.vla_forward_raw(*args, mode=TP, segments=-1, workspace=ws.data_ptr(), workspace_bytes=need_tp)
    assert vla.status_string(rc) == "VLA_ERR_INVALID_ARG"
    torch.cuda.synchronize()


# ------------------------------------------------------------------ value heads of another size than the key heads
SEG_KEY_SIZES = [32, 64, 96, 128]
VALUE_SIZES = [16, 32, 64, 96, 128]
SEG_RECT_PAIRS = [(dk, dv) for dk in SEG_KEY_SIZES for dv in VALUE_SIZES if dk != dv]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("dk,dv", SEG_RECT_PAIRS)
def test_value_heads_of_another_size_run_in_the_segment_modes(dk, dv, dtype):
    """S is d_v x d_k (eq. (s-update), eq. (output)): the A side of the segment modes only sees the keys, the S rows
    kernel shares the d_v / 16 row slabs of S out to its d_k / 16 waves in turn (one to four slots per wave, some
    waves with none), the per-segment maps are P [d_k][d_k] and Q [d_v][d_k].  Four segments of six blocks with a
    ragged last block and a given S0, time-parallel and two-phase."""
    B, H, T = 2, 3, 333
    q, k, v = vla_inputs.gaussian_qkv(B, H, T, dk, seed=1500 + dk + dv, d_v=dv)
    S0 = np.random.default_rng(dk + dv).standard_normal((B, H, dv, dk)).astype(np.float32)
    for mode, segments in ((TP, 4), (3, None)):
        errs, _, _ = check_parity(q, k, v, S0, None, dtype=dtype, lambda0=0.1, mode=mode, segments=segments)
        print(dk, dv, dtype, mode, errs)


@pytest.mark.parametrize("optset", ["normalised read-out", "penalty direction"])
@pytest.mark.parametrize("dk,dv", [(32, 128), (64, 96), (64, 16), (96, 128), (128, 32), (128, 96)])
def test_options_on_value_heads_of_another_size_in_the_time_parallel_mode(dk, dv, optset):
    """The options the segment modes carry (separate penalty directions, normalised read-out with a carried key
    sum, ELU+1) with d_k != d_v: the A chain of the option kernel feeds the same S rows kernel."""
    import torch

    import paper_2605_11196_amd as vla
    from parity_utils import to_np

    B, H, T = 1, 5, 300
    rng = np.random.default_rng(70 + dk + dv)
    q, k, u = (rng.standard_normal((B, H, T, dk)).astype(np.float32) for _ in range(3))
    v = rng.standard_normal((B, H, T, dv)).astype(np.float32)
    S0 = rng.standard_normal((B, H, dv, dk)).astype(np.float32)
    z0 = np.abs(rng.standard_normal((B, H, dk))).astype(np.float32)
    with_u = optset == "penalty direction"
    opt = dict(lambda0=0.1)
    if with_u:
        opt["u_scale"] = dk ** -0.5
    else:
        opt.update(normalise_output=True, feature_map=True)
    norm = bool(opt.get("normalise_output"))
    ref = oracle.forward(q, k, v, S0, None, u=u if with_u else None, zkey0=z0 if norm else None, **opt)
    dev = torch.device("cuda:0")
    t = lambda x: torch.from_numpy(x).to(dev)
    out = vla.vla_forward(t(q), t(k), t(v), t(S0), None, u=t(u) if with_u else None,
                          zkey0=t(z0) if norm else None, return_zkey=norm, mode=TP, segments=3, **opt)
    torch.cuda.synchronize()
    o, S_T, A_T = out[:3]
    errs = dict(o=slab_rel_err(to_np(o), ref["o"], 2), S=slab_rel_err(to_np(S_T), ref["S_T"], 2),
                A=slab_rel_err(to_np(A_T), ref["A_T"], 2))
    if norm:
        errs["z"] = slab_rel_err(to_np(out[3]), ref["zkey_T"], 1)
    print(dk, dv, optset, errs)
    assert max(errs.values()) <= 1e-4, errs
