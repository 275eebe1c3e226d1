"""GPU parity of the decode entry point: one token per call on a state updated in place, against the fp64
oracle run over the same tokens as one sequence (the state carried from call to call is the whole memory)."""
import numpy as np
import pytest

import oracle
import vla_inputs
from parity_utils import TOL, slab_rel_err, to_np

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("d", [16, 32, 64, 96, 128])
def test_decode_steps_follow_the_sequence_oracle(d, dtype):
    import torch

    import paper_2605_11196_amd as vla

    B, H, steps = 2, 3, 24
    q, k, v = vla_inputs.gaussian_qkv(B, H, steps, d, seed=4000 + d)
    if dtype == "bf16":
        q, k, v = (vla_inputs.round_to_bf16(x) for x in (q, k, v))
    ref = oracle.forward(q, k, v, lambda0=0.1)
    dev = torch.device("cuda:0")
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    tq, tk, tv = (torch.from_numpy(x).to(dev).to(tdt) for x in (q, k, v))
    S = torch.zeros(B, H, d, d, device=dev)
    A = (torch.eye(d, device=dev) * (1.0 / np.float32(0.1))).repeat(B, H, 1, 1).contiguous()
    outs = []
    for t in range(steps):
        outs.append(vla.vla_decode_step(tq[:, :, t].contiguous(), tk[:, :, t].contiguous(),
                                        tv[:, :, t].contiguous(), S, A))
    torch.cuda.synchronize()
    o = to_np(torch.stack(outs, dim=2))
    errs = dict(o=slab_rel_err(o, ref["o"], 2), S=slab_rel_err(to_np(S), ref["S_T"], 2),
                A=slab_rel_err(to_np(A), ref["A_T"], 2))
    assert max(errs.values()) <= TOL[dtype], errs


def test_decode_step_continues_a_prefill_and_matches_forward_with_one_token():
    """Prefill with vla_forward, then decode: the same state, the same result as a one-token vla_forward."""
    import torch

    import paper_2605_11196_amd as vla

    d, T = 128, 300
    q, k, v = vla_inputs.gaussian_qkv(2, 2, T + 1, d, seed=77)
    dev = torch.device("cuda:0")
    tq, tk, tv = (torch.from_numpy(x).to(dev) for x in (q, k, v))
    _, S, A = vla.vla_forward(tq[:, :, :T].contiguous(), tk[:, :, :T].contiguous(), tv[:, :, :T].contiguous())
    last = [x[:, :, T:].contiguous() for x in (tq, tk, tv)]
    o1, S1, A1 = vla.vla_forward(*last, S, A, mode=vla.MODE_SCAN)
    o2 = vla.vla_decode_step(*(x[:, :, 0].contiguous() for x in last), S, A)   # S, A updated in place
    torch.cuda.synchronize()
    ref = oracle.forward(q, k, v, lambda0=0.1)
    assert slab_rel_err(to_np(o2)[:, :, None], ref["o"][:, :, T:], 2) <= TOL["f32"]
    assert slab_rel_err(to_np(S), ref["S_T"], 2) <= TOL["f32"] and slab_rel_err(to_np(A), ref["A_T"], 2) <= TOL["f32"]
    assert slab_rel_err(to_np(o2), to_np(o1[:, :, 0]), 1) <= 1e-5
    assert slab_rel_err(to_np(S), to_np(S1), 2) <= 1e-5 and slab_rel_err(to_np(A), to_np(A1), 2) <= 1e-5


def test_decode_step_degenerate_tokens():
    """A zero key writes nothing (S, A unchanged bit for bit) and still reads; a key below eps is clamped."""
    import torch

    import paper_2605_11196_amd as vla

    d = 64
    rng = np.random.default_rng(5)
    dev = torch.device("cuda:0")
    S0 = rng.standard_normal((1, 2, d, d)).astype(np.float32)
    X = rng.standard_normal((1, 2, d, 3 * d))
    A0 = np.linalg.inv(0.1 * np.eye(d) + X @ X.transpose(0, 1, 3, 2) / d).astype(np.float32)
    A0 = 0.5 * (A0 + A0.transpose(0, 1, 3, 2))
    q = rng.standard_normal((1, 2, 1, d)).astype(np.float32)
    v = rng.standard_normal((1, 2, 1, d)).astype(np.float32)
    k = np.zeros((1, 2, 1, d), np.float32)
    k[0, 1, 0, :] = 1e-6 * rng.standard_normal(d)       # head 1: norm far below eps = 1e-4
    ref = oracle.forward(q, k, v, S0, A0)
    S, A = torch.from_numpy(S0.copy()).to(dev), torch.from_numpy(A0.copy()).to(dev)
    o = vla.vla_decode_step(*(torch.from_numpy(x[:, :, 0].copy()).to(dev) for x in (q, k, v)), S, A)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(S)[0, 0], S0[0, 0]) and np.array_equal(to_np(A)[0, 0], A0[0, 0])
    assert slab_rel_err(to_np(o)[:, :, None], ref["o"], 2) <= TOL["f32"]
    assert slab_rel_err(to_np(S), ref["S_T"], 2) <= TOL["f32"] and slab_rel_err(to_np(A), ref["A_T"], 2) <= TOL["f32"]


OPTION_SETS = {
    "u_scaled": dict(u=True, u_scale="rsqrt_d"),
    "refresh": dict(refresh_period=5, refresh_eta=1e-3),
    "normalised_elu": dict(normalise_output=1, feature_map=1),
    "algorithm1": dict(u=True, u_scale="rsqrt_d", refresh_period=4, refresh_eta=1e-3, normalise_output=1,
                       feature_map=1),
}


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("name", sorted(OPTION_SETS))
@pytest.mark.parametrize("d", [16, 64, 96, 128])
def test_decode_steps_with_the_optional_lines_of_algorithm_1(d, name, dtype):
    """A chain of decode calls with options (refresh phase and key sum carried from call to call) against the
    oracle run over the same tokens as one sequence with the same options."""
    import torch

    import paper_2605_11196_amd as vla

    B, H, steps = 2, 2, 17
    opt = dict(OPTION_SETS[name])
    q, k, v = vla_inputs.gaussian_qkv(B, H, steps, d, seed=5000 + d)
    u = np.random.default_rng(d).standard_normal((B, H, steps, d)).astype(np.float32) if opt.pop("u", False) else None
    if opt.get("u_scale") == "rsqrt_d":
        opt["u_scale"] = d ** -0.5
    if dtype == "bf16":
        q, k, v = (vla_inputs.round_to_bf16(x) for x in (q, k, v))
        u = None if u is None else vla_inputs.round_to_bf16(u)
    ref = oracle.forward(q, k, v, lambda0=0.1, u=u, **opt)
    dev = torch.device("cuda:0")
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    tq, tk, tv = (torch.from_numpy(x).to(dev).to(tdt) for x in (q, k, v))
    tu = None if u is None else torch.from_numpy(u).to(dev).to(tdt)
    S = torch.zeros(B, H, d, d, device=dev)
    A = (torch.eye(d, device=dev) * (1.0 / np.float32(0.1))).repeat(B, H, 1, 1).contiguous()
    zkey = torch.zeros(B, H, d, device=dev) if opt.get("normalise_output") else None
    outs = []
    for t in range(steps):
        outs.append(vla.vla_decode_step(tq[:, :, t].contiguous(), tk[:, :, t].contiguous(),
                                        tv[:, :, t].contiguous(), S, A, step_offset=t, zkey=zkey,
                                        u=None if tu is None else tu[:, :, t].contiguous(), **opt))
    torch.cuda.synchronize()
    o = to_np(torch.stack(outs, dim=2))
    errs = dict(o=slab_rel_err(o, ref["o"], 2), S=slab_rel_err(to_np(S), ref["S_T"], 2),
                A=slab_rel_err(to_np(A), ref["A_T"], 2))
    if zkey is not None:
        errs["zkey"] = slab_rel_err(to_np(zkey), ref["zkey_T"], 1)
    assert max(errs.values()) <= TOL[dtype], errs


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("dk,dv", [(dk, dv) for dk in (16, 32, 64, 96, 128) for dv in (16, 32, 64, 96, 128) if dk != dv])
def test_decode_steps_with_value_heads_of_another_size(dk, dv, dtype):
    """d_k != d_v in the decode step: S is d_v x d_k, A is d_k x d_k."""
    import torch

    import paper_2605_11196_amd as vla

    B, H, steps = 2, 3, 20
    rng = np.random.default_rng(dk * 7 + dv)
    q, k = (rng.standard_normal((B, H, steps, dk)).astype(np.float32) for _ in range(2))
    v = rng.standard_normal((B, H, steps, dv)).astype(np.float32)
    S0 = rng.standard_normal((B, H, dv, dk)).astype(np.float32)
    if dtype == "bf16":
        q, k, v = (vla_inputs.round_to_bf16(x) for x in (q, k, v))
    ref = oracle.forward(q, k, v, S0, None, lambda0=0.1)
    dev = torch.device("cuda:0")
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    tq, tk, tv = (torch.from_numpy(x).to(dev).to(tdt) for x in (q, k, v))
    S = torch.from_numpy(S0).to(dev)
    A = (torch.eye(dk, device=dev) * (1.0 / np.float32(0.1))).repeat(B, H, 1, 1).contiguous()
    outs = []
    for t in range(steps):
        outs.append(vla.vla_decode_step(tq[:, :, t].contiguous(), tk[:, :, t].contiguous(),
                                        tv[:, :, t].contiguous(), S, A))
    torch.cuda.synchronize()
    o = to_np(torch.stack(outs, dim=2))
    assert o.shape == (B, H, steps, dv)
    errs = dict(o=slab_rel_err(o, ref["o"], 2), S=slab_rel_err(to_np(S), ref["S_T"], 2),
                A=slab_rel_err(to_np(A), ref["A_T"], 2))
    assert max(errs.values()) <= TOL[dtype], errs


@pytest.mark.parametrize("name", sorted(OPTION_SETS))
@pytest.mark.parametrize("dk,dv", [(dk, dv) for dk in (16, 32, 64, 96, 128) for dv in (16, 32, 64, 96, 128) if dk != dv])
def test_decode_steps_with_options_and_value_heads_of_another_size(dk, dv, name):
    """The optional lines of Algorithm 1 in the decode step with d_k != d_v (refresh phase and key sum carried
    from call to call), against the oracle run over the same tokens as one sequence."""
    import torch

    import paper_2605_11196_amd as vla

    B, H, steps = 1, 3, 13
    opt = dict(OPTION_SETS[name])
    rng = np.random.default_rng(dk * 11 + dv)
    q, k = (rng.standard_normal((B, H, steps, dk)).astype(np.float32) for _ in range(2))
    v = rng.standard_normal((B, H, steps, dv)).astype(np.float32)
    u = rng.standard_normal((B, H, steps, dk)).astype(np.float32) if opt.pop("u", False) else None
    if opt.get("u_scale") == "rsqrt_d":
        opt["u_scale"] = dk ** -0.5
    S0 = rng.standard_normal((B, H, dv, dk)).astype(np.float32)
    ref = oracle.forward(q, k, v, S0, None, lambda0=0.1, u=u, **opt)
    dev = torch.device("cuda:0")
    tq, tk, tv = (torch.from_numpy(x).to(dev) for x in (q, k, v))
    tu = None if u is None else torch.from_numpy(u).to(dev)
    S = torch.from_numpy(S0).to(dev)
    A = (torch.eye(dk, device=dev) * (1.0 / np.float32(0.1))).repeat(B, H, 1, 1).contiguous()
    zkey = torch.zeros(B, H, dk, device=dev) if opt.get("normalise_output") else None
    outs = []
    for t in range(steps):
        outs.append(vla.vla_decode_step(tq[:, :, t].contiguous(), tk[:, :, t].contiguous(),
                                        tv[:, :, t].contiguous(), S, A, step_offset=t, zkey=zkey,
                                        u=None if tu is None else tu[:, :, t].contiguous(), **opt))
    torch.cuda.synchronize()
    o = to_np(torch.stack(outs, dim=2))
    assert o.shape == (B, H, steps, dv)
    errs = dict(o=slab_rel_err(o, ref["o"], 2), S=slab_rel_err(to_np(S), ref["S_T"], 2),
                A=slab_rel_err(to_np(A), ref["A_T"], 2))
    if zkey is not None:
        errs["zkey"] = slab_rel_err(to_np(zkey), ref["zkey_T"], 1)
    assert max(errs.values()) <= TOL["f32"], errs
