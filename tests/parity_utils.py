"""Helpers shared by the GPU parity tests: error metric and the oracle/GPU call pair."""
import numpy as np

import oracle
import vla_inputs

TOL = {"f32": 1e-4, "bf16": 2e-2}   # max relative error bound per I/O type


def slab_rel_err(got, ref, slab_ndim):
    """max over slabs of ||got-ref||_inf / ||ref||_inf, a slab being the trailing `slab_ndim` axes
    (one (b,h) output sequence, or one state matrix)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    axes = tuple(range(got.ndim - slab_ndim, got.ndim))
    num = np.abs(got - ref).max(axis=axes) if got.size else np.zeros(got.shape[:-slab_ndim])
    den = np.abs(ref).max(axis=axes) if ref.size else np.ones(ref.shape[:-slab_ndim])
    den = np.where(den > 0, den, 1.0)
    out = num / den
    return float(out.max()) if out.size else 0.0


def to_np(t):
    import torch

    if t.dtype == torch.bfloat16:
        return t.detach().float().cpu().numpy()
    return t.detach().cpu().numpy()


def gpu_forward(q, k, v, S0=None, A0=None, *, dtype="f32", lambda0=0.1, eps=1e-4, mode=None,
                segments=None):
    """numpy float32 inputs -> GPU call through the C ABI -> numpy outputs (o widened to f32)."""
    import torch

    import paper_2605_11196_amd as vla

    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    dev = torch.device("cuda:0")
    tq, tk, tv = (torch.from_numpy(np.ascontiguousarray(x)).to(dev).to(tdt) for x in (q, k, v))
    tS0 = None if S0 is None else torch.from_numpy(np.ascontiguousarray(S0, dtype=np.float32)).to(dev)
    tA0 = None if A0 is None else torch.from_numpy(np.ascontiguousarray(A0, dtype=np.float32)).to(dev)
    o, S_T, A_T = vla.vla_forward(tq, tk, tv, tS0, tA0, lambda0=lambda0, eps=eps, mode=mode,
                                  segments=segments)
    torch.cuda.synchronize()
    return to_np(o), to_np(S_T), to_np(A_T)


def oracle_inputs(q, k, v, dtype):
    """What the oracle should see: the bf16-rounded values when the GPU gets bf16 tensors."""
    if dtype == "bf16":
        return tuple(vla_inputs.round_to_bf16(x) for x in (q, k, v))
    return q, k, v


def check_parity(q, k, v, S0=None, A0=None, *, dtype="f32", lambda0=0.1, eps=1e-4, mode=None,
                 tol=None, segments=None):
    """Run both sides on the same inputs and assert the three outputs are within tolerance."""
    tol = TOL[dtype] if tol is None else tol
    qo, ko, vo = oracle_inputs(q, k, v, dtype)
    ref = oracle.forward(qo, ko, vo, S0, A0, lambda0=lambda0, eps=eps)
    o, S_T, A_T = gpu_forward(qo, ko, vo, S0, A0, dtype=dtype, lambda0=lambda0, eps=eps, mode=mode,
                              segments=segments)
    errs = dict(o=slab_rel_err(o, ref["o"], 2), S=slab_rel_err(S_T, ref["S_T"], 2),
                A=slab_rel_err(A_T, ref["A_T"], 2))
    assert np.isfinite(o).all() and np.isfinite(S_T).all() and np.isfinite(A_T).all()
    assert errs["o"] <= tol and errs["S"] <= tol and errs["A"] <= tol, errs
    return errs, ref, (o, S_T, A_T)
