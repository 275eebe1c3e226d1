"""vla_forward_static: the entry point that allocates nothing (the library's static array is its workspace).

Checked against vla_forward on the same inputs and mode: the two run the same kernels, so the results are
compared at the usual parity bar against each other (and are in fact bit-identical), on two calls in a row, the
second with a smaller input -- the array then still holds the first call's records."""
import numpy as np
import pytest

import vla_inputs

pytestmark = pytest.mark.gpu

STATIC_BYTES = 64 << 20


def _both(q, k, v, mode, lambda0=0.1, segments=None):
    import torch

    import paper_2605_11196_amd as vla

    B, H, T, d = q.shape
    io = vla.VLA_F32 if q.dtype == torch.float32 else vla.VLA_BF16
    dev = q.device
    st = torch.cuda.current_stream().cuda_stream
    need = vla.vla_forward_workspace_bytes(B, H, T, d, d, io, mode=mode, segments=segments)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
    outs = []
    for static in (False, True):
        o = torch.full_like(v, float("nan"))
        S_T = torch.full((B, H, d, d), float("nan"), device=dev)
        A_T = torch.full((B, H, d, d), float("nan"), device=dev)
        if static:
            rc = vla.vla_forward_static_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), 0, 0, o.data_ptr(),
                                            S_T.data_ptr(), A_T.data_ptr(), B, H, T, d, d, io, lambda0=lambda0,
                                            mode=mode, stream=st, segments=segments)
        else:
            rc = vla.vla_forward_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), 0, 0, o.data_ptr(),
                                     S_T.data_ptr(), A_T.data_ptr(), B, H, T, d, d, io, lambda0=lambda0,
                                     mode=mode, workspace=ws.data_ptr(), workspace_bytes=need, stream=st,
                                     segments=segments)
        assert rc == 0, vla.status_string(rc)
        torch.cuda.synchronize()
        outs.append((o, S_T, A_T))
    return need, outs


@pytest.mark.parametrize("mode", [4, 3, 0])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_static_workspace_matches_caller_workspace_twice_in_a_row(mode, dtype):
    import torch

    from parity_utils import TOL, slab_rel_err, to_np

    dev = torch.device("cuda:0")
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    # first a larger input, then a smaller one (other head count, length and segment count): the array still
    # holds what the first call left there
    for (B, H, T, d, segments) in ((2, 4, 1500, 64, 5), (1, 3, 333, 64, 3)):
        q, k, v = (torch.from_numpy(x).to(dev).to(tdt)
                   for x in vla_inputs.gaussian_qkv(B, H, T, d, seed=900 + T))
        need, (ref, got) = _both(q, k, v, mode, segments=segments if mode == 4 else None)
        assert mode == 0 or 0 < need <= STATIC_BYTES
        for name, a, b in zip(("o", "S_T", "A_T"), ref, got):
            assert torch.isfinite(b.float()).all(), name
            err = slab_rel_err(to_np(b), to_np(a), 2)
            assert err <= TOL[dtype], (name, err)
            assert torch.equal(a, b), name      # same kernels on the same records: not one bit differs


def test_static_workspace_serves_auto_and_the_modes_that_need_none():
    import torch

    import paper_2605_11196_amd as vla

    dev = torch.device("cuda:0")
    # few heads on a long enough sequence: AUTO resolves to the time-parallel mode and uses the array
    q, k, v = (torch.from_numpy(x).to(dev) for x in vla_inputs.gaussian_qkv(1, 4, 2048, 32, seed=77))
    assert vla.resolve_mode(1, 4, 2048, 32, 32, vla.VLA_F32) == vla.MODE_TIME_PARALLEL
    _, (ref, got) = _both(q, k, v, 0)
    assert all(torch.equal(a, b) for a, b in zip(ref, got))
    for mode in (vla.MODE_SCAN, vla.MODE_CHUNKED):
        _, (ref, got) = _both(q[:, :, :200].contiguous(), k[:, :, :200].contiguous(),
                              v[:, :, :200].contiguous(), mode)
        assert all(torch.equal(a, b) for a, b in zip(ref, got))


def test_request_beyond_the_static_array_is_refused_or_rerouted():
    import torch

    import paper_2605_11196_amd as vla

    dev = torch.device("cuda:0")
    B, H, T, d = 1, 8, 32768, 64
    assert vla.vla_forward_workspace_bytes(B, H, T, d, d, vla.VLA_BF16, mode=vla.MODE_TWO_PHASE) > STATIC_BYTES
    q, k, v = vla_inputs.device_gaussian(B, H, T, d, 5, 1.0, torch.bfloat16)
    o = torch.empty_like(v)
    st = torch.cuda.current_stream().cuda_stream
    for mode in (vla.MODE_TWO_PHASE, vla.MODE_TIME_PARALLEL):
        rc = vla.vla_forward_static_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), 0, 0, o.data_ptr(), 0, 0,
                                        B, H, T, d, d, vla.VLA_BF16, mode=mode, stream=st)
        assert vla.status_string(rc) == "VLA_ERR_WORKSPACE"
    # AUTO falls back to the fused block kernel, as vla_forward does without a workspace
    ref = torch.empty_like(v)
    rc = vla.vla_forward_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), 0, 0, ref.data_ptr(), 0, 0, B, H, T, d, d,
                             vla.VLA_BF16, mode=vla.MODE_CHUNKED, stream=st)
    assert rc == 0
    rc = vla.vla_forward_static_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), 0, 0, o.data_ptr(), 0, 0,
                                    B, H, T, d, d, vla.VLA_BF16, stream=st)
    assert rc == 0
    torch.cuda.synchronize()
    assert torch.equal(o, ref)


@pytest.mark.parametrize("mode", [4, 0])
def test_static_entry_point_records_into_a_graph_and_replays(mode):
    """The callers this entry point is for: under stream capture nothing may allocate.  After one eager call
    (which looks the array up), the call is recorded into a graph; every replay, with other data in the same
    input buffers and eager work in between, must reproduce the eager result bit for bit."""
    import torch

    import paper_2605_11196_amd as vla

    dev = torch.device("cuda:0")
    B, H, T, d, segments = 1, 6, 1100, 64, (4 if mode == 4 else None)
    q, k, v = (torch.from_numpy(x).to(dev).to(torch.bfloat16) for x in vla_inputs.gaussian_qkv(B, H, T, d, seed=31))
    o = torch.empty_like(v)
    S_T = torch.empty((B, H, d, d), device=dev)
    A_T = torch.empty((B, H, d, d), device=dev)

    def call(stream):
        rc = vla.vla_forward_static_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), 0, 0, o.data_ptr(),
                                        S_T.data_ptr(), A_T.data_ptr(), B, H, T, d, d, vla.VLA_BF16, lambda0=0.1,
                                        mode=mode, stream=stream, segments=segments)
        assert rc == 0, vla.status_string(rc)

    call(torch.cuda.current_stream().cuda_stream)     # eager: the first call on a device looks the array up
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call(torch.cuda.current_stream().cuda_stream)
    for rep in range(4):
        fresh = [torch.from_numpy(x).to(dev).to(torch.bfloat16)
                 for x in vla_inputs.gaussian_qkv(B, H, T, d, seed=40 + rep)]
        for dst, src in zip((q, k, v), fresh):
            dst.copy_(src)
        call(torch.cuda.current_stream().cuda_stream)  # eager reference on the same buffers
        torch.cuda.synchronize()
        want = (o.clone(), S_T.clone(), A_T.clone())
        for t in (o, S_T, A_T):
            t.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        for name, a, b in zip(("o", "S_T", "A_T"), want, (o, S_T, A_T)):
            assert torch.equal(a, b), (name, rep)
