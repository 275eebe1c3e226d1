"""The C ABI from plain C: tests/c_abi_client.c (gcc, include/vla.h, the HIP runtime's C interface; no Python
or PyTorch in the process) runs vla_forward on seeded inputs handed over as raw files; the result is compared
with the fp64 oracle to the same tolerances as the other parity tests."""
import os
import subprocess

import numpy as np
import pytest

import oracle
import vla_inputs
from parity_utils import TOL, slab_rel_err

pytestmark = pytest.mark.gpu

CLIENT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_abi_client")


@pytest.mark.parametrize("B,H,T,d,dtype,mode", [
    (2, 3, 77, 64, "f32", 0),        # AUTO -> block kernel
    (1, 2, 1500, 64, "f32", 0),      # AUTO -> time-parallel, workspace sized by the query call
    (2, 2, 100, 128, "bf16", 2),
    (1, 2, 300, 32, "bf16", 3),
    (2, 2, 50, 96, "f32", 1),
])
def test_plain_c_client_matches_the_oracle(tmp_path, B, H, T, d, dtype, mode):
    if not os.path.exists(CLIENT):   # normally built by __graft_entry__.build(); a 0.2 s gcc run otherwise
        import c_abi_build

        c_abi_build.build()
    q, k, v = vla_inputs.gaussian_qkv(B, H, T, d, seed=1000 + d + T)
    if dtype == "bf16":
        q, k, v = (vla_inputs.round_to_bf16(x) for x in (q, k, v))
        raw = lambda x: (x.astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)   # exact: already rounded
    else:
        raw = lambda x: x.astype(np.float32)
    fin, fout = tmp_path / "in.bin", tmp_path / "out.bin"
    with open(fin, "wb") as f:
        for x in (q, k, v):
            f.write(np.ascontiguousarray(raw(x)).tobytes())
    run = subprocess.run([CLIENT, str(fin), str(fout), str(B), str(H), str(T), str(d),
                          "1" if dtype == "bf16" else "0", str(mode)], capture_output=True, text=True, timeout=100)
    print(run.stdout, run.stderr)
    assert run.returncode == 0
    blob = open(fout, "rb").read()
    n_io, n_state = B * H * T * d, B * H * d * d
    if dtype == "bf16":
        o = (np.frombuffer(blob, dtype=np.uint16, count=n_io).astype(np.uint32) << 16).view(np.float32)
        off = 2 * n_io
    else:
        o = np.frombuffer(blob, dtype=np.float32, count=n_io)
        off = 4 * n_io
    S_T = np.frombuffer(blob, dtype=np.float32, count=n_state, offset=off)
    A_T = np.frombuffer(blob, dtype=np.float32, count=n_state, offset=off + 4 * n_state)
    ref = oracle.forward(q, k, v, lambda0=0.1)
    errs = dict(o=slab_rel_err(o.reshape(B, H, T, d).astype(np.float64), ref["o"], 2),
                S=slab_rel_err(S_T.reshape(B, H, d, d).astype(np.float64), ref["S_T"], 2),
                A=slab_rel_err(A_T.reshape(B, H, d, d).astype(np.float64), ref["A_T"], 2))
    print(errs)
    assert max(errs.values()) <= TOL[dtype], errs
