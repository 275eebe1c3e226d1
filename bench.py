#!/usr/bin/env python3
"""Benchmark of the VLA forward hot path on one MI355X.

A "step" is one vla_forward call (the whole per-head recurrence: key normalisation,
Sherman-Morrison update of A, write direction, residual update of S, read-out) over one
batch of synthetic input already resident in HBM.  Default workload: the large-batch
configuration (B=64, H=32, T=8192, d_h=128, bf16 q/k/v/o, float32 A and S).

Prints ONE JSON line: whole-job head-tokens/s, the roofline object for the dominant
kernel (HIP-event timed on the launch stream) and the fp64 oracle timed on the host
cores on a bounded sample of the same workload (a reported baseline, not a target).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_TFLOPS = 157.3   # MI355X FP32 vector (and FP32 matrix) peak, TFLOP/s
PEAK_HBM_GBS = 8000.0

# HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE, each scaled by the
# same counter's reading for a plain copy kernel of known size); see profiles/. None = not measured.
MEASURED_TRAFFIC_BYTES = {
    # (B, H, T, d_h, io dtype, resolved mode): bytes per launch --
    # profiles/chunk_kernel_large_batch_hbm_traffic.txt
    (64, 32, 8192, 128, "bf16", 2): 17044037 * 1024,
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="large_batch",
                    choices=["tiny", "norm_growth", "recall", "long_context", "large_batch"])
    ap.add_argument("--T", type=int, default=None, help="sequence length override (long_context)")
    ap.add_argument("--B", type=int, default=None, help="batch override (experiments only)")
    ap.add_argument("--d", type=int, default=None, help="head size override (experiments only)")
    ap.add_argument("--mode", type=int, default=0, help="vla_mode (0 = auto)")
    ap.add_argument("--segments", type=int, default=None,
                    help="time segments for the time-parallel mode (default: the library chooses)")
    ap.add_argument("--decode", action="store_true",
                    help="time vla_decode_step (one token for every head of the workload, state in place) "
                         "instead of vla_forward; the roofline is then the HBM one")
    ap.add_argument("--options", default="none", choices=["none", "paper"],
                    help="'paper': switch on every optional line of Algorithm 1 (separate penalty directions u "
                         "with u_scale = 1/sqrt(d_h), identity refresh every 20 steps, normalised read-out, "
                         "ELU+1 features); the flop count per head-token is then 12 d^2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 1 GiB -> 1 GiB elementwise copy kernel (calibration of the "
                         "FETCH_SIZE / WRITE_SIZE counters under rocprofv3 --pmc)")
    ap.add_argument("--cpu-heads", type=int, default=None, help="heads in the oracle timing sample")
    return ap.parse_args()


def decode_main(args):
    """One decode step per timed step: every head of the workload advances by one token on its resident state.
    Algorithmic traffic per head-token: S and A read and written (4 d^2 float32) + q, k, v read and o written."""
    import torch

    import paper_2605_11196_amd as vla
    import vla_inputs

    c = dict(vla_inputs.CONFIGS[args.workload])
    B, H, d = args.B or c["B"], c["H"], args.d or c["d"]
    dtype = c["dtype"]
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    io = vla.VLA_BF16 if dtype == "bf16" else vla.VLA_F32
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(c["seed"])
    n_tok = args.warmup + args.steps
    q, k, v = ((torch.randn(n_tok, B, H, d, device=dev, generator=gen) * d ** -0.5).to(tdt) for _ in range(3))
    S = torch.zeros(B, H, d, d, device=dev)
    A = (torch.eye(d, device=dev) / c["lambda0"]).repeat(B, H, 1, 1).contiguous()
    o = torch.empty(B, H, d, dtype=tdt, device=dev)
    stream = torch.cuda.current_stream(dev)

    def step(t):
        rc = vla.vla_decode_step_raw(q[t].data_ptr(), k[t].data_ptr(), v[t].data_ptr(), S.data_ptr(),
                                     A.data_ptr(), o.data_ptr(), B, H, d, d, io, stream=stream.cuda_stream)
        if rc != 0:
            raise RuntimeError(vla.status_string(rc))

    for t in range(args.warmup):
        step(t)
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i, (a, b) in enumerate(ev):
        a.record(stream)
        step(args.warmup + i)
        b.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    avg_launch_s = sum(a.elapsed_time(b) for a, b in ev) / len(ev) / 1e3
    heads = B * H
    nbytes = heads * (4 * d * d * 4 + 4 * d * (2 if dtype == "bf16" else 4))
    gbps = nbytes / avg_launch_s / 1e9
    print(json.dumps({
        "metric": "VLA decode step tokens/sec (B*H/s)", "value": heads * args.steps / wall,
        "unit": "head-tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"decode: {heads} heads (B={B} H={H}) d_h={d} {dtype} q/k/v/o, fp32 A and S "
                               f"updated in place, one token per step", "io_dtype": dtype},
        "roofline": {"bound": "hbm", "achieved": gbps, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": gbps / PEAK_HBM_GBS, "traffic": None, "kernel_ms": avg_launch_s * 1e3,
                     "algorithmic_bytes_per_launch": nbytes},
    }))


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (heads are independent, so more GPUs "
              "would only split the batch); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.decode:
        decode_main(args)
        return

    import numpy as np
    import torch

    import paper_2605_11196_amd as vla
    import vla_inputs

    c = dict(vla_inputs.CONFIGS[args.workload])
    if args.workload == "long_context":
        c["T"] = args.T or 131072
    elif args.T:
        c["T"] = args.T
    if args.B:
        c["B"] = args.B
    if args.d:
        c["d"] = args.d
        if "std" in c and args.workload == "large_batch":
            c["std"] = args.d ** -0.5
    B, H, T, d = c["B"], c["H"], c["T"], c["d"]
    dtype = c["dtype"]
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    io = vla.VLA_BF16 if dtype == "bf16" else vla.VLA_F32
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.workload == "recall":
        qn, kn, vn, _ = vla_inputs.recall_task(B, H, T, d, c["seed"], c["n_pairs"])
        q, k, v = (torch.from_numpy(x).to(dev) for x in (qn, kn, vn))
    elif dtype == "bf16":
        q, k, v = vla_inputs.device_gaussian(B, H, T, d, c["seed"], c["std"], tdt)
    else:
        q, k, v = (torch.from_numpy(x).to(dev)
                   for x in vla_inputs.gaussian_qkv(B, H, T, d, c["seed"], c["std"]))

    extra = {}
    if args.options == "paper":
        gen_u = torch.Generator(device=dev)
        gen_u.manual_seed(c["seed"] + 1000)
        u = torch.randn(B, H, T, d, device=dev, generator=gen_u).to(tdt)
        extra = dict(u=u.data_ptr(), u_scale=d ** -0.5, refresh_period=20, refresh_eta=1e-3,
                     normalise_output=1, feature_map=1)
    o = torch.empty_like(v)
    S_T = torch.empty((B, H, d, d), dtype=torch.float32, device=dev)
    A_T = torch.empty((B, H, d, d), dtype=torch.float32, device=dev)
    mode = args.mode
    need = vla.vla_forward_workspace_bytes(B, H, T, d, d, io, lambda0=c["lambda0"], mode=mode,
                                           segments=args.segments, **extra)
    ws = torch.empty((max(need, 16),), dtype=torch.uint8, device=dev)
    resolved = vla.resolve_mode(B, H, T, d, d, io, mode=mode, **extra)
    stream = torch.cuda.current_stream(dev)

    def step():
        rc = vla.vla_forward_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), 0, 0, o.data_ptr(),
                                 S_T.data_ptr(), A_T.data_ptr(), B, H, T, d, d, io,
                                 lambda0=c["lambda0"], mode=mode, workspace=ws.data_ptr(),
                                 workspace_bytes=need, stream=stream.cuda_stream, segments=args.segments,
                                 **extra)
        if rc != 0:
            raise RuntimeError(vla.status_string(rc))

    if args.copy_probe:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)   # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.mul(src, 1.0, out=dst)                                 # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # per-launch device time with HIP events recorded on the launch stream
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a, b in ev:
        a.record(stream)
        step()
        b.record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    wall = t1 - t0
    dev_ms = [a.elapsed_time(b) for a, b in ev]
    avg_launch_s = sum(dev_ms) / len(dev_ms) / 1e3

    head_tokens = B * H * T
    value = head_tokens * args.steps / wall
    # algorithmic flop per launch: 5 d^2 FMA per head-token, 6 d^2 with separate penalty directions
    flops = (12.0 if args.options == "paper" else 10.0) * d * d * head_tokens
    n_streams = 5 if args.options == "paper" else 4                  # q,k,v (and u) read + o written
    io_bytes = (2 if dtype == "bf16" else 4) * n_streams * d * head_tokens
    achieved_tflops = flops / avg_launch_s / 1e12
    mode_names = {1: "scan", 2: "chunked", 3: "two_phase", 4: "time_parallel"}
    workload = (f"{args.workload}: B={B} H={H} T={T} d_h={d} {dtype} q/k/v/o, fp32 A and S, "
                f"lambda0={c['lambda0']}")
    if args.options == "paper":
        workload += ", every option of Algorithm 1 on (u with u_scale=1/sqrt(d_h), refresh 20, normalised, ELU+1)"
    out = {
        "metric": "VLA forward tokens/sec (B*H*T/s)",
        "value": value,
        "unit": "head-tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": workload, "io_dtype": dtype, "kernel_mode": mode_names.get(resolved, str(resolved)),
                   "global_batch": B, "heads": H, "seq_len": T, "d_h": d, "parallelism": "single-gpu"},
        "roofline": {
            "bound": "mfma" if resolved in (2, 3, 4) else "alu",
            "achieved": achieved_tflops,
            "peak": PEAK_FP32_TFLOPS,
            "unit": "TFLOP/s",
            "frac": achieved_tflops / PEAK_FP32_TFLOPS,
            "traffic": MEASURED_TRAFFIC_BYTES.get((B, H, T, d, dtype, resolved)) if args.options == "none" else None,
            "kernel_ms": avg_launch_s * 1e3,
            "algorithmic_flop_per_launch": flops,
            "algorithmic_bytes_per_launch": io_bytes,
            "hbm_GBps": io_bytes / avg_launch_s / 1e9,
            "hbm_frac": io_bytes / avg_launch_s / 1e9 / PEAK_HBM_GBS,
        },
    }

    if not args.no_cpu_baseline:
        import oracle

        # bounded sample: a deterministic subset of heads over the full sequence
        n_all = B * H
        want = args.cpu_heads or max(1, min(n_all, int(3.0e6 * (128.0 / d) ** 2 / max(T, 1))))
        idx = sorted(set(int(i) for i in np.linspace(0, n_all - 1, num=min(want, n_all))))
        sel = torch.tensor(idx, device=dev)
        pick = lambda x: x.reshape(n_all, *x.shape[2:]).index_select(0, sel).float().cpu().numpy()[None]
        qs, ks, vs = (pick(x).astype(np.float64) for x in (q, k, v))
        oracle.load()
        oracle_opt = {}
        if args.options == "paper":
            oracle_opt = dict(u=pick(u).astype(np.float64), u_scale=extra["u_scale"],
                              refresh_period=extra["refresh_period"], refresh_eta=extra["refresh_eta"],
                              normalise_output=True, feature_map=True)
        tc0 = time.perf_counter()
        ref = oracle.forward(qs, ks, vs, lambda0=c["lambda0"], **oracle_opt)
        tc1 = time.perf_counter()
        cpu_rate = len(idx) * T / (tc1 - tc0)
        got = pick(o).astype(np.float64)
        err = float((np.abs(got - ref["o"]).max(axis=(2, 3)) / np.abs(ref["o"]).max(axis=(2, 3))).max())
        out["cpu_baseline"] = {
            "value": cpu_rate, "unit": "head-tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{len(idx)} of {n_all} heads (evenly spaced) x all {T} tokens, fp64, "
                      f"{tc1 - tc0:.1f} s",
            "gpu_vs_oracle_max_rel_err_o": err,
        }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
