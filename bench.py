#!/usr/bin/env python3
"""Benchmark of the VLA forward hot path on one MI355X.

A "step" is one vla_forward call (the whole per-head recurrence: key normalisation,
Sherman-Morrison update of A, write direction, residual update of S, read-out) over one
batch of synthetic input already resident in HBM.  Default workload: the large-batch
configuration (B=64, H=32, T=8192, d_h=128, bf16 q/k/v/o, float32 A and S).

Prints ONE JSON line: whole-job head-tokens/s, the roofline object for the dominant
kernel (HIP-event timed on the launch stream) and the fp64 oracle timed on the host
cores on a bounded sample of the same workload (a reported baseline, not a target).
The default run adds a `secondary` array to the same line: the other head size the
metric is quoted at (d_h = 64 at large batch), the long-context sweep (five sequence
lengths at d_h = 64 and one at d_h = 128, the library's own choice of mode), the large-batch workload with every optional
line of Algorithm 1 switched on, and the decode step; each entry is timed the same way
(median of at least 10 launches) and checked against the oracle on a few heads.
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_TFLOPS = 157.3   # MI355X FP32 vector (and FP32 matrix) peak, TFLOP/s
PEAK_HBM_GBS = 8000.0
MODE_NAMES = {1: "scan", 2: "chunked", 3: "two_phase", 4: "time_parallel"}

# HBM bytes per launch read with rocprofv3 --pmc in a separate run (FETCH_SIZE + WRITE_SIZE, each scaled by
# the same counter's reading for a plain copy kernel of known size).  A stored reading of the named profile
# summary, valid for that shape and mode only; every other case reports null.
PROFILED_TRAFFIC_BYTES = {
    # (B, H, T, d_h, io dtype, resolved mode): (bytes per launch, summary)
    (64, 32, 8192, 128, "bf16", 2): (17045169 * 1024, "profiles/chunk_kernel_large_batch_hbm_traffic.txt"),
    (1, 16, 131072, 64, "bf16", 4): (4013682 * 1024, "profiles/time_parallel_long_context_hbm_traffic.txt"),
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
    ap.add_argument("--options", default="none", choices=["none", "paper", "paper_no_refresh"],
                    help="'paper': switch on every optional line of Algorithm 1 (separate penalty directions u "
                         "with u_scale = 1/sqrt(d_h), identity refresh every 20 steps, normalised read-out, "
                         "ELU+1 features); the flop count per head-token is then 12 d^2.  'paper_no_refresh': the "
                         "same without the identity refresh (what the time-parallel mode carries)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-secondary", action="store_true",
                    help="print the headline entry only (the secondary entries belong to the default workload)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 1 GiB -> 1 GiB elementwise copy kernel (calibration of the "
                         "FETCH_SIZE / WRITE_SIZE counters under rocprofv3 --pmc)")
    ap.add_argument("--cpu-heads", type=int, default=None, help="heads in the oracle timing sample")
    return ap.parse_args()


def sig(x, n=5):
    """Round to n significant digits (keeps the secondary entries short)."""
    return float(f"{x:.{n}g}") if isinstance(x, float) else x


def timed_launches(step, steps, warmup, stream):
    """W untimed launches, then K launches between two synchronisations, each bracketed by HIP events recorded
    on the launch stream.  Returns (wall seconds for the K launches, per-launch device milliseconds)."""
    import torch

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a, b in ev:
        a.record(stream)
        step()
        b.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return wall, [a.elapsed_time(b) for a, b in ev]


def make_case(workload, T=None, B=None, d=None):
    import vla_inputs

    c = dict(vla_inputs.CONFIGS[workload])
    if workload == "long_context":
        c["T"] = T or 131072
    elif T:
        c["T"] = T
    if B:
        c["B"] = B
    if d:
        c["d"] = d
        if "std" in c and workload == "large_batch":
            c["std"] = d ** -0.5
    c["workload"] = workload
    return c


def forward_case(c, *, mode=0, segments=None, options="none", steps=10, warmup=3, oracle_heads=0,
                 time_oracle=False, copy_probe=False):
    """One vla_forward workload: inputs on the GPU, timing, roofline, and the oracle on `oracle_heads` evenly
    spaced heads over the full sequence (error of o; its rate when time_oracle)."""
    import numpy as np
    import torch

    import paper_2605_11196_amd as vla
    import vla_inputs

    B, H, T, d = c["B"], c["H"], c["T"], c["d"]
    dtype = c["dtype"]
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    io = vla.VLA_BF16 if dtype == "bf16" else vla.VLA_F32
    dev = torch.device("cuda:0")
    if c["workload"] == "recall":
        qn, kn, vn, _ = vla_inputs.recall_task(B, H, T, d, c["seed"], c["n_pairs"])
        q, k, v = (torch.from_numpy(x).to(dev) for x in (qn, kn, vn))
    elif dtype == "bf16":
        q, k, v = vla_inputs.device_gaussian(B, H, T, d, c["seed"], c["std"], tdt)
    else:
        q, k, v = (torch.from_numpy(x).to(dev)
                   for x in vla_inputs.gaussian_qkv(B, H, T, d, c["seed"], c["std"]))
    extra = {}
    u = None
    if options != "none":
        gen_u = torch.Generator(device=dev)
        gen_u.manual_seed(c["seed"] + 1000)
        u = torch.randn(B, H, T, d, device=dev, generator=gen_u).to(tdt)
        extra = dict(u=u.data_ptr(), u_scale=d ** -0.5, normalise_output=1, feature_map=1)
        if options == "paper":
            extra.update(refresh_period=20, refresh_eta=1e-3)
    o = torch.empty_like(v)
    S_T = torch.empty((B, H, d, d), dtype=torch.float32, device=dev)
    A_T = torch.empty((B, H, d, d), dtype=torch.float32, device=dev)
    need = vla.vla_forward_workspace_bytes(B, H, T, d, d, io, lambda0=c["lambda0"], mode=mode,
                                           segments=segments, **extra)
    ws = torch.empty((max(need, 16),), dtype=torch.uint8, device=dev)
    resolved = vla.resolve_mode(B, H, T, d, d, io, mode=mode, **extra)
    stream = torch.cuda.current_stream(dev)

    def step():
        rc = vla.vla_forward_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), 0, 0, o.data_ptr(),
                                 S_T.data_ptr(), A_T.data_ptr(), B, H, T, d, d, io,
                                 lambda0=c["lambda0"], mode=mode, workspace=ws.data_ptr(),
                                 workspace_bytes=need, stream=stream.cuda_stream, segments=segments,
                                 **extra)
        if rc != 0:
            raise RuntimeError(vla.status_string(rc))

    if copy_probe:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)   # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.mul(src, 1.0, out=dst)                                 # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    wall, dev_ms = timed_launches(step, steps, warmup, stream)
    avg_s = sum(dev_ms) / len(dev_ms) / 1e3
    med_s = statistics.median(dev_ms) / 1e3
    head_tokens = B * H * T
    # algorithmic work per launch: 5 d^2 FMA per head-token (6 d^2 with separate penalty directions); q, k, v
    # (and u) read and o written once, S_T and A_T written once per head
    flops = (12.0 if options != "none" else 10.0) * d * d * head_tokens
    n_streams = 5 if options != "none" else 4
    io_bytes = (2 if dtype == "bf16" else 4) * n_streams * d * head_tokens + B * H * 2 * d * d * 4
    tflops = flops / avg_s / 1e12
    traffic, traffic_src = PROFILED_TRAFFIC_BYTES.get((B, H, T, d, dtype, resolved), (None, None))
    if options != "none":
        traffic, traffic_src = None, None
    workload = (f"{c['workload']}: B={B} H={H} T={T} d_h={d} {dtype} q/k/v/o, fp32 A and S, "
                f"lambda0={c['lambda0']}")
    if options == "paper":
        workload += ", every option of Algorithm 1 on (u with u_scale=1/sqrt(d_h), refresh 20, normalised, ELU+1)"
    elif options == "paper_no_refresh":
        workload += ", options of Algorithm 1 on (u with u_scale=1/sqrt(d_h), normalised, ELU+1; no refresh)"
    res = {
        "workload": workload, "io_dtype": dtype, "kernel_mode": MODE_NAMES.get(resolved, str(resolved)),
        "B": B, "H": H, "T": T, "d": d, "head_tokens": head_tokens, "steps": steps, "warmup": warmup,
        "wall_s": wall, "value": head_tokens * steps / wall, "ms_per_step": wall / steps * 1e3,
        "roofline": {
            "bound": "mfma" if resolved in (2, 3, 4) else "alu",
            "achieved": tflops, "peak": PEAK_FP32_TFLOPS, "unit": "TFLOP/s", "frac": tflops / PEAK_FP32_TFLOPS,
            "traffic": traffic, "traffic_source": traffic_src,
            "kernel_ms": avg_s * 1e3, "kernel_ms_median": med_s * 1e3,
            "frac_median": flops / med_s / 1e12 / PEAK_FP32_TFLOPS,
            "algorithmic_flop_per_launch": flops, "algorithmic_bytes_per_launch": io_bytes,
            "hbm_GBps": io_bytes / avg_s / 1e9, "hbm_frac": io_bytes / avg_s / 1e9 / PEAK_HBM_GBS,
        },
    }
    if oracle_heads:
        import oracle

        n_all = B * H
        idx = sorted(set(int(i) for i in np.linspace(0, n_all - 1, num=min(oracle_heads, n_all))))
        sel = torch.tensor(idx, device=dev)
        pick = lambda x: x.reshape(n_all, *x.shape[2:]).index_select(0, sel).float().cpu().numpy()[None]
        qs, ks, vs = (pick(x).astype(np.float64) for x in (q, k, v))
        oracle.load()
        oracle_opt = {}
        if options != "none":
            oracle_opt = dict(u=pick(u).astype(np.float64), u_scale=extra["u_scale"],
                              refresh_period=extra.get("refresh_period", 0),
                              refresh_eta=extra.get("refresh_eta", 1e-3),
                              normalise_output=True, feature_map=True)
        tc0 = time.perf_counter()
        ref = oracle.forward(qs, ks, vs, lambda0=c["lambda0"], **oracle_opt)
        tc1 = time.perf_counter()
        got = pick(o).astype(np.float64)
        den = np.abs(ref["o"]).max(axis=(2, 3))
        res["oracle"] = {
            "heads": len(idx), "n_all": n_all, "seconds": tc1 - tc0, "rate": len(idx) * T / (tc1 - tc0),
            "cores": oracle.num_threads(),
            "max_rel_err_o": float((np.abs(got - ref["o"]).max(axis=(2, 3)) / np.where(den > 0, den, 1.0)).max()),
        }
    del q, k, v, o, S_T, A_T, ws, u
    torch.cuda.empty_cache()
    return res


def decode_case(c, *, steps=10, warmup=3, oracle_heads=0):
    """One decode step per timed step: every head of the workload advances by one token on its resident state.
    Algorithmic traffic per head-token: S and A read and written (4 d^2 float32) + q, k, v read and o written."""
    import numpy as np
    import torch

    import paper_2605_11196_amd as vla

    B, H, d = c["B"], c["H"], c["d"]
    dtype = c["dtype"]
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    io = vla.VLA_BF16 if dtype == "bf16" else vla.VLA_F32
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(c["seed"])
    n_tok = warmup + steps
    q, k, v = ((torch.randn(n_tok, B, H, d, device=dev, generator=gen) * d ** -0.5).to(tdt) for _ in range(3))
    S = torch.zeros(B, H, d, d, device=dev)
    A = (torch.eye(d, device=dev) / c["lambda0"]).repeat(B, H, 1, 1).contiguous()
    o = torch.empty(n_tok, B, H, d, dtype=tdt, device=dev)
    stream = torch.cuda.current_stream(dev)
    tok = [0]

    def step():
        t = tok[0]
        tok[0] += 1
        rc = vla.vla_decode_step_raw(q[t].data_ptr(), k[t].data_ptr(), v[t].data_ptr(), S.data_ptr(),
                                     A.data_ptr(), o[t].data_ptr(), B, H, d, d, io, stream=stream.cuda_stream)
        if rc != 0:
            raise RuntimeError(vla.status_string(rc))

    wall, dev_ms = timed_launches(step, steps, warmup, stream)
    avg_s = sum(dev_ms) / len(dev_ms) / 1e3
    med_s = statistics.median(dev_ms) / 1e3
    heads = B * H
    nbytes = heads * (4 * d * d * 4 + 4 * d * (2 if dtype == "bf16" else 4))
    gbps = nbytes / avg_s / 1e9
    res = {
        "workload": f"decode: {heads} heads (B={B} H={H}) d_h={d} {dtype} q/k/v/o, fp32 A and S "
                    f"updated in place, one token per step",
        "io_dtype": dtype, "kernel_mode": "decode", "B": B, "H": H, "T": 1, "d": d, "head_tokens": heads,
        "steps": steps, "warmup": warmup, "wall_s": wall, "value": heads * steps / wall,
        "ms_per_step": wall / steps * 1e3,
        "roofline": {"bound": "hbm", "achieved": gbps, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": gbps / PEAK_HBM_GBS, "traffic": None, "kernel_ms": avg_s * 1e3,
                     "kernel_ms_median": med_s * 1e3, "frac_median": nbytes / med_s / 1e9 / PEAK_HBM_GBS,
                     "algorithmic_bytes_per_launch": nbytes},
    }
    if oracle_heads:
        import oracle

        idx = sorted(set(int(i) for i in np.linspace(0, heads - 1, num=min(oracle_heads, heads))))
        sel = torch.tensor(idx, device=dev)
        # the whole token sequence of the sampled heads, [1, n, n_tok, d], from S = 0 and A = I / lambda0
        pick = lambda x: x.reshape(n_tok, heads, d).index_select(1, sel).float().cpu().numpy().transpose(1, 0, 2)[None]
        ref = oracle.forward(pick(q).astype(np.float64), pick(k).astype(np.float64), pick(v).astype(np.float64),
                             lambda0=c["lambda0"])
        got = pick(o).astype(np.float64)
        den = np.abs(ref["o"]).max(axis=(2, 3))
        gS = S.reshape(heads, d, d).index_select(0, sel).cpu().numpy().astype(np.float64)[None]
        res["oracle"] = {
            "heads": len(idx), "n_all": heads,
            "max_rel_err_o": float((np.abs(got - ref["o"]).max(axis=(2, 3)) / den).max()),
            "max_rel_err_S": float((np.abs(gS - ref["S_T"]).max(axis=(2, 3)) /
                                    np.abs(ref["S_T"]).max(axis=(2, 3))).max()),
        }
    return res


def secondary_entry(name, r):
    rf = r["roofline"]
    e = {"name": name, "shape": f"B={r['B']} H={r['H']} T={r['T']} d_h={r['d']} {r['io_dtype']}",
         "kernel_mode": r["kernel_mode"],
         "value": sig(r["value"]), "unit": "head-tokens/s", "steps": r["steps"],
         "ms_per_step": sig(r["ms_per_step"]), "kernel_ms": sig(rf["kernel_ms"]),
         "kernel_ms_median": sig(rf["kernel_ms_median"]),
         "roofline": {"bound": rf["bound"], "achieved": sig(rf["achieved"]), "peak": rf["peak"],
                      "unit": rf["unit"], "frac": sig(rf["frac"]), "frac_median": sig(rf["frac_median"])}}
    if "oracle" in r:
        e["oracle_heads"] = r["oracle"]["heads"]
        e["max_rel_err_o"] = sig(r["oracle"]["max_rel_err_o"], 3)
        if "max_rel_err_S" in r["oracle"]:
            e["max_rel_err_S"] = sig(r["oracle"]["max_rel_err_S"], 3)
    return e


def headline_line(r, args, metric="VLA forward tokens/sec (B*H*T/s)"):
    out = {
        "metric": metric, "value": r["value"], "unit": "head-tokens/s", "n_gpus": 1,
        "steps": r["steps"], "warmup": r["warmup"], "ms_per_step": r["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": r["workload"], "io_dtype": r["io_dtype"], "kernel_mode": r["kernel_mode"],
                   "global_batch": r["B"], "heads": r["H"], "seq_len": r["T"], "d_h": r["d"],
                   "parallelism": "single-gpu"},
        "roofline": r["roofline"],
    }
    if "oracle" in r and "rate" in r["oracle"]:
        oc = r["oracle"]
        out["cpu_baseline"] = {
            "value": oc["rate"], "unit": "head-tokens/s", "cores": oc["cores"], "kind": "oracle",
            "sample": f"{oc['heads']} of {oc['n_all']} heads (evenly spaced) x all {r['T']} tokens, fp64, "
                      f"{oc['seconds']:.1f} s",
            "gpu_vs_oracle_max_rel_err_o": oc["max_rel_err_o"],
        }
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (heads are independent, so more GPUs "
              "would only split the batch); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch

    torch.cuda.set_device(torch.device("cuda:0"))
    c = make_case(args.workload, args.T, args.B, args.d)
    if args.decode:
        r = decode_case(c, steps=args.steps, warmup=args.warmup)
        print(json.dumps(headline_line(r, args, metric="VLA decode step tokens/sec (B*H/s)")))
        return

    default_run = (args.workload == "large_batch" and not (args.T or args.B or args.d or args.mode or args.segments)
                   and args.options == "none")
    n_all = c["B"] * c["H"]
    want = 0 if args.no_cpu_baseline else (
        args.cpu_heads or max(1, min(n_all, int(3.0e6 * (128.0 / c["d"]) ** 2 / max(c["T"], 1)))))
    r = forward_case(c, mode=args.mode, segments=args.segments, options=args.options, steps=args.steps,
                     warmup=args.warmup, oracle_heads=want, time_oracle=True, copy_probe=args.copy_probe)
    out = headline_line(r, args)

    if default_run and not args.no_secondary:
        # at least 10 timed launches each (the median is reported next to the mean)
        k2, w2 = max(10, args.steps), max(2, min(args.warmup, 3))
        sec = []
        sec.append(secondary_entry("large_batch_d64", forward_case(
            make_case("large_batch", d=64), steps=k2, warmup=w2, oracle_heads=8)))
        # the long-context calls take 0.2 to 3 ms and each follows seconds of oracle work on the host, during
        # which the GPU clocks fall: more warm-up launches and 30 timed ones (about 0.1 s per entry)
        k3, w3 = max(30, args.steps), 10
        for T in make_case("long_context")["T_sweep"]:
            sec.append(secondary_entry(f"long_context_T{T}", forward_case(
                make_case("long_context", T=T), steps=k3, warmup=w3, oracle_heads=2)))
        sec.append(secondary_entry("long_context_T32768_d128", forward_case(
            make_case("long_context", T=32768, d=128), steps=k3, warmup=w3, oracle_heads=1)))
        sec.append(secondary_entry("long_context_T131072_options_no_refresh", forward_case(
            make_case("long_context", T=131072), options="paper_no_refresh", steps=k3, warmup=w3, oracle_heads=2)))
        sec.append(secondary_entry("large_batch_options_paper", forward_case(
            make_case("large_batch"), options="paper", steps=k2, warmup=w2, oracle_heads=4)))
        sec.append(secondary_entry("decode_large_batch_heads", decode_case(
            make_case("large_batch"), steps=k3, warmup=w3, oracle_heads=8)))
        out["secondary"] = sec
    print(json.dumps(out))


if __name__ == "__main__":
    main()
