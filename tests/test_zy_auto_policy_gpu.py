"""AUTO's choice of kernel family against the named modes, timed on the GPU at shapes away from the ones the
thresholds were measured at: the mode AUTO resolves to must not be much slower than the best named block mode
(fused block kernel or time-parallel)."""
import statistics

import pytest

pytestmark = pytest.mark.gpu

CHUNKED, TIME_PARALLEL = 2, 4
# A timing test: the bound leaves room for launch-to-launch noise at sub-millisecond sizes and for the width of the
# crossover region (measured: AUTO picks the faster mode at every shape below), a shape that misses it is
# timed once more before it counts, and the file sorts after the parity tests so that a noisy box cannot hide them.
SLACK = 1.6

SHAPES = [  # (d, heads, T)
    (64, 16, 700), (64, 16, 3000), (64, 16, 24000), (64, 48, 600), (64, 48, 5000), (64, 100, 1500),
    (64, 100, 20000), (64, 160, 4096), (64, 224, 9000), (64, 512, 2048), (64, 2048, 1024),
    (128, 8, 1500), (128, 24, 700), (128, 40, 9000), (128, 80, 6000), (128, 112, 20000), (128, 160, 4096), (128, 512, 2048),
    (32, 32, 800), (32, 200, 3000), (32, 300, 6000), (32, 1500, 2048),
    (96, 16, 1500), (96, 40, 6000), (96, 112, 20000), (96, 200, 3000), (96, 48, 1100), (96, 120, 5000),
    (128, 120, 10000), (128, 8, 40000), (64, 300, 6000), (32, 200, 600),
]


def _time(fn, reps=7):
    import torch

    for _ in range(2):
        fn()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    st = torch.cuda.current_stream()
    for a, b in ev:
        a.record(st)
        fn()
        b.record(st)
    torch.cuda.synchronize()
    return statistics.median(a.elapsed_time(b) for a, b in ev)


RECT_SHAPES = [  # (d_k, d_v, heads, T): value heads of another size than the key heads
    (64, 128, 16, 6000), (64, 128, 350, 6000), (64, 128, 600, 3000), (128, 64, 120, 5000), (128, 16, 200, 4096),
    (32, 128, 900, 3000), (64, 16, 16, 20000), (96, 32, 100, 9000), (32, 16, 2000, 2048),
]


@pytest.mark.parametrize("d,heads,T", SHAPES)
def test_auto_is_close_to_the_best_named_mode(d, heads, T):
    _check(d, d, heads, T)


@pytest.mark.parametrize("d,d_v,heads,T", RECT_SHAPES)
def test_auto_is_close_to_the_best_named_mode_with_value_heads_of_another_size(d, d_v, heads, T):
    _check(d, d_v, heads, T)


def _check(d, d_v, heads, T):
    import torch

    import paper_2605_11196_amd as vla

    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev)
    g.manual_seed(d + heads + T)
    q, k = ((torch.randn(1, heads, T, d, device=dev, generator=g) * d ** -0.5).to(torch.bfloat16) for _ in range(2))
    v = (torch.randn(1, heads, T, d_v, device=dev, generator=g) * d ** -0.5).to(torch.bfloat16)
    o = torch.empty_like(v)
    st = torch.cuda.current_stream().cuda_stream
    def measure():
      times = {}
      for mode in (0, CHUNKED, TIME_PARALLEL):
          if mode and vla.resolve_mode(1, heads, T, d, d_v, vla.VLA_BF16, mode=mode) != mode:
              continue
          need = vla.vla_forward_workspace_bytes(1, heads, T, d, d_v, vla.VLA_BF16, mode=mode)
          ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)

          def call(mode=mode, ws=ws, need=need):
              rc = vla.vla_forward_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), 0, 0, o.data_ptr(), 0, 0, 1, heads,
                                       T, d, d_v, vla.VLA_BF16, mode=mode, workspace=ws.data_ptr(),
                                       workspace_bytes=need, stream=st)
              assert rc == 0

          times[mode] = _time(call)
      return times

    times = measure()
    best = min(t for m, t in times.items() if m)
    resolved = vla.resolve_mode(1, heads, T, d, d_v, vla.VLA_BF16)
    print(f"d={d} d_v={d_v} heads={heads} T={T}: auto -> mode {resolved}: {times[0]:.3f} ms; "
          + ", ".join(f"mode {m}: {t:.3f}" for m, t in times.items() if m))
    if times[0] > SLACK * best:      # once more before it counts
        times = measure()
        best = min(t for m, t in times.items() if m)
    assert times[0] <= SLACK * best, (resolved, times)
