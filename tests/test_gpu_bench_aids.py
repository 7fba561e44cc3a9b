"""The library's benchmark aids on the GPU: they are not steps of the layer, but bench.py's ceilings and the
evidence under profiles/ rest on them, so they are checked for what they claim to do."""
import numpy as np
import pytest

from paper_2504_03871_amd import binding as B

pytestmark = pytest.mark.gpu


def test_stream_copy_and_fill():
    import torch
    dev = "cuda:0"
    n = (1 << 22) + 4096                      # not a multiple of the kernel's per-block span
    src = torch.randint(-2 ** 31, 2 ** 31 - 1, (n // 4,), dtype=torch.int32, device=dev)
    dst = torch.full((n // 4 + 64,), 7, dtype=torch.int32, device=dev)
    B.moe_bench_stream(dst, src, n, 0)
    torch.cuda.synchronize()
    assert torch.equal(dst[: n // 4], src) and bool((dst[n // 4:] == 7).all())     # copied exactly, nothing past the end
    B.moe_bench_stream(dst, src, n, 1)
    torch.cuda.synchronize()
    assert bool((dst[: n // 4] == 0).all()) and bool((dst[n // 4:] == 7).all())


def test_clock_probe_counts_cycles():
    import torch
    dev = "cuda:0"
    n = 200
    samples = torch.zeros(2 * n, dtype=torch.int64, device=dev)
    B.moe_bench_clock_probe(samples, n, 4)
    torch.cuda.synchronize()
    sm = samples.cpu().numpy().reshape(n, 2)
    d_shader, d_real = np.diff(sm[:, 0]), np.diff(sm[:, 1])
    assert (d_shader > 0).all() and (d_real > 0).all()
    mhz = d_shader.sum() / d_real.sum() * 100.0          # the second counter ticks at 100 MHz
    assert 300.0 < mhz < 3000.0


def test_mfma_loop_runs_and_is_deterministic():
    import torch
    dev = "cuda:0"
    opnd = (torch.randn(64 * 1024, device=dev) * 0.5).to(torch.bfloat16)
    for kind in (0, 1):
        sinks = []
        for _ in range(2):
            sink = torch.full((1024 * 512,), float("nan"), dtype=torch.float32, device=dev)
            B.moe_bench_mfma_loop(kind, 3, opnd, sink)
            torch.cuda.synchronize()
            sinks.append(sink)
        assert bool(torch.isfinite(sinks[0]).all()) and torch.equal(sinks[0], sinks[1])
        assert float(sinks[0].abs().max()) > 0.0
