"""ef_stream_probe of libef_bench (the bandwidth probe bench.py sets beside the worker kernel): runs, reports a
positive time, touches nothing beyond the whole tiles it is given, and rejects bad arguments."""
import ctypes

import pytest
import torch

import paper_1905_10936_amd as ef
from paper_1905_10936_amd import bench_probe

pytestmark = pytest.mark.gpu


def test_probe_runs_and_stays_in_bounds():
    n = 37 * 4096 + 100                      # 37 whole tiles and a tail the probe must leave alone
    g = torch.randn(n, device="cuda")
    m = torch.randn(n, device="cuda")
    e = torch.randn(n, device="cuda")
    g0, m0, e0 = g.clone(), m.clone(), e.clone()
    ms, nbytes = bench_probe.ef_stream_probe(g, m, e, repeats=2)
    torch.cuda.synchronize()
    assert ms > 0.0 and nbytes == 20 * 37 * 4096
    assert torch.equal(g, g0)
    assert torch.equal(m[37 * 4096:], m0[37 * 4096:]) and torch.equal(e[37 * 4096:], e0[37 * 4096:])
    assert not torch.equal(m[:4096], m0[:4096])
    assert bool(torch.isfinite(m).all()) and bool(torch.isfinite(e).all())


@pytest.mark.parametrize("group", [0, 1, 3, 16, 256])
def test_grouped_probe_runs_and_stays_in_bounds(group):
    n = 37 * 4096 + 100
    g = torch.randn(n, device="cuda")
    m = torch.randn(n, device="cuda")
    e = torch.randn(n, device="cuda")
    g0, m0, e0 = g.clone(), m.clone(), e.clone()
    ms, nbytes = bench_probe.ef_stream_probe_grouped(g, m, e, group=group, repeats=2)
    torch.cuda.synchronize()
    assert ms > 0.0 and nbytes == 20 * 37 * 4096
    assert torch.equal(g, g0)
    assert torch.equal(m[37 * 4096:], m0[37 * 4096:]) and torch.equal(e[37 * 4096:], e0[37 * 4096:])
    # three passes (one warm-up) of m <- m/2 + g, e <- e/2 + m on every whole tile
    mm, ee = m0[:37 * 4096].clone(), e0[:37 * 4096].clone()
    for _ in range(3):
        mm = 0.5 * mm + g0[:37 * 4096]
        ee = 0.5 * ee + mm
    assert torch.allclose(m[:37 * 4096], mm, rtol=1e-5, atol=1e-6) and torch.allclose(e[:37 * 4096], ee, rtol=1e-5, atol=1e-6)
    with pytest.raises(ef.EfError):
        bench_probe.ef_stream_probe_grouped(g, m, e, group=257)


def test_probe_argument_checks():
    g = torch.zeros(8192, device="cuda")
    with pytest.raises(ef.EfError):
        bench_probe.ef_stream_probe(g[:100], g[:100].clone(), g[:100].clone())        # less than a tile
    with pytest.raises(ef.EfError):
        bench_probe.ef_stream_probe(g, g.clone(), g.clone(), repeats=0)
    with pytest.raises(ef.EfError):
        bench_probe.ef_stream_probe(g[1:4097], g.clone()[:4096], g.clone()[:4096])      # off 16 bytes
    ms = ctypes.c_float(0.0)
    assert bench_probe.lib().ef_stream_probe(None, None, None, 4096, 1, ctypes.byref(ms), None) == ef.EF_ERR_NULL
