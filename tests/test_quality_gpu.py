"""GPU parity of the compressor-quality diagnostics (phi of Proposition 1,
delta of the non-block compressor, Section 3.2) against the CPU oracle.

Both sides add non-negative fp64 terms, in different orders: the sums agree to
n * 2^-53 relative (below 1e-10 for every size used here), the ratios to three
times that; the tests allow 1e-9.  Repeated calls must give the same bits.
"""
import zlib

import numpy as np
import pytest
import torch

import ef_workloads as wl
import oracle
import paper_1905_10936_amd as ef
from tests.parity_util import F
from tests.test_parity_gpu import LAYOUTS, _offs

pytestmark = pytest.mark.gpu
REL = 1e-9


def _vectors(rng, n, d, offs):
    v = rng.standard_normal((n, d)) * np.repeat(10.0 ** rng.uniform(-3, 2, len(offs) - 1), np.diff(offs))
    v = v.astype(F)
    v[0, rng.random(d) < 0.5] = 0.0                  # a sparse vector: small ratios
    if n > 1:
        v[1, : offs[1]] = 0.0                        # a block of zeros is skipped
    if n > 2:
        v[2] = 0.0                                   # all zeros: (1, 1)
    return v


@pytest.mark.parametrize("name", list(LAYOUTS))
def test_quality_parity(name):
    offs = _offs(LAYOUTS[name])
    d = int(offs[-1])
    n = 4
    rng = np.random.default_rng(zlib.crc32(name.encode()) + 41)
    v = _vectors(rng, n, d, offs)
    ds = (d + 3) // 4 * 4
    dev = torch.device("cuda:0")
    plan = ef.Plan(offs, n)
    vg = torch.zeros((n, ds), dtype=torch.float32, device=dev)
    vg[:, :d].copy_(torch.from_numpy(v))
    out = torch.full((n, 2), -1.0, dtype=torch.float64, device=dev)
    ef.ef_compressor_quality(plan, vg, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    for i in range(n):
        phi, delta = oracle.quality(v[i], offs)
        assert got[i, 0] == pytest.approx(phi, rel=REL), "%s vector %d phi" % (name, i)
        assert got[i, 1] == pytest.approx(delta, rel=REL), "%s vector %d delta" % (name, i)
    out2 = torch.full((n, 2), -1.0, dtype=torch.float64, device=dev)
    ef.ef_compressor_quality(plan, vg, out2)
    torch.cuda.synchronize()
    assert torch.equal(out, out2), "repeated call changed bits"
    plan.close()


def test_quality_constant_magnitude_example_on_gpu():
    """The Section 3.2 example: phi = 1, delta = (1+a)(1-a^B) / (B (1-a)(1+a^B))."""
    alpha, B, n = 0.5, 8, 5000                       # blocks of 5000: tiles hold parts of two blocks
    c = np.array([alpha ** (B - 1 - b) for b in range(B)])
    rng = np.random.default_rng(2)
    v = (np.repeat(c, n) * rng.choice([-1.0, 1.0], size=B * n)).astype(F)
    offs = np.arange(B + 1) * n
    dev = torch.device("cuda:0")
    plan = ef.Plan(offs, 1)
    out = torch.zeros(2, dtype=torch.float64, device=dev)
    ef.ef_compressor_quality(plan, torch.from_numpy(v).to(dev), out)
    torch.cuda.synchronize()
    phi, delta = out.cpu().numpy()
    assert phi == pytest.approx(1.0, rel=1e-12)
    assert delta == pytest.approx((1 + alpha) * (1 - alpha ** B) / (B * (1 - alpha) * (1 + alpha ** B)), rel=1e-9)
    plan.close()


def test_quality_resnet50_full_size():
    w = wl.get("resnet50_like")
    dev = torch.device("cuda:0")
    plan = ef.Plan(w.offsets, 2)
    ds = (w.d + 3) // 4 * 4
    vg = torch.zeros((2, ds), dtype=torch.float32, device=dev)
    for i in range(2):
        w.grad(0, i, device=dev, out=vg[i, :w.d])
    out = torch.zeros((2, 2), dtype=torch.float64, device=dev)
    ef.ef_compressor_quality(plan, vg, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    for i in range(2):
        phi, delta = oracle.quality(np.ascontiguousarray(vg[i, :w.d].cpu().numpy()), w.offsets)
        assert got[i, 0] == pytest.approx(phi, rel=REL) and got[i, 1] == pytest.approx(delta, rel=REL)
        assert got[i, 0] > got[i, 1]            # per-tensor blocks beat one global scale (Fig. 1(b) of the paper)
    plan.close()


def test_quality_rejects_bad_arguments():
    offs = _offs([100, 28])
    dev = torch.device("cuda:0")
    plan = ef.Plan(offs, 1)
    v = torch.zeros((2, 128), dtype=torch.float32, device=dev)
    out = torch.zeros((2, 2), dtype=torch.float64, device=dev)
    with pytest.raises(ef.EfError) as ei:
        ef.ef_compressor_quality(plan, v, out)          # more vectors than the plan allows
    assert ei.value.code == ef.EF_ERR_ARG
    plan.close()
