"""GPU parity of the parameter update with weight decay (Appendix A) against
the CPU oracle.

The update is elementwise fp32 with one rounding per operation on both sides,
fed with the same payload, so parameters and decay momentum must agree bit for
bit after every step.
"""
import zlib

import numpy as np
import pytest
import torch

import oracle
import paper_1905_10936_amd as ef
from tests.parity_util import F, to_np
from tests.test_parity_gpu import LAYOUTS, _offs

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", list(LAYOUTS))
def test_apply_wd_parity(name):
    offs = _offs(LAYOUTS[name])
    d = int(offs[-1])
    rng = np.random.default_rng(zlib.crc32(name.encode()) + 5)
    x = rng.standard_normal(d).astype(F)
    mt = np.zeros(d, F)
    dev = torch.device("cuda:0")
    plan = ef.Plan(offs, 1)
    xg = torch.from_numpy(x.copy()).to(dev)
    mg = torch.zeros(d, dtype=torch.float32, device=dev)
    mu, lam = 0.9, 5e-4
    for t, eta in enumerate([0.1, 0.1, 0.05]):
        v = rng.standard_normal(d).astype(F)
        v[rng.random(d) < 0.05] = 0.0
        signs, scales = oracle.compress(v, offs)
        oracle.apply_wd(x, mt, signs, scales, offs, F(eta), F(mu), F(lam))
        sg = torch.from_numpy(signs.view(np.int64)).to(dev)
        cg = torch.from_numpy(scales).to(dev)
        ef.ef_apply_wd(plan, xg, mg, sg, cg, eta, mu, lam)
        torch.cuda.synchronize()
        assert np.array_equal(to_np(xg).view(np.uint32), x.view(np.uint32)), "params differ at step %d" % t
        assert np.array_equal(to_np(mg).view(np.uint32), mt.view(np.uint32)), "decay momentum differs at step %d" % t
    plan.close()


def test_apply_wd_without_decay_equals_apply():
    """lambda = 0 and a zero decay momentum: ef_apply_wd and ef_apply write the same bits."""
    offs = _offs(LAYOUTS["mixed_tiny_and_big"])
    d = int(offs[-1])
    rng = np.random.default_rng(11)
    dev = torch.device("cuda:0")
    plan = ef.Plan(offs, 1)
    x0 = torch.from_numpy(rng.standard_normal(d).astype(F)).to(dev)
    signs, scales = oracle.compress(rng.standard_normal(d).astype(F), offs)
    sg = torch.from_numpy(signs.view(np.int64)).to(dev)
    cg = torch.from_numpy(scales).to(dev)
    xa, xb = x0.clone(), x0.clone()
    mg = torch.zeros(d, dtype=torch.float32, device=dev)
    ef.ef_apply(plan, xa, sg, cg, 0.1)
    ef.ef_apply_wd(plan, xb, mg, sg, cg, 0.1, 0.9, 0.0)
    torch.cuda.synchronize()
    assert torch.equal(xa, xb) and not bool(mg.any())
    plan.close()


def test_apply_wd_rejects_bad_arguments():
    offs = _offs([100, 28])
    dev = torch.device("cuda:0")
    plan = ef.Plan(offs, 1)
    x = torch.zeros(128, dtype=torch.float32, device=dev)
    m = torch.zeros(128, dtype=torch.float32, device=dev)
    s = torch.zeros(2, dtype=torch.int64, device=dev)
    c = torch.zeros(2, dtype=torch.float32, device=dev)
    for eta, mu, lam in ((0.0, 0.9, 0.0), (0.1, 1.0, 0.0), (0.1, -0.1, 0.0), (0.1, 0.9, -1e-4),
                         (0.1, 0.9, float("nan"))):
        with pytest.raises(ef.EfError):
            ef.ef_apply_wd(plan, x, m, s, c, eta, mu, lam)
    plan.close()
