"""GPU parity of the momentum-free worker (Algorithm 3, dist-EF-blockSGD)
against the CPU oracle, with a stepsize that rises and falls so that the
eta_{t-1}/eta_t factor of the residual is exercised on both sides of 1.
Bar as for the momentum worker: sign words bit-exact, scales within 1e-6
relative, residuals bit-exact wherever the block's scale is bit-equal.
"""
import zlib

import numpy as np
import pytest
import torch

import oracle
import paper_1905_10936_amd as ef
from tests.parity_util import F, GpuState, check_scales, check_vector, to_np
from tests.test_parity_gpu import LAYOUTS, _grads, _offs

pytestmark = pytest.mark.gpu

ETAS = [0.05, 0.1, 0.2, 0.1, 0.025]


@pytest.mark.parametrize("route", ["one_pass", "two_pass", "deferred", "direct", "direct_mixed"])
@pytest.mark.parametrize("name", list(LAYOUTS))
def test_sgd_worker_parity(name, route):
    offs = _offs(LAYOUTS[name])
    d = int(offs[-1])
    M = 3
    rng = np.random.default_rng(zlib.crc32(name.encode()) + 29)
    g = _grads(rng, len(ETAS), M, d, zeros=0.05)
    st = GpuState(offs, M, route=route)
    e_ref = np.zeros((M, d), F)
    eta_prev = 0.0
    for t, eta in enumerate(ETAS):
        st.set_grads(g[t])
        st.ws.fill_(0x5555555555555555)
        st.wc.fill_(-7.0)
        # the oracle starts each step from the GPU's residual: errors cannot compound
        e_ref[:] = to_np(st.e[:, :d])
        ef.ef_worker_step_sgd(st.plan, st.g, st.e, eta_prev, eta, st.ws, st.wc)
        torch.cuda.synchronize()
        ws, wc = to_np(st.ws), to_np(st.wc)
        for i in range(M):
            s_ref, c_ref = oracle.worker_step_sgd(g[t, i], e_ref[i], offs, F(eta_prev), F(eta))
            tag = "%s/%s t=%d worker %d" % (name, route, t, i)
            assert np.array_equal(ws[i], s_ref), tag + ": sign words differ"
            same = check_scales(wc[i], c_ref, tag)
            check_vector(to_np(st.e[i, :d]), e_ref[i], c_ref, same, offs, tag + " residual")
        assert not to_np(st.m).any(), "the momentum-free worker wrote a momentum buffer it was never given"
        eta_prev = eta
    st.plan.close()


def test_sgd_worker_equals_momentum_worker_at_mu_zero():
    """Section 4.1: mu = 0 in Algorithm 4 gives Algorithm 3; on the GPU the two
    entry points must emit the same payloads and residuals."""
    offs = _offs(LAYOUTS["mixed_tiny_and_big"])
    d = int(offs[-1])
    M = 2
    rng = np.random.default_rng(3)
    a, b = GpuState(offs, M), GpuState(offs, M)
    eta_prev = 0.0
    for t, eta in enumerate(ETAS):
        g = _grads(rng, 1, M, d)[0]
        a.set_grads(g)
        b.set_grads(g)
        ef.ef_worker_step(a.plan, a.g, a.m, a.e, 0.0, eta_prev, eta, a.ws, a.wc)
        ef.ef_worker_step_sgd(b.plan, b.g, b.e, eta_prev, eta, b.ws, b.wc)
        torch.cuda.synchronize()
        assert torch.equal(a.ws, b.ws) and torch.equal(a.wc, b.wc) and torch.equal(a.e, b.e), "step %d" % t
        eta_prev = eta
    a.plan.close()
    b.plan.close()
