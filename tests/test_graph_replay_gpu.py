"""A captured HIP graph of one whole iteration (worker, server, apply) replayed
several times must give, replay after replay, the bits of the same calls made
eagerly: what differs between two calls (call number, tags of the scratch
sets, which list counters are in use) is read by the kernels from device
memory, so the recorded kernel arguments stay valid.  Between the replays the
test does eager work (new gradients, an eager reference step on a second plan)
and synchronises, and every replay is compared; the last state is also checked
against the CPU oracle.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_1905_10936_amd as ef
from tests.parity_util import F, GpuState, synced_step, to_np
from tests.test_parity_gpu import LAYOUTS, _offs

pytestmark = pytest.mark.gpu


def _eager_step(st, mu, eta_prev, eta):
    ef.ef_worker_step(st.plan, st.g, st.m, st.e, mu, eta_prev, eta, st.ws, st.wc)
    ef.ef_server_step(st.plan, st.M, st.ws, st.wc, st.te, eta_prev, eta, st.ss, st.sc)
    ef.ef_apply(st.plan, st.x, st.ss, st.sc, eta)


@pytest.mark.parametrize("route", ["one_pass", "direct", "deferred", "two_pass", "direct_mixed", "direct_deferred"])
def test_graph_replays_match_eager_calls(route):
    offs = _offs(LAYOUTS["mixed_tiny_and_big"])
    d = int(offs[-1])
    M, mu, eta = 3, 0.9, 0.1
    rng = np.random.default_rng(77)
    x0 = rng.standard_normal(d).astype(F)
    a = GpuState(offs, M, x0=x0, route=route)        # replayed from a graph
    b = GpuState(offs, M, x0=x0, route=route)        # the same calls made eagerly
    g0 = rng.standard_normal((M, d)).astype(F)
    for st in (a, b):                                # first iteration (stepsize ratio 0) eagerly on both
        st.set_grads(g0)
        _eager_step(st, mu, 0.0, eta)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    a.set_grads(rng.standard_normal((M, d)).astype(F))
    snapshot = [t.clone() for t in (a.m, a.e, a.te, a.x)]
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        _eager_step(a, mu, eta, eta)                 # recorded, not run
    torch.cuda.synchronize()
    for t, s in zip((a.m, a.e, a.te, a.x), snapshot):    # capture must not have touched the state
        assert torch.equal(t, s)

    for k in range(5):
        g = rng.standard_normal((M, d)).astype(F)
        g[rng.random((M, d)) < 0.05] = 0.0
        a.set_grads(g)
        b.set_grads(g)
        torch.cuda.synchronize()
        graph.replay()
        _eager_step(b, mu, eta, eta)
        torch.cuda.synchronize()
        for name in ("ws", "wc", "ss", "sc", "m", "e", "te", "x"):
            assert torch.equal(getattr(a, name), getattr(b, name)), "replay %d: %s differs from the eager calls" % (k, name)
    # and the eager side is what the oracle computes: one more step on both, checked stage by stage
    g = rng.standard_normal((M, d)).astype(F)
    b.set_grads(g)
    synced_step(b, mu, eta, eta, None, "after the replays")
    a.set_grads(g)
    graph.replay()
    torch.cuda.synchronize()
    for name in ("ws", "ss", "m", "e", "te", "x"):
        assert torch.equal(getattr(a, name), getattr(b, name)), "last replay: %s" % name
    a.plan.close()
    b.plan.close()
