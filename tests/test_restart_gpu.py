"""Restart on the GPU: the state of Algorithm 4 is the momentum and residual of every worker, the
server residual, the parameters and the previous stepsize (its initialisation line); a run of T
steps must equal, bit for bit, T1 steps + a snapshot of exactly that state taken to the host + a
fresh plan and fresh buffers restored from it + the remaining steps.  In the deferred-correction
mode the snapshot is taken after ef_flush, as its contract asks."""
import numpy as np
import pytest
import torch

import paper_1905_10936_amd as ef
from tests.parity_util import F, GpuState, to_np
from tests.test_lazy_gpu import SIZES, _offs, _raw_step

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("lazy", [False, True])
@pytest.mark.parametrize("route", ["one_pass", "direct", "two_pass"])
def test_restart_from_host_snapshot_is_bit_identical(route, lazy):
    offs = _offs(SIZES["ragged_large"])
    d = int(offs[-1])
    M, T, T1, mu = 3, 6, 2, 0.9
    etas = [0.4, 0.4, 0.2, 0.2, 0.1, 0.05]
    rng = np.random.default_rng(808)
    grads = [rng.standard_normal((M, d)).astype(F) for _ in range(T)]
    x0 = rng.standard_normal(d).astype(F)

    def fresh():
        st = GpuState(offs, M, x0=x0, route=route)
        if lazy:
            if route != "two_pass":
                st.plan.tune(fuse_limit=3)
            st.plan.set_lazy(True)
        return st

    def run(st, t_from, t_to):
        for t in range(t_from, t_to):
            st.set_grads(grads[t])
            _raw_step(st, "sgdm", mu, etas[t - 1] if t else 0.0, etas[t])

    whole = fresh()
    run(whole, 0, T)
    first = fresh()
    run(first, 0, T1)
    if lazy:
        ef.ef_flush(first.plan, first.e, first.te)
    torch.cuda.synchronize()
    snap = {k: to_np(getattr(first, k)).copy() for k in ("m", "e", "te", "x")}     # host copy: the whole state
    first.plan.close()
    del first
    second = fresh()
    for k, v in snap.items():
        getattr(second, k).copy_(torch.as_tensor(v))
    run(second, T1, T)
    for st in (whole, second):
        if lazy:
            ef.ef_flush(st.plan, st.e, st.te)
    torch.cuda.synchronize()
    for k in ("m", "e", "te", "x", "ws", "wc", "ss", "sc"):
        a, b = to_np(getattr(whole, k)), to_np(getattr(second, k))
        a = a.view(np.uint32) if a.dtype == np.float32 else a
        b = b.view(np.uint32) if b.dtype == np.float32 else b
        assert np.array_equal(a, b), "%s differs after the restart (%d entries)" % (k, int((a != b).sum()))
    whole.plan.close()
    second.plan.close()
