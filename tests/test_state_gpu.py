"""Optimizer state held by the library (ef_state_create and the *_state calls): the iterates must be
those of the caller-owned calls, which tests/parity_util.py checks against the oracle at every
step (sign words and momentum bit-exact, scales within 1e-6 relative, residuals and parameters
bit-exact where the scale is): payloads and parameters equal bit for bit at every step, and the
exported m, e, e~ equal to the caller-owned buffers.  Export + import must work as a checkpoint:
a run that is cut, exported, and continued on a fresh plan and state gives the bits of the
uninterrupted one.

The layouts put blocks above the deferred mode's one-pass limit (64 tiles), so the held buffers
really go through the deferred correction; that is checked too (the raw export-free path is
exercised by two steps in a row before any export).
"""
import zlib

import numpy as np
import pytest
import torch

import paper_1905_10936_amd as ef
from tests.parity_util import F, GpuState, synced_step, to_np

pytestmark = pytest.mark.gpu

TILE = 4096
SIZES = {
    "large_and_small": [70 * TILE + 17, 3, 1, 700, 130 * TILE - 5, TILE, 3 * TILE, 2 * TILE + 1, 33],
    "one_large_block": [90 * TILE + 1234],
}


def _offs(sizes):
    return np.concatenate([[0], np.cumsum(np.asarray(sizes, dtype=np.int64))])


def _same(a, b, what):
    a, b = to_np(a), to_np(b)
    a = a.view(np.uint32) if a.dtype == np.float32 else a
    b = b.view(np.uint32) if b.dtype == np.float32 else b
    assert np.array_equal(a, b), "%s: %d entries differ" % (what, int((a != b).sum()))


class Held:
    """Payload buffers + parameters of a run whose m, e, e~ the library holds."""

    def __init__(self, offs, M):
        self.plan = ef.ef_plan_create(offs, M)
        self.state = ef.ef_state_create(self.plan, M)
        d, B, W = self.plan.d, self.plan.B, self.plan.W
        dev = torch.device("cuda")
        self.M = M
        self.ws = torch.zeros((M, W), dtype=torch.int64, device=dev)
        self.wc = torch.zeros((M, B), dtype=torch.float32, device=dev)
        self.ss = torch.zeros(W, dtype=torch.int64, device=dev)
        self.sc = torch.zeros(B, dtype=torch.float32, device=dev)
        self.x = torch.zeros(d, dtype=torch.float32, device=dev)

    def step(self, g, mu, eta_prev, eta):
        ef.ef_worker_step_state(self.plan, self.state, g, mu, eta_prev, eta, self.ws, self.wc)
        ef.ef_server_step_state(self.plan, self.state, self.M, self.ws, self.wc, eta_prev, eta, self.ss, self.sc)
        ef.ef_apply(self.plan, self.x, self.ss, self.sc, eta)
        torch.cuda.synchronize()

    def export(self, like):
        m, e, te = torch.full_like(like.m, 7.0), torch.full_like(like.e, 7.0), torch.full_like(like.te, 7.0)
        ef.ef_state_export(self.plan, self.state, m, e, te)
        torch.cuda.synchronize()
        return m, e, te

    def close(self):
        self.state.close()
        self.plan.close()


@pytest.mark.parametrize("layout", sorted(SIZES))
@pytest.mark.parametrize("M", [1, 3])
def test_held_state_gives_the_iterates_of_the_caller_owned_calls(layout, M):
    offs = _offs(SIZES[layout])
    d = int(offs[-1])
    rng = np.random.default_rng(zlib.crc32(layout.encode()) + M)
    ref = GpuState(offs, M, pad=1)              # caller-owned buffers, default mode, checked against the oracle
    held = Held(offs, M)
    assert held.plan.lazy and held.plan.fuse_limit == 64
    eta_prev = 0.0
    for t, eta in enumerate([0.1, 0.1, 0.05, 0.2]):
        g = rng.standard_normal((M, d)).astype(F)
        g[rng.random((M, d)) < 0.03] = 0.0
        ref.set_grads(g)
        synced_step(ref, 0.9, eta_prev, eta, None, "%s M=%d step %d" % (layout, M, t))
        held.step(ref.g, 0.9, eta_prev, eta)
        tag = "%s M=%d step %d" % (layout, M, t)
        _same(held.ws, ref.ws, tag + " worker sign words")
        _same(held.wc, ref.wc, tag + " worker scales")
        _same(held.ss, ref.ss, tag + " server sign words")
        _same(held.sc, ref.sc, tag + " server scales")
        _same(held.x, ref.x, tag + " parameters")
        if t in (1, 3):         # two steps have run without an export in between
            m, e, te = held.export(ref)
            _same(m[:, :d], ref.m[:, :d], tag + " exported momentum")
            _same(e[:, :d], ref.e[:, :d], tag + " exported residuals")
            _same(te, ref.te, tag + " exported server residual")
            assert bool((m[:, d:] == 7.0).all()) and bool((e[:, d:] == 7.0).all()), tag + ": export wrote past d"
        eta_prev = eta
    held.close()
    ref.plan.close()


def test_export_and_import_work_as_a_checkpoint():
    offs = _offs(SIZES["large_and_small"])
    d, M = int(offs[-1]), 2
    rng = np.random.default_rng(5)
    grads = [rng.standard_normal((M, d)).astype(F) for _ in range(5)]
    dev = torch.device("cuda")

    def run(held, ts, eta_prev):
        for t in ts:
            g = torch.zeros((M, (d + 3) // 4 * 4), dtype=torch.float32, device=dev)     # row stride: a multiple of 4
            g[:, :d].copy_(torch.as_tensor(grads[t]))
            held.step(g, 0.9, eta_prev, 0.1)
            eta_prev = 0.1
        return eta_prev

    whole = Held(offs, M)
    run(whole, range(5), 0.0)
    first = Held(offs, M)
    eta_prev = run(first, range(2), 0.0)
    m = torch.zeros((M, d + 8), dtype=torch.float32, device=dev)     # a checkpoint with another row stride
    e = torch.zeros((M, d + 8), dtype=torch.float32, device=dev)
    te = torch.zeros(d, dtype=torch.float32, device=dev)
    ef.ef_state_export(first.plan, first.state, m, e, te)
    x_ckpt = first.x.clone()
    torch.cuda.synchronize()
    first.close()
    second = Held(offs, M)
    ef.ef_state_import(second.plan, second.state, m, e, te)
    second.x.copy_(x_ckpt)
    run(second, range(2, 5), eta_prev)
    for a, b, what in ((second.ws, whole.ws, "worker sign words"), (second.wc, whole.wc, "worker scales"),
                       (second.ss, whole.ss, "server sign words"), (second.sc, whole.sc, "server scales"),
                       (second.x, whole.x, "parameters")):
        _same(a, b, "continued run: " + what)
    ma, ea, ta = (torch.zeros((M, d), device=dev), torch.zeros((M, d), device=dev), torch.zeros(d, device=dev))
    mb, eb, tb = (torch.zeros((M, d), device=dev), torch.zeros((M, d), device=dev), torch.zeros(d, device=dev))
    ef.ef_state_export(second.plan, second.state, ma, ea, ta)
    ef.ef_state_export(whole.plan, whole.state, mb, eb, tb)
    torch.cuda.synchronize()
    _same(ma, mb, "continued run: momentum")
    _same(ea, eb, "continued run: residuals")
    _same(ta, tb, "continued run: server residual")
    second.close()
    whole.close()


def test_state_rules():
    offs = _offs([3 * TILE, 100])
    plan = ef.ef_plan_create(offs, 2)
    with pytest.raises(ef.EfError):
        ef.ef_state_create(plan, 3)                 # more workers than the plan allows
    st = ef.ef_state_create(plan, 2)
    with pytest.raises(ef.EfError):
        ef.ef_state_create(plan, 1)                 # one state per plan
    with pytest.raises(ef.EfError):
        plan.set_lazy(False)                        # the state keeps the mode on
    other = ef.ef_plan_create(offs, 2)
    g = torch.zeros((2, int(offs[-1])), device="cuda")
    ws = torch.zeros((2, plan.W), dtype=torch.int64, device="cuda")
    wc = torch.zeros((2, plan.B), device="cuda")
    with pytest.raises(ef.EfError):
        ef.ef_worker_step_state(other, st, g, 0.9, 0.0, 0.1, ws, wc)    # a state belongs to its plan
    assert ef.lib().ef_plan_destroy(plan._h) == ef.EF_ERR_ARG            # the state goes first
    st.close()
    assert not plan.lazy
    plan.close()
    other.close()
