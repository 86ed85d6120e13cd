"""Deferred residual correction (ef_plan_set_lazy): a plan in that mode must
produce, step after step, the bits of a plan in the default mode fed the same
gradients: sign words, scales, momentum and parameters equal at every step, and
the residual buffers equal once ef_flush has run.  The default-mode plan is
itself checked against the CPU oracle at every step (tests/parity_util.py: sign
words and momentum bit-exact, scales within 1e-6 relative, residuals and
parameters bit-exact where the scale is), so the chain oracle == default ==
deferred holds to that bar.

The layouts put the one-pass limit (fuse_limit) below the size of some blocks,
so that those blocks' whole tiles take the deferred route; the tests also check
that the mode really was in effect (the buffer differs from e before the
flush), that worker counts may change between calls, and that the settings
which would invalidate pending corrections are refused until ef_flush.
"""
import numpy as np
import pytest
import torch

import paper_1905_10936_amd as ef
from tests.parity_util import F, GpuState, synced_step, to_np

pytestmark = pytest.mark.gpu

TILE = 4096

# sizes in elements; with fuse_limit 3 the blocks of 5+ tiles are "large"
SIZES = {
    "ragged_large": [5 * TILE + 17, 3, 1, 700, 12 * TILE - 5, TILE, 3 * TILE, 2 * TILE + 1, 7 * TILE + 2048, 33],
    "aligned_large": [4 * TILE, 8 * TILE, TILE, 2 * TILE, 6 * TILE],
    "one_large_block": [9 * TILE + 1234],
    "tiny_then_large": [1] * 70 + [10 * TILE + 1, 5, 4 * TILE + 4095],
}


def _offs(sizes):
    return np.concatenate([[0], np.cumsum(np.asarray(sizes, dtype=np.int64))])


def _raw_step(st, variant, mu, eta_prev, eta, n=None):
    n = st.M if n is None else n
    if st.fused:                 # as tests/parity_util.py poisons the padding bytes of the messages
        st.wmsg.fill_(0xA5)
        st.smsg.fill_(0xA5)
    if variant == "sgd":
        ef.ef_worker_step_sgd(st.plan, st.g[:n], st.e[:n], eta_prev, eta, st.ws[:n], st.wc[:n])
    elif st.fused:
        ef.ef_worker_step_fused(st.plan, st.g[:n], st.m[:n], st.e[:n], mu, eta_prev, eta, st.wmsg[:n])
    else:
        ef.ef_worker_step(st.plan, st.g[:n], st.m[:n], st.e[:n], mu, eta_prev, eta, st.ws[:n], st.wc[:n])
    if st.fused and variant != "sgd":
        ef.ef_server_step_fused(st.plan, n, st.wmsg[:n], st.te, eta_prev, eta, st.smsg)
        ef.ef_apply_fused(st.plan, st.x, st.smsg, eta)
    else:
        ef.ef_server_step(st.plan, n, st.ws[:n], st.wc[:n], st.te, eta_prev, eta, st.ss, st.sc)
        ef.ef_apply(st.plan, st.x, st.ss, st.sc, eta)
    torch.cuda.synchronize()


def _same_bits(a, b, what):
    a, b = to_np(a), to_np(b)
    a = a.view(np.uint32) if a.dtype == np.float32 else a
    b = b.view(np.uint32) if b.dtype == np.float32 else b
    assert np.array_equal(a, b), "%s: %d entries differ" % (what, int((a != b).sum()))


def _compare_outputs(lazy, ref, tag, n=None):
    n = lazy.M if n is None else n
    if lazy.fused:
        _same_bits(lazy.wmsg[:n], ref.wmsg[:n], tag + " worker messages")
        _same_bits(lazy.smsg, ref.smsg, tag + " server message")
    else:
        _same_bits(lazy.ws[:n], ref.ws[:n], tag + " worker sign words")
        _same_bits(lazy.wc[:n], ref.wc[:n], tag + " worker scales")
        _same_bits(lazy.ss, ref.ss, tag + " server sign words")
        _same_bits(lazy.sc, ref.sc, tag + " server scales")
    _same_bits(lazy.m, ref.m, tag + " momentum")
    _same_bits(lazy.x, ref.x, tag + " parameters")


@pytest.mark.parametrize("fused", [False, True])
@pytest.mark.parametrize("route", ["one_pass", "direct"])
@pytest.mark.parametrize("layout", sorted(SIZES))
def test_deferred_equals_default_and_oracle(layout, route, fused):
    offs = _offs(SIZES[layout])
    d = int(offs[-1])
    M, mu = 3, 0.9
    rng = np.random.default_rng(4242)
    x0 = rng.standard_normal(d).astype(F)
    ref = GpuState(offs, M, x0=x0, route=route, fused=fused, pad=1)
    lazy = GpuState(offs, M, x0=x0, route=route, fused=fused, pad=1)
    for st in (ref, lazy):
        st.plan.tune(fuse_limit=3)
    lazy.plan.set_lazy(True)
    assert lazy.plan.lazy and not ref.plan.lazy
    eta_prev = 0.0
    for t in range(4):
        eta = [0.4, 0.4, 0.1, 0.05][t]
        g = rng.standard_normal((M, d)).astype(F)
        g[rng.random((M, d)) < 0.05] = 0.0
        ref.set_grads(g)
        lazy.set_grads(g)
        tag = "%s/%s step %d" % (layout, route, t)
        synced_step(ref, mu, eta_prev, eta, None, tag)          # default mode against the oracle
        _raw_step(lazy, "sgdm", mu, eta_prev, eta)
        _compare_outputs(lazy, ref, tag)
        eta_prev = eta
    # the mode was in effect: before the flush the buffers hold p, not e, in the large blocks
    assert not np.array_equal(to_np(lazy.e), to_np(ref.e))
    assert not np.array_equal(to_np(lazy.te), to_np(ref.te))
    with pytest.raises(ef.EfError):
        lazy.plan.tune(fuse_limit=5)
    with pytest.raises(ef.EfError):
        lazy.plan.set_persistent(route != "one_pass")
    with pytest.raises(ef.EfError):
        lazy.plan.set_lazy(False)
    ef.ef_flush(lazy.plan, lazy.e, lazy.te)
    torch.cuda.synchronize()
    _same_bits(lazy.e, ref.e, layout + " residuals after flush (padding columns included)")
    _same_bits(lazy.te, ref.te, layout + " server residual after flush")
    # a second flush changes nothing, and the settings are accepted again
    ef.ef_flush(lazy.plan, lazy.e, lazy.te)
    torch.cuda.synchronize()
    _same_bits(lazy.e, ref.e, layout + " residuals after a second flush")
    lazy.plan.tune(fuse_limit=3)
    # and the run goes on from flushed buffers
    g = rng.standard_normal((M, d)).astype(F)
    for st in (ref, lazy):
        st.set_grads(g)
    synced_step(ref, mu, eta_prev, 0.05, None, layout + " after flush")
    _raw_step(lazy, "sgdm", mu, eta_prev, 0.05)
    _compare_outputs(lazy, ref, layout + " after flush")
    for st in (ref, lazy):
        st.plan.close()


@pytest.mark.parametrize("route", ["one_pass", "direct"])
def test_deferred_momentum_free_and_changing_worker_count(route):
    """Algorithm 3 calls, with the number of workers changing from call to call: a worker left out
    of a call keeps its pending correction until the next call that includes it."""
    offs = _offs(SIZES["ragged_large"])
    d = int(offs[-1])
    M = 4
    rng = np.random.default_rng(99)
    x0 = rng.standard_normal(d).astype(F)
    ref = GpuState(offs, M, x0=x0, route=route)
    lazy = GpuState(offs, M, x0=x0, route=route)
    for st in (ref, lazy):
        st.plan.tune(fuse_limit=3)
    lazy.plan.set_lazy(True)
    eta_prev = 0.0
    for t, n in enumerate([4, 2, 3, 1, 4]):
        eta = [0.2, 0.2, 0.1, 0.1, 0.05][t]
        g = rng.standard_normal((M, d)).astype(F)
        for st in (ref, lazy):
            st.set_grads(g)
            _raw_step(st, "sgd", 0.0, eta_prev, eta, n)
        _compare_outputs(lazy, ref, "%s call %d with %d workers" % (route, t, n), n)
        eta_prev = eta
    ef.ef_flush(lazy.plan, lazy.e, lazy.te)
    torch.cuda.synchronize()
    _same_bits(lazy.e, ref.e, "residuals after flush")
    _same_bits(lazy.te, ref.te, "server residual after flush")
    for st in (ref, lazy):
        st.plan.close()


@pytest.mark.parametrize("route", ["one_pass", "direct"])
def test_deferred_mode_with_its_own_limits(route):
    """Without a limit set by the caller the deferred mode picks its own (no waiting for scales
    where that was measured faster); results stay those of the default mode."""
    offs = _offs(SIZES["ragged_large"])
    d = int(offs[-1])
    M = 2
    rng = np.random.default_rng(5)
    ref = GpuState(offs, M, route=route)
    lazy = GpuState(offs, M, route=route)
    lazy.plan.set_lazy(True)
    for t in range(3):
        g = rng.standard_normal((M, d)).astype(F)
        for st in (ref, lazy):
            st.set_grads(g)
            _raw_step(st, "sgdm", 0.9, 0.1 if t else 0.0, 0.1)
        _compare_outputs(lazy, ref, "step %d" % t)
    assert not np.array_equal(to_np(lazy.te), to_np(ref.te))
    ef.ef_flush(lazy.plan, lazy.e, lazy.te)
    torch.cuda.synchronize()
    _same_bits(lazy.e, ref.e, "residuals after flush")
    _same_bits(lazy.te, ref.te, "server residual after flush")
    lazy.plan.set_lazy(False)                # nothing pending any more
    for t in range(2):
        g = rng.standard_normal((M, d)).astype(F)
        for st in (ref, lazy):
            st.set_grads(g)
            _raw_step(st, "sgdm", 0.9, 0.1, 0.1)
        _compare_outputs(lazy, ref, "default mode again, step %d" % t)
        _same_bits(lazy.e, ref.e, "residuals in the default mode")
        _same_bits(lazy.te, ref.te, "server residual in the default mode")
    for st in (ref, lazy):
        st.plan.close()


def test_flush_argument_checks():
    offs = _offs([3 * TILE])
    plan = ef.ef_plan_create(offs, 2)
    e = torch.zeros((3, 3 * TILE), dtype=torch.float32, device="cuda")
    with pytest.raises(ef.EfError):
        ef.ef_flush(plan, e)                 # more rows than max_workers
    ef.ef_flush(plan, e[:2])
    ef.ef_flush(plan)                        # nothing to do
    with pytest.raises(ef.EfError):
        ef.ef_flush(plan, e[:2, 1:].contiguous().view(-1)[1:3 * TILE + 1])   # off 16 bytes
    torch.cuda.synchronize()
    plan.close()


@pytest.mark.parametrize("route", ["one_pass", "direct"])
def test_deferred_mode_in_a_replayed_graph(route):
    """A captured iteration in the deferred mode, replayed: which buffers wait for a correction is
    device state, so every replay corrects what the replay before it left."""
    offs = _offs(SIZES["ragged_large"])
    d = int(offs[-1])
    M, mu, eta = 3, 0.9, 0.1
    rng = np.random.default_rng(31)
    x0 = rng.standard_normal(d).astype(F)
    a = GpuState(offs, M, x0=x0, route=route)        # deferred mode, replayed from a graph
    b = GpuState(offs, M, x0=x0, route=route)        # default mode, eager calls
    for st in (a, b):
        st.plan.tune(fuse_limit=3)
    a.plan.set_lazy(True)
    g0 = rng.standard_normal((M, d)).astype(F)
    for st in (a, b):
        st.set_grads(g0)
        _raw_step(st, "sgdm", mu, 0.0, eta)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        ef.ef_worker_step(a.plan, a.g, a.m, a.e, mu, eta, eta, a.ws, a.wc)
        ef.ef_server_step(a.plan, M, a.ws, a.wc, a.te, eta, eta, a.ss, a.sc)
        ef.ef_apply(a.plan, a.x, a.ss, a.sc, eta)
    torch.cuda.synchronize()
    for k in range(4):
        g = rng.standard_normal((M, d)).astype(F)
        a.set_grads(g)
        b.set_grads(g)
        torch.cuda.synchronize()
        graph.replay()
        _raw_step(b, "sgdm", mu, eta, eta)
        _compare_outputs(a, b, "%s replay %d" % (route, k))
    ef.ef_flush(a.plan, a.e, a.te)
    torch.cuda.synchronize()
    _same_bits(a.e, b.e, "residuals after flush")
    _same_bits(a.te, b.te, "server residual after flush")
    # the default-mode side is what the oracle computes
    g = rng.standard_normal((M, d)).astype(F)
    b.set_grads(g)
    synced_step(b, mu, eta, eta, None, "after the replays")
    for st in (a, b):
        st.plan.close()


@pytest.mark.parametrize("workload,steps", [("one_block_2p28", 3), ("skewed_blocks", 3), ("transformer_like", 2)])
def test_deferred_full_size(workload, steps):
    """Bench configurations (full size, default limits and kernels) of the layouts with blocks beyond
    the one-pass limit: one block of 2^28 elements; a million tiny blocks around four of 8 Mi; the
    transformer-like layout with its 51 M-element embedding and 16 workers.  Deferred and default
    mode side by side on the same gradients.  The default mode at these sizes is checked against the
    oracle in tests/test_parity_full_gpu.py."""
    import ef_workloads as wl
    w = wl.get(workload)
    dev = torch.device("cuda")
    d, B, M = w.d, w.B, w.M
    W = (d + 63) // 64
    ds = (d + 3) // 4 * 4            # row stride: the ABI wants a multiple of 4 elements
    g = torch.zeros((M, ds), dtype=torch.float32, device=dev)

    class Side:
        def __init__(self, lazy):
            self.plan = ef.ef_plan_create(w.offsets, M)
            self.plan.set_lazy(lazy)
            self.m = torch.zeros((M, ds), dtype=torch.float32, device=dev)
            self.e = torch.zeros((M, ds), dtype=torch.float32, device=dev)
            self.te = torch.zeros(d, dtype=torch.float32, device=dev)
            self.x = torch.zeros(d, dtype=torch.float32, device=dev)
            self.ws = torch.zeros((M, W), dtype=torch.int64, device=dev)
            self.wc = torch.zeros((M, B), dtype=torch.float32, device=dev)
            self.ss = torch.zeros(W, dtype=torch.int64, device=dev)
            self.sc = torch.zeros(B, dtype=torch.float32, device=dev)

    ref, lazy = Side(False), Side(True)
    eta_prev = 0.0
    for t in range(steps):
        print("[%s deferred] step %d" % (workload, t), flush=True)
        for i in range(M):
            w.grad(t, i, device=dev, out=g[i, :d])
        for s in (ref, lazy):
            ef.ef_worker_step(s.plan, g, s.m, s.e, w.mu, eta_prev, w.eta, s.ws, s.wc)
            ef.ef_server_step(s.plan, M, s.ws, s.wc, s.te, eta_prev, w.eta, s.ss, s.sc)
            ef.ef_apply(s.plan, s.x, s.ss, s.sc, w.eta)
        torch.cuda.synchronize()
        for name in ("ws", "wc", "ss", "sc", "m", "x"):
            assert torch.equal(getattr(lazy, name), getattr(ref, name)), "step %d: %s differs" % (t, name)
        eta_prev = w.eta
    assert not torch.equal(lazy.e, ref.e) and not torch.equal(lazy.te, ref.te)
    ef.ef_flush(lazy.plan, lazy.e, lazy.te)
    torch.cuda.synchronize()
    assert torch.equal(lazy.e.view(torch.int32), ref.e.view(torch.int32)), "residuals after flush"
    assert torch.equal(lazy.te.view(torch.int32), ref.te.view(torch.int32)), "server residual after flush"
    for s in (ref, lazy):
        s.plan.close()


def test_deferred_mode_refuses_other_buffers():
    """While corrections are waiting the plan accepts only the buffers that wait for them."""
    offs = _offs(SIZES["aligned_large"])
    d = int(offs[-1])
    M = 2
    st = GpuState(offs, M)
    st.plan.tune(fuse_limit=3)
    st.plan.set_lazy(True)
    st.set_grads(np.random.default_rng(3).standard_normal((M, d)).astype(F))
    _raw_step(st, "sgdm", 0.9, 0.0, 0.1)
    other_e, other_te = st.e.clone(), st.te.clone()
    with pytest.raises(ef.EfError):
        ef.ef_worker_step(st.plan, st.g, st.m, other_e, 0.9, 0.1, 0.1, st.ws, st.wc)
    with pytest.raises(ef.EfError):
        ef.ef_worker_step(st.plan, st.g[1:], st.m[1:], st.e[1:], 0.9, 0.1, 0.1, st.ws[1:], st.wc[1:])   # worker 1 as worker 0
    with pytest.raises(ef.EfError):
        ef.ef_server_step(st.plan, M, st.ws, st.wc, other_te, 0.1, 0.1, st.ss, st.sc)
    with pytest.raises(ef.EfError):
        ef.ef_flush(st.plan, other_e, None)
    with pytest.raises(ef.EfError):
        ef.ef_flush(st.plan, None, other_te)
    ef.ef_flush(st.plan, st.e[:1], None)             # worker 0 only: worker 1 still waits
    with pytest.raises(ef.EfError):
        ef.ef_worker_step(st.plan, st.g, st.m, other_e, 0.9, 0.1, 0.1, st.ws, st.wc)
    ef.ef_flush(st.plan, st.e, st.te)
    torch.cuda.synchronize()
    other_e.copy_(st.e)
    other_te.copy_(st.te)
    ef.ef_worker_step(st.plan, st.g, st.m, other_e, 0.9, 0.1, 0.1, st.ws, st.wc)     # nothing waits: any buffer will do
    ef.ef_server_step(st.plan, M, st.ws, st.wc, other_te, 0.1, 0.1, st.ss, st.sc)
    torch.cuda.synchronize()
    st.plan.close()


@pytest.mark.parametrize("seed", range(24))
def test_deferred_equals_default_on_random_layouts(seed):
    """Random partitions (the generator of tests/test_random_layouts_gpu.py), random one-pass limit,
    worker count changing from step to step, flushes at random steps."""
    from tests.test_random_layouts_gpu import _random_sizes
    rng = np.random.default_rng(5000 + seed)
    offs = _offs(_random_sizes(rng))
    d = int(offs[-1])
    M = int(rng.integers(1, 6))
    route = ["one_pass", "direct"][seed % 2]
    fused = bool(rng.integers(0, 2))
    pad = int(rng.integers(0, 3))
    ref = GpuState(offs, M, route=route, fused=fused, pad=pad)
    lazy = GpuState(offs, M, route=route, fused=fused, pad=pad)
    if rng.integers(0, 3) > 0:
        lim = int(rng.integers(0, 8))
        ref.plan.tune(fuse_limit=lim)
        lazy.plan.tune(fuse_limit=lim)
    lazy.plan.set_lazy(True)
    variant = "sgd" if (seed % 3 == 0 and not fused) else "sgdm"
    eta_prev = 0.0
    for t in range(5):
        eta = float(rng.choice([0.4, 0.1, 0.05]))
        n = int(rng.integers(1, M + 1))
        g = (rng.standard_normal((M, d)) * 10.0 ** rng.uniform(-3, 1)).astype(F)
        g[rng.random((M, d)) < 0.1] = 0.0
        for st in (ref, lazy):
            st.set_grads(g)
            _raw_step(st, variant, 0.9, eta_prev, eta, n)
        _compare_outputs(lazy, ref, "seed %d step %d" % (seed, t), n)
        if rng.integers(0, 4) == 0:
            ef.ef_flush(lazy.plan, lazy.e, lazy.te)
            torch.cuda.synchronize()
            _same_bits(lazy.e, ref.e, "seed %d: residuals after a flush at step %d" % (seed, t))
        eta_prev = eta
    ef.ef_flush(lazy.plan, lazy.e, lazy.te)
    torch.cuda.synchronize()
    _same_bits(lazy.e, ref.e, "seed %d: residuals" % seed)
    _same_bits(lazy.te, ref.te, "seed %d: server residual" % seed)
    for st in (ref, lazy):
        st.plan.close()


@pytest.mark.parametrize("group", [0, 1, 2, 3, 5, 16, 256])
@pytest.mark.parametrize("layout", ["ragged_large", "one_large_block"])
def test_writing_out_in_step_changes_nothing(layout, group):
    """ef_plan_set_sync_group: whole tiles of blocks beyond the one-pass limit wait for their
    neighbours before they write (one workgroup per tile).  Any group size, default and deferred
    mode: the default mode against the oracle, the deferred mode against the default mode."""
    offs = _offs(SIZES[layout])
    d = int(offs[-1])
    M, mu = 3, 0.9
    rng = np.random.default_rng(77 + group)
    x0 = rng.standard_normal(d).astype(F)
    ref = GpuState(offs, M, x0=x0, route="direct")
    lazy = GpuState(offs, M, x0=x0, route="direct")
    for st in (ref, lazy):
        st.plan.tune(fuse_limit=3)
        st.plan.set_sync_group(group)
    lazy.plan.set_lazy(True)
    eta_prev = 0.0
    for t in range(3):
        eta = [0.4, 0.1, 0.1][t]
        g = rng.standard_normal((M, d)).astype(F)
        ref.set_grads(g)
        lazy.set_grads(g)
        synced_step(ref, mu, eta_prev, eta, None, "%s group %d step %d" % (layout, group, t))
        _raw_step(lazy, "sgdm", mu, eta_prev, eta)
        _compare_outputs(lazy, ref, "%s group %d step %d" % (layout, group, t))
        eta_prev = eta
    ef.ef_flush(lazy.plan, lazy.e, lazy.te)
    torch.cuda.synchronize()
    _same_bits(lazy.e, ref.e, "residuals after flush")
    with pytest.raises(ef.EfError):
        ref.plan.set_sync_group(257)
    with pytest.raises(ef.EfError):
        ref.plan.set_sync_group(-1)
    for st in (ref, lazy):
        st.plan.close()
