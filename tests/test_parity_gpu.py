"""GPU parity: the HIP path through the C ABI against the CPU oracle, element
by element on the same seeded inputs.

Bar: sign words, packed payloads and momentum bit-exact; scales within 1e-6
relative; residuals and parameters bit-exact wherever the block's scale is
bit-equal, else within 1e-6 of that scale (see tests/parity_util.py).  Sizes are
chosen so that the oracle finishes in seconds while the layouts still span
several 4096-element tiles, ragged tails and blocks from 1 element up.
"""
import zlib

import numpy as np
import pytest
import torch

import ef_workloads as wl
import oracle
import paper_1905_10936_amd as ef
from tests.parity_util import F, GpuState, check_scales, check_vector, synced_step, to_np

pytestmark = pytest.mark.gpu


def _offs(sizes):
    return np.concatenate([[0], np.cumsum(np.asarray(sizes, dtype=np.int64))])


def _layouts():
    rng = np.random.default_rng(42)
    tiny = np.clip(np.floor(np.exp(rng.uniform(0, np.log(65), 3000))), 1, 64).astype(np.int64)
    mixed = np.concatenate([tiny[:700], [20000], tiny[700:1500], [4096 * 3], tiny[1500:], [9000]])
    return {
        "one_elem": [1],
        "d3": [2, 1],
        "d63": [63],
        "d64": [64],
        "d65_two": [1, 64],
        "tile_minus1": [4095],
        "tile_exact": [4096],
        "tile_plus1": [4097],
        "single_block_5tiles_ragged": [5 * 4096 + 77],
        "aligned_tiles": [4096] * 6,
        "blocks_1000": [1000] * 37 + [123],
        "all_ones": [1] * 9000,
        "threes": [3] * 5000,                    # 1366 segments per tile: more than a quarter of the server's scale stage
        "tiny_blocks": tiny,
        "mixed_tiny_and_big": mixed,
        "two_big": [3 * 4096 + 5, 7 * 4096 - 5],
        "straddle_65": [4064, 65, 4063, 130, 12000],
    }


LAYOUTS = _layouts()


def _grads(rng, T, M, d, zeros=0.0, scale=1.0):
    g = (scale * rng.standard_normal((T, M, d))).astype(F)
    if zeros:
        g[rng.random((T, M, d)) < zeros] = 0.0
    return g


ROUTES = ["one_pass", "two_pass", "deferred", "mixed", "direct", "direct_deferred", "direct_mixed"]


@pytest.mark.parametrize("route", ROUTES)
@pytest.mark.parametrize("name", list(LAYOUTS))
def test_step_parity_small_layouts(name, route):
    """Every layout through every route by which the residual of a block that
    spans several tiles can be finished (in-kernel wait, second kernel for
    large blocks, deferral after a wait that gave up): same bits each way."""
    offs = _offs(LAYOUTS[name])
    d = int(offs[-1])
    M, T = 3, 3
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    g = _grads(rng, T, M, d, zeros=0.05)
    st = GpuState(offs, M, x0=rng.standard_normal(d).astype(F), route=route)
    etas = [0.1, 0.1, 0.05]
    eta_prev = 0.0
    stats = {}
    for t in range(T):
        st.set_grads(g[t])
        synced_step(st, 0.9, eta_prev, etas[t], stats, "%s step %d" % (name, t))
        eta_prev = etas[t]
    assert stats["scales_not_bit_equal"] == 0


@pytest.mark.parametrize("M", [1, 2, 5, 8, 16])
def test_server_worker_counts(M):
    offs = _offs(LAYOUTS["mixed_tiny_and_big"])
    d = int(offs[-1])
    rng = np.random.default_rng(M)
    st = GpuState(offs, M, route=ROUTES[M % len(ROUTES)])
    eta_prev = 0.0
    for t in range(2):
        st.set_grads(_grads(rng, 1, M, d)[0])
        synced_step(st, 0.9, eta_prev, 0.1, None, "M=%d step %d" % (M, t))
        eta_prev = 0.1


def test_strided_state_rows_and_mu_zero():
    """Row stride larger than d (padding untouched) and Algorithm 3 (mu = 0)."""
    offs = _offs([5000, 3, 4100, 1])
    d = int(offs[-1])
    rng = np.random.default_rng(5)
    st = GpuState(offs, 2, pad=3)
    eta_prev = 0.0
    for t, eta in enumerate([0.2, 0.05, 0.1]):
        st.set_grads(_grads(rng, 1, 2, d)[0])
        synced_step(st, 0.0, eta_prev, eta, None, "strided step %d" % t)
        eta_prev = eta


def test_zero_gradients_and_zero_blocks():
    """All-zero blocks: scale 0, every bit 1, residual 0 (zero-sign reading)."""
    offs = _offs([100, 5000, 64, 9000])
    d = int(offs[-1])
    st = GpuState(offs, 2)
    g = np.zeros((2, d), F)
    g[:, 100:5100] = np.random.default_rng(1).standard_normal((2, 5000)).astype(F)
    g[0, 200] = -0.0
    st.set_grads(g)
    synced_step(st, 0.9, 0.0, 0.1, None, "zeros")
    wc, ws = to_np(st.wc), to_np(st.ws)
    assert wc[0, 0] == 0 and wc[0, 2] == 0 and wc[0, 3] == 0
    bits = np.unpackbits(ws[0].view(np.uint8), bitorder="little")[:d]
    assert bits[:100].all() and bits[5100:].all()
    assert not to_np(st.e[:, :100]).any()


def test_resnet20_like_config_free_running():
    """Configuration 1 (ResNet-20-like layout, M = 2, 5 steps) step by step,
    plus a free-running oracle that is never re-synchronised: when every scale
    of every step is bit-equal, the two trajectories must be identical."""
    w = wl.get("resnet20_like")
    st = GpuState(w.offsets, w.M)
    d, M = w.d, w.M
    m = np.zeros((M, d), F)
    e = np.zeros((M, d), F)
    te = np.zeros(d, F)
    x = np.zeros(d, F)
    eta_prev = 0.0
    stats = {}
    for t in range(w.steps):
        g = np.stack([w.grad(t, i).numpy() for i in range(M)])
        st.set_grads(g)
        synced_step(st, w.mu, eta_prev, w.eta, stats, "resnet20 step %d" % t)
        oracle.step(g, m, e, te, x, w.offsets, F(w.mu), F(eta_prev), F(w.eta))
        eta_prev = w.eta
    if stats["scales_not_bit_equal"] == 0:
        h = st.host()
        assert np.array_equal(h["x"], x) and np.array_equal(h["te"], te)
        assert np.array_equal(h["m"], m) and np.array_equal(h["e"], e)


def test_repeat_call_is_deterministic():
    """Same inputs twice -> identical payload bits (no order-dependent sums)."""
    offs = _offs(LAYOUTS["mixed_tiny_and_big"])
    d = int(offs[-1])
    rng = np.random.default_rng(77)
    g = _grads(rng, 1, 4, d)[0]
    outs = []
    for _ in range(2):
        st = GpuState(offs, 4)
        st.set_grads(g)
        ef.ef_worker_step(st.plan, st.g, st.m, st.e, 0.9, 0.0, 0.1, st.ws, st.wc)
        ef.ef_server_step(st.plan, 4, st.ws, st.wc, st.te, 0.0, 0.1, st.ss, st.sc)
        torch.cuda.synchronize()
        outs.append([to_np(t).copy() for t in (st.ws, st.wc, st.ss, st.sc, st.e, st.te)])
    for a, b in zip(*outs):
        assert np.array_equal(a.view(np.uint8), b.view(np.uint8))


def test_abi_error_codes_on_device():
    offs = _offs([100, 200])
    st = GpuState(offs, 2)
    with pytest.raises(ef.EfError) as ei:
        ef.ef_worker_step(st.plan, st.g, st.m, st.e, 1.0, 0.0, 0.1, st.ws, st.wc)      # mu = 1
    assert ei.value.code == ef.EF_ERR_ARG
    with pytest.raises(ef.EfError) as ei:
        ef.ef_worker_step(st.plan, st.g, st.m, st.e, 0.9, 0.0, 0.0, st.ws, st.wc)      # eta = 0
    assert ei.value.code == ef.EF_ERR_ARG
    with pytest.raises(ef.EfError) as ei:
        ef.ef_server_step(st.plan, 3, torch.zeros(3 * st.W, dtype=torch.int64, device="cuda"),
                          torch.zeros(3 * st.B, device="cuda"), st.te, 0.0, 0.1, st.ss, st.sc)  # M > max
    assert ei.value.code == ef.EF_ERR_ARG
    with pytest.raises(ef.EfError) as ei:
        ef.ef_apply(st.plan, st.x, st.ss, st.sc, float("nan"))
    assert ei.value.code == ef.EF_ERR_ARG
    big = torch.zeros(st.d + 8, device="cuda")
    with pytest.raises(ef.EfError) as ei:
        ef.ef_apply(st.plan, big[1:st.d + 1], st.ss, st.sc, 0.1)                          # misaligned
    assert ei.value.code == ef.EF_ERR_ALIGN


def test_outputs_that_overlap_inputs_are_refused():
    """In-place updating is the contract for mom, err, server_err and params only: a payload
    buffer that shares bytes with the state or with the incoming payloads is an error, and
    nothing is enqueued."""
    offs = _offs([100, 200, 4096 * 3])
    st = GpuState(offs, 2)
    d, W, B = st.d, st.W, st.B
    before = to_np(st.e).copy()
    as_words = st.e.view(torch.int64).view(-1)      # sign words that alias the residual buffer
    with pytest.raises(ef.EfError) as ei:
        ef.ef_worker_step(st.plan, st.g, st.m, st.e, 0.9, 0.0, 0.1, as_words[:2 * W], st.wc)
    assert ei.value.code == ef.EF_ERR_ARG
    with pytest.raises(ef.EfError) as ei:           # scales inside the gradient buffer
        ef.ef_worker_step(st.plan, st.g, st.m, st.e, 0.9, 0.0, 0.1, st.ws, st.g.view(-1)[:2 * B])
    assert ei.value.code == ef.EF_ERR_ARG
    with pytest.raises(ef.EfError) as ei:           # momentum and residual rows that interleave
        ef.ef_worker_step(st.plan, st.g, st.m, st.m, 0.9, 0.0, 0.1, st.ws, st.wc)
    assert ei.value.code == ef.EF_ERR_ARG
    with pytest.raises(ef.EfError) as ei:           # server output inside the server residual
        ef.ef_server_step(st.plan, 2, st.ws, st.wc, st.te, 0.0, 0.1, st.te.view(torch.int64)[:W], st.sc)
    assert ei.value.code == ef.EF_ERR_ARG
    with pytest.raises(ef.EfError) as ei:           # server output on top of a worker's payload
        ef.ef_server_step(st.plan, 2, st.ws, st.wc, st.te, 0.0, 0.1, st.ws[1], st.sc)
    assert ei.value.code == ef.EF_ERR_ARG
    torch.cuda.synchronize()
    assert np.array_equal(to_np(st.e), before)


def test_one_worker_needs_no_stride():
    """A single vector whose length is not a multiple of 4: with n_workers = 1 the row stride is
    never used, so any value passes, and the step matches the oracle."""
    offs = _offs([4099, 7, 4096 + 1])
    st = GpuState(offs, 1)
    d = st.d
    assert d % 4 != 0
    rng = np.random.default_rng(5)
    g = rng.standard_normal(d).astype(F)
    gt, mt, et = (torch.zeros(d, dtype=torch.float32, device="cuda") for _ in range(3))
    gt.copy_(torch.as_tensor(g))
    ef.ef_worker_step(st.plan, gt, mt, et, 0.9, 0.0, 0.1, st.ws, st.wc)         # stride = d, not a multiple of 4
    torch.cuda.synchronize()
    m_ref, e_ref = np.zeros(d, F), np.zeros(d, F)
    s_ref, c_ref = oracle.worker_step(g, m_ref, e_ref, offs, F(0.9), F(0.0), F(0.1))
    assert np.array_equal(to_np(st.ws)[0], s_ref)
    assert np.array_equal(to_np(mt).view(np.uint32), m_ref.view(np.uint32))
    same = check_scales(to_np(st.wc)[0], c_ref, "single vector")
    check_vector(to_np(et), e_ref, c_ref, same, offs, "single vector residual")


def test_many_steps_with_changing_worker_count_and_stepsize():
    """Twelve iterations on one plan, the number of workers per call varying
    (the per-set tags and the call epoch must stay consistent), the stepsize
    going up and down (Section 3.1: the residual is rescaled by eta_{t-1}/eta_t)."""
    offs = _offs([3 * 4096 + 17, 40, 4096, 9 * 4096 - 57, 2, 6000])
    d = int(offs[-1])
    rng = np.random.default_rng(12)
    st = GpuState(offs, 4, x0=rng.standard_normal(d).astype(F))
    etas = [0.02, 0.05, 0.1, 0.1, 0.2, 0.1, 0.05, 0.05, 0.025, 0.0125, 0.1, 0.1]
    eta_prev = 0.0
    for t, eta in enumerate(etas):
        st.set_grads(_grads(rng, 1, 4, d, zeros=0.02)[0])
        if t % 3 == 1:
            # a call with fewer workers in between: its outputs are checked against the oracle directly
            n = 1 + t % 2
            g, m, e = st.g[:n].clone(), st.m[:n].clone(), st.e[:n].clone()
            ws = torch.zeros((n, st.W), dtype=torch.int64, device="cuda")
            wc = torch.zeros((n, st.B), dtype=torch.float32, device="cuda")
            hm, he = to_np(m[:, :d]).copy(), to_np(e[:, :d]).copy()
            ef.ef_worker_step(st.plan, g, m, e, 0.9, eta_prev, eta, ws, wc)
            torch.cuda.synchronize()
            for i in range(n):
                s_ref, c_ref = oracle.worker_step(to_np(g[i, :d]).copy(), hm[i], he[i], offs, F(0.9), F(eta_prev), F(eta))
                assert np.array_equal(to_np(ws[i]), s_ref)
                assert np.array_equal(to_np(wc[i]).view(np.uint32), c_ref.view(np.uint32))
                assert np.array_equal(to_np(e[i, :d]).view(np.uint32), he[i].view(np.uint32))
        synced_step(st, 0.9, eta_prev, eta, None, "long run step %d" % t)
        eta_prev = eta


def test_sixty_four_workers():
    """EF_MAX_WORKERS workers in one call."""
    offs = _offs([5000, 100, 8192, 77])
    d = int(offs[-1])
    rng = np.random.default_rng(64)
    st = GpuState(offs, 64)
    st.set_grads(_grads(rng, 1, 64, d)[0])
    synced_step(st, 0.9, 0.0, 0.1, None, "64 workers")


def test_calls_on_a_side_stream():
    """The ABI takes the stream to enqueue on; results do not depend on it."""
    offs = _offs(LAYOUTS["mixed_tiny_and_big"])
    d = int(offs[-1])
    rng = np.random.default_rng(5)
    g = _grads(rng, 1, 2, d)[0]
    outs = []
    for use_side in (False, True):
        st = GpuState(offs, 2)
        st.set_grads(g)
        torch.cuda.synchronize()
        stream = torch.cuda.Stream() if use_side else torch.cuda.current_stream()
        with torch.cuda.stream(stream):
            ef.ef_worker_step(st.plan, st.g, st.m, st.e, 0.9, 0.0, 0.1, st.ws, st.wc, stream=stream)
            ef.ef_server_step(st.plan, 2, st.ws, st.wc, st.te, 0.0, 0.1, st.ss, st.sc, stream=stream)
            ef.ef_apply(st.plan, st.x, st.ss, st.sc, 0.1, stream=stream)
        stream.synchronize()
        outs.append([to_np(t).copy() for t in (st.ws, st.wc, st.ss, st.sc, st.m, st.e, st.te, st.x)])
    for a, b in zip(*outs):
        assert np.array_equal(a.view(np.uint8), b.view(np.uint8))


def test_fallback_counters():
    """The diagnostic counters: none on the one-pass route, every waiting tile
    when the spin budget is zero."""
    offs = _offs([4096 * 40, 4096 * 24 + 100, 50])
    d = int(offs[-1])
    rng = np.random.default_rng(8)
    for route, expect_parked in (("direct", False), ("direct_deferred", True), ("one_pass", False), ("deferred", True)):
        st = GpuState(offs, 2, route=route)
        st.set_grads(_grads(rng, 1, 2, d)[0])
        ef.ef_worker_step(st.plan, st.g, st.m, st.e, 0.9, 0.0, 0.1, st.ws, st.wc)
        parked, late = st.plan.last_fallbacks()
        if expect_parked:
            assert parked >= 2 * (40 + 23) and late == 4     # every full single-block tile, both big blocks x 2 workers
        else:
            assert parked == 0 and late == 0


def test_two_plans_on_two_streams_at_once():
    """Calls on different plans may overlap on the device.  Their kernels compete
    for the same compute units, and every wait in them is bounded, so at worst
    some tiles take the two-pass route: the results must be those of the same
    calls made one after the other."""
    offs_a = _offs(LAYOUTS["two_big"])
    offs_b = _offs([6 * 4096] * 40)
    rng = np.random.default_rng(8)
    outs = []
    for overlap in (False, True):
        sa, sb = GpuState(offs_a, 4, route="direct"), GpuState(offs_b, 8, route="one_pass")
        rng_run = np.random.default_rng(9)
        streams = (torch.cuda.Stream(), torch.cuda.Stream())
        eta_prev = 0.0
        for t in range(4):
            for st in (sa, sb):
                st.set_grads(rng_run.standard_normal((st.M, st.d)).astype(F))
            torch.cuda.synchronize()
            for st, stream in ((sa, streams[0]), (sb, streams[1])):
                with torch.cuda.stream(stream):
                    ef.ef_worker_step(st.plan, st.g, st.m, st.e, 0.9, eta_prev, 0.1, st.ws, st.wc, stream=stream)
                    ef.ef_server_step(st.plan, st.M, st.ws, st.wc, st.te, eta_prev, 0.1, st.ss, st.sc, stream=stream)
                    ef.ef_apply(st.plan, st.x, st.ss, st.sc, 0.1, stream=stream)
                if not overlap:
                    stream.synchronize()
            torch.cuda.synchronize()
            eta_prev = 0.1
        outs.append([to_np(t).copy() for st in (sa, sb) for t in (st.ws, st.wc, st.ss, st.sc, st.m, st.e, st.te, st.x)])
        sa.plan.close()
        sb.plan.close()
    for u, v in zip(*outs):
        assert np.array_equal(u.view(np.uint8), v.view(np.uint8))


def test_kernel_choice_follows_the_block_sizes():
    """Plan creation picks the worker kernel from the layout (include/ef.h, ef_plan_set_persistent):
    one workgroup per tile where the blocks are mostly up to 512 tiles or the layout is small, the
    persistent kernel where they are larger or where only it finishes them in one pass."""
    import ef_workloads as wl
    expect = {"flat_2p28": False, "odd_tiles": False, "resnet50_like": False, "resnet20_like": False,
              "transformer_like": True, "skewed_blocks": True}
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    for name, persistent in expect.items():
        w = wl.get(name)
        plan = ef.ef_plan_create(w.offsets, w.M)
        assert plan.persistent == persistent, name
        # half of what the kernel's workgroups hold at once: resident workgroups per compute unit
        # (1 to 8 of 256 threads) x compute units, x 6 tiles each in the persistent kernel
        per_cu, rest = divmod(2 * plan.fuse_limit, cus * (6 if persistent else 1))
        assert rest == 0 and 1 <= per_cu <= 8, (name, plan.fuse_limit)
        if cus == 256:
            assert plan.fuse_limit == (2304 if persistent else 1024), name     # 3 and 8 workgroups per unit
        plan.set_lazy(True)                  # deferred mode: one workgroup per tile unless asked otherwise
        assert not plan.persistent and plan.fuse_limit == 64, name
        plan.set_persistent(True)
        assert plan.persistent and plan.fuse_limit == 0, name
        plan.set_lazy(False)
        plan.set_persistent(None)
        assert plan.persistent == persistent, name
        plan.close()


@pytest.mark.parametrize("route", ["one_pass", "direct", "two_pass"])
def test_subnormal_values_are_kept(route):
    """Gradients in and around the subnormal range of fp32 (below 1.2e-38): Algorithm 4's products,
    sums and sign decisions must treat them as IEEE-754 does on the host, nothing flushed to zero
    (a flushed negative subnormal would flip its sign bit to +1)."""
    offs = _offs(LAYOUTS["mixed_tiny_and_big"])
    d = int(offs[-1])
    M = 3
    rng = np.random.default_rng(4141)
    st = GpuState(offs, M, x0=(rng.standard_normal(d) * 1e-39).astype(F), route=route)
    eta_prev = 0.0
    for t in range(3):
        scale = 10.0 ** rng.uniform(-44, -37, size=(M, d))
        g = (rng.standard_normal((M, d)) * scale).astype(F)
        g[rng.random((M, d)) < 0.05] = 0.0
        assert (np.abs(g[g != 0]) < 1.1754944e-38).mean() > 0.3          # many subnormal inputs
        st.set_grads(g)
        synced_step(st, 0.9, eta_prev, 0.1, None, "subnormal %s step %d" % (route, t))
        eta_prev = 0.1
    st.plan.close()


@pytest.mark.parametrize("route", ["one_pass", "direct", "two_pass"])
def test_gpu_scales_against_the_exactly_rounded_sum(route):
    """The GPU's fixed-tree fp64 sums checked against the exactly rounded L1 norm (math.fsum), not
    against the oracle: with mu = 0 and a zero residual p is the gradient itself, so the scale of
    block b is ||g_b||_1 / d_b (Section 3.2).  It must be the correctly rounded fp32 value or its
    neighbour, and the correctly rounded one away from rounding boundaries."""
    import math
    rng = np.random.default_rng(31337)
    sizes = [100003, 1 << 20, 5, 250000, 4096, 3 * 4096 + 1]
    offs = _offs(sizes)
    d = int(offs[-1])
    st = GpuState(offs, 1, route=route)
    g = (rng.standard_normal((1, d)) * 10.0 ** rng.uniform(-6, 3, (1, d))).astype(F)
    st.set_grads(g)
    ef.ef_worker_step(st.plan, st.g, st.m, st.e, 0.0, 0.0, 0.1, st.ws, st.wc)
    torch.cuda.synchronize()
    scales = to_np(st.wc)[0]
    for b, n in enumerate(sizes):
        seg = np.abs(g[0, offs[b]:offs[b + 1]].astype(np.float64))
        exact = math.fsum(seg.tolist()) / n
        want = np.float32(exact)
        ulp = float(np.spacing(want))
        assert abs(float(scales[b]) - float(want)) <= ulp, (b, scales[b], want)
        lo, hi = float(want) - ulp / 2, float(want) + ulp / 2
        if min(exact - lo, hi - exact) > abs(exact) * n * 2.0 ** -52:
            assert scales[b] == want, (b, scales[b], want)
    st.plan.close()
