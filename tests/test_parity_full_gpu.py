"""GPU parity at the full sizes of the benchmark configurations, in the launch
configuration bench.py times (all M workers in one ef_worker_step call, default
plan settings).

Every stage of Algorithm 4 is block-separable (a block's outputs depend only on
that block's inputs), so the oracle is run on a sample of whole blocks: their
state is gathered from the GPU before the step, the oracle steps the
concatenation of those blocks, and its outputs are compared with the GPU's
outputs on the same blocks.  Bar as in tests/parity_util.py: sign bits and
momentum bit-exact, scales within 1e-6 relative, residuals and parameters
bit-exact where the block's scale is bit-equal and within 1e-6 of the scale
otherwise.  On top of the samples, properties that hold at any size are checked
over the whole vectors on the GPU (payload padding bits, Proposition 1 energy
identity, the reconstruction p = C(p) + e').
"""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import ef_workloads as wl
import oracle
import paper_1905_10936_amd as ef
from tests.parity_util import F, check_scales, check_vector

pytestmark = pytest.mark.gpu

# oracle calls of independent workers run side by side (each call is the plain single-thread code)
ORACLE_THREADS = max(1, min(8, (os.cpu_count() or 1)))


def _cat(t, offs, blocks):
    """Concatenate the element ranges of `blocks` from the last dim of t -> numpy."""
    parts = [t[..., int(offs[b]):int(offs[b + 1])] for b in blocks]
    return torch.cat(parts, dim=-1).cpu().numpy()


def _bits(words, offs, blocks):
    """Sign bits (0/1 uint8) of the element ranges of `blocks`; words: int64 tensor [..., W]."""
    out = []
    for b in blocks:
        a, e = int(offs[b]), int(offs[b + 1])
        w0, w1 = a // 64, (e + 63) // 64
        w = words[..., w0:w1].cpu().numpy().view(np.uint64)
        bits = np.unpackbits(w.view(np.uint8), axis=-1, bitorder="little")
        out.append(bits[..., a - 64 * w0:e - 64 * w0])
    return np.concatenate(out, axis=-1)


def _pack(bits):
    """uint8 bits [..., n] -> uint64 words [..., ceil(n/64)], LSB first."""
    n = bits.shape[-1]
    pad = (-n) % 64
    if pad:
        bits = np.concatenate([bits, np.zeros(bits.shape[:-1] + (pad,), np.uint8)], axis=-1)
    return np.ascontiguousarray(np.packbits(bits, axis=-1, bitorder="little")).view(np.uint64)


def _sample_blocks(w, rng, n_random, max_elems):
    sizes = np.diff(w.offsets)
    picks = {0, w.B - 1, int(np.argmax(sizes)), int(np.argmin(sizes))}
    # blocks around tile boundaries of the largest block, and some random ones
    picks.update(int(b) for b in rng.choice(w.B, size=min(n_random, w.B), replace=False))
    picks = sorted(picks)
    # respect the element budget, keeping the largest block if it fits
    out, tot = [], 0
    for b in sorted(picks, key=lambda b: -sizes[b]):
        if tot + sizes[b] <= max_elems:
            out.append(b)
            tot += int(sizes[b])
    return sorted(out)


def _decode_full(w, ws, wc):
    """Delta of a payload over the whole vector, fp64 on the device, and the per-element scale."""
    dev = ws.device
    sizes = torch.as_tensor(np.diff(w.offsets), device=dev)
    bid = torch.repeat_interleave(torch.arange(w.B, device=dev), sizes)
    scale_b = wc[bid].double()
    del bid
    idx = torch.arange(w.d, device=dev)
    bits = ((ws[idx // 64] >> (idx % 64)) & 1).bool()
    return bits, scale_b


def _props_from_p(w, tag, p_full, mag, ws, wc, e_new):
    """Properties of one compression step that hold at any size, over the whole vector, in fp64
    torch operations on the device (neither the library nor the oracle is involved): the payload's
    bits are the signs of p, its scales are the blocks' mean |p|, p = C(p) + e' elementwise, the
    Proposition 1 identity ||e'_b||^2 = ||p_b||^2 - ||p_b||_1^2 / d_b per block, and zero padding
    bits.  p_full: p evaluated in fp64 from the inputs; mag: the size of its fp32 terms (bounds the
    rounding of the fp32 evaluation); ws, wc, e_new: the step's outputs."""
    dev = p_full.device
    offs, d = w.offsets, w.d
    bits, scale_b = _decode_full(w, ws, wc)
    rec = torch.where(bits, scale_b, -scale_b) + e_new.double()
    assert bool(((rec - p_full).abs() <= 2e-6 * (mag + scale_b) + 1e-30).all()), tag + ": p = C(p) + e' violated"
    assert bool((bits == (p_full >= 0))[p_full.abs() > 1e-5 * (mag + scale_b)].all()), tag + ": a sign bit is not sign(p)"
    del rec, bits, scale_b
    # per-block sums as differences of fp64 running sums (index_add_ would serialise
    # millions of atomic adds on the one address of a large block)
    ends = torch.as_tensor(offs[1:] - 1, device=dev)

    def block_sums(v):
        cs = torch.cumsum(v, 0)[ends]
        return torch.diff(cs, prepend=torch.zeros(1, dtype=torch.float64, device=dev))

    l1, l2, en = block_sums(p_full.abs()), block_sums(p_full * p_full), block_sums(e_new.double() ** 2)
    db = torch.as_tensor(np.diff(offs), device=dev).double()
    tot = float(p_full.abs().sum())          # the running sums carry ~1e-16 * total of rounding
    assert bool(((en - (l2 - l1 * l1 / db)).abs() <= 1e-5 * l2 + 1e-12 * tot * tot + 1e-30).all()), \
        tag + ": Proposition 1 identity violated"
    assert bool(((wc.double() - l1 / db).abs() <= 2e-6 * (l1 / db) + 1e-12 * tot + 1e-30).all()), \
        tag + ": a scale is not the block's mean |p|"
    if d % 64:
        assert int(ws[-1].item()) >> (d % 64) == 0, tag + ": padding bits set"


def whole_vector_props(w, tag, g, m_pre, e_pre, has_prev, ws, wc, e_new):
    """_props_from_p for one worker's step.  g, m_pre, e_pre: the worker's gradient and its state
    before the step (constant stepsize, so the ratio of Algorithm 4 is 1 after the first step)."""
    p_full = w.mu * (w.mu * m_pre.double() + g.double()) + g.double()
    mag = w.mu * w.mu * m_pre.double().abs() + (1 + w.mu) * g.double().abs()   # size of the fp32 terms
    if has_prev:
        p_full += e_pre.double()
        mag += e_pre.double().abs()
    _props_from_p(w, tag, p_full, mag, ws, wc, e_new)


def whole_vector_props_server(w, tag, ws_all, wc_all, te_pre, has_prev, ss, sc, te_new):
    """_props_from_p for the server's step: p~ = (1/M) sum_i Delta_i + e~ (constant stepsize)."""
    M = ws_all.shape[0]
    p_full = torch.zeros(w.d, dtype=torch.float64, device=ss.device)
    mag = torch.zeros_like(p_full)
    for i in range(M):
        bits, scale_b = _decode_full(w, ws_all[i], wc_all[i])
        p_full += torch.where(bits, scale_b, -scale_b)
        mag += scale_b
        del bits, scale_b
    p_full /= M
    mag /= M
    mag *= 1 + M / 16.0          # M fp32 additions, each within half an ulp of a partial sum no larger than mag * M
    if has_prev:
        p_full += te_pre.double()
        mag += te_pre.double().abs()
    _props_from_p(w, tag, p_full, mag, ss, sc, te_new)


def _run_sampled(w, steps, blocks, workers=None, check_props=True, variant="sgdm", etas=None):
    """variant: "sgdm" Algorithm 4 through the unfused calls; "sgd" the momentum-free worker
    (Algorithm 3); "fused" one message per worker (Section 4.2); "wd" the parameter update with
    weight decay (Appendix A).  etas: stepsize per step (default: the workload's constant one)."""
    assert variant in ("sgdm", "sgd", "fused", "wd")
    assert not (check_props and (variant == "sgd" or etas))
    dev = torch.device("cuda")
    d, B, M = w.d, w.B, w.M
    W = (d + 63) // 64
    offs = w.offsets
    sizes = np.diff(offs)[blocks]
    sub_offs = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    workers = list(range(M)) if workers is None else workers
    plan = ef.ef_plan_create(offs, M)
    ds = (d + 3) // 4 * 4                  # row stride: the ABI wants a multiple of 4 elements
    g_rows = torch.zeros((M, ds), dtype=torch.float32, device=dev)
    m_rows = torch.zeros((M, ds), dtype=torch.float32, device=dev)
    e_rows = torch.zeros((M, ds), dtype=torch.float32, device=dev)
    g, m, e = g_rows[:, :d], m_rows[:, :d], e_rows[:, :d]
    te = torch.zeros(d, dtype=torch.float32, device=dev)
    x = torch.zeros(d, dtype=torch.float32, device=dev)
    ws = torch.zeros((M, W), dtype=torch.int64, device=dev)
    wc = torch.zeros((M, B), dtype=torch.float32, device=dev)
    ss = torch.zeros(W, dtype=torch.int64, device=dev)
    sc = torch.zeros(B, dtype=torch.float32, device=dev)
    bsel = torch.as_tensor(blocks, device=dev)
    if variant == "fused":
        pb, so = ef.ef_payload_bytes(plan), ef.ef_payload_scales_offset(plan)
        wmsg = torch.zeros((M, pb), dtype=torch.uint8, device=dev)
        smsg = torch.zeros(pb, dtype=torch.uint8, device=dev)
        # the unfused arrays become views of the messages: sign words first, scales at the stated offset
        ws = wmsg[:, :so].view(torch.int64)
        wc = wmsg[:, so:so + 4 * B].view(torch.float32)
        ss = smsg[:so].view(torch.int64)
        sc = smsg[so:so + 4 * B].view(torch.float32)
    if variant == "wd":
        lam = 5e-4
        mt = torch.zeros(d, dtype=torch.float32, device=dev)
        x.copy_(torch.randn(d, generator=torch.Generator(device=dev).manual_seed(7), device=dev))
    eta_prev = 0.0
    loose = 0
    for t in range(steps):
        eta = etas[t] if etas else w.eta
        print("[%s] step %d: generating gradients" % (w.name, t), flush=True)
        for i in range(M):
            w.grad(t, i, device=dev, out=g[i])
        # ---- state of the sampled blocks before the step
        g_s, m_s, e_s = _cat(g, offs, blocks), _cat(m, offs, blocks), _cat(e, offs, blocks)
        te_s, x_s = _cat(te, offs, blocks), _cat(x, offs, blocks)
        if check_props:
            m_pre, e_pre = m.clone(), e.clone()
        ws.fill_(0x5555555555555555)
        wc.fill_(-7.0)
        print("[%s/%s] step %d: worker step on the GPU" % (w.name, variant, t), flush=True)
        if variant == "sgd":
            ef.ef_worker_step_sgd(plan, g_rows, e_rows, eta_prev, eta, ws, wc)
        elif variant == "fused":
            ef.ef_worker_step_fused(plan, g_rows, m_rows, e_rows, w.mu, eta_prev, eta, wmsg)
        else:
            ef.ef_worker_step(plan, g_rows, m_rows, e_rows, w.mu, eta_prev, eta, ws, wc)
        torch.cuda.synchronize()
        print("[%s] step %d: oracle on %d sampled elements x %d workers" % (w.name, t, int(sub_offs[-1]), len(workers)),
              flush=True)
        wbits = _bits(ws, offs, blocks)
        wc_s = wc[:, bsel].cpu().numpy()
        m_out, e_out = _cat(m, offs, blocks), _cat(e, offs, blocks)

        def oracle_worker(i):
            mi, ei = np.ascontiguousarray(m_s[i]), np.ascontiguousarray(e_s[i])
            if variant == "sgd":
                s_ref, c_ref = oracle.worker_step_sgd(np.ascontiguousarray(g_s[i]), ei, sub_offs, F(eta_prev), F(eta))
            else:
                s_ref, c_ref = oracle.worker_step(np.ascontiguousarray(g_s[i]), mi, ei, sub_offs, F(w.mu),
                                                  F(eta_prev), F(eta))
            return mi, ei, s_ref, c_ref

        # the workers are independent: one oracle call each, side by side on the host's cores
        with ThreadPoolExecutor(max_workers=ORACLE_THREADS) as pool:
            refs = list(pool.map(oracle_worker, workers))
        for i, (mi, ei, s_ref, c_ref) in zip(workers, refs):
            tag = "%s step %d worker %d" % (w.name, t, i)
            ref_bits = np.unpackbits(s_ref.view(np.uint8), bitorder="little")[:wbits.shape[-1]]
            assert np.array_equal(wbits[i], ref_bits), "%s: %d sign bits differ" % (tag, (wbits[i] != ref_bits).sum())
            assert np.array_equal(m_out[i].view(np.uint32), mi.view(np.uint32)), tag + ": momentum differs"
            same = check_scales(wc_s[i], c_ref, tag)
            loose += int((~same).sum())
            check_vector(e_out[i], ei, c_ref, same, sub_offs, tag + " residual")
        if check_props:
            print("[%s] step %d: whole-vector properties, all %d workers" % (w.name, t, M), flush=True)
            for i in range(M):
                whole_vector_props(w, "%s step %d worker %d" % (w.name, t, i), g[i], m_pre[i], e_pre[i], bool(eta_prev),
                                   ws[i], wc[i], e[i])
            del m_pre, e_pre
        # ---- server on the GPU's worker payloads
        ss.fill_(0x5555555555555555)
        sc.fill_(-7.0)
        print("[%s] step %d: server step" % (w.name, t), flush=True)
        if check_props:
            te_pre = te.clone()
        if variant == "fused":
            ef.ef_server_step_fused(plan, M, wmsg, te, eta_prev, eta, smsg)
        else:
            ef.ef_server_step(plan, M, ws, wc, te, eta_prev, eta, ss, sc)
        torch.cuda.synchronize()
        if check_props:
            whole_vector_props_server(w, "%s step %d server" % (w.name, t), ws, wc, te_pre, bool(eta_prev), ss, sc, te)
            del te_pre
        te_ref = np.ascontiguousarray(te_s)
        ss_ref, sc_ref = oracle.server_step(_pack(wbits), np.ascontiguousarray(wc_s), te_ref, sub_offs, F(eta_prev),
                                            F(eta))
        sbits = _bits(ss, offs, blocks)
        ref_bits = np.unpackbits(ss_ref.view(np.uint8), bitorder="little")[:sbits.shape[-1]]
        tag = "%s step %d server" % (w.name, t)
        assert np.array_equal(sbits, ref_bits), "%s: %d sign bits differ" % (tag, (sbits != ref_bits).sum())
        sc_s = sc[bsel].cpu().numpy()
        same = check_scales(sc_s, sc_ref, tag)
        loose += int((~same).sum())
        check_vector(_cat(te, offs, blocks), te_ref, sc_ref, same, sub_offs, tag + " residual")
        # ---- apply
        x_ref = np.ascontiguousarray(x_s)
        if variant == "wd":
            mt_ref = np.ascontiguousarray(_cat(mt, offs, blocks))
            ef.ef_apply_wd(plan, x, mt, ss, sc, eta, w.mu, lam)
            oracle.apply_wd(x_ref, mt_ref, _pack(sbits), np.ascontiguousarray(sc_s), sub_offs, F(eta), F(w.mu), F(lam))
            torch.cuda.synchronize()
            assert np.array_equal(_cat(mt, offs, blocks).view(np.uint32), mt_ref.view(np.uint32)), \
                tag + ": decay momentum differs"
        else:
            if variant == "fused":
                ef.ef_apply_fused(plan, x, smsg, eta)
            else:
                ef.ef_apply(plan, x, ss, sc, eta)
            torch.cuda.synchronize()
            oracle.apply(x_ref, _pack(sbits), np.ascontiguousarray(sc_s), sub_offs, F(eta))
        assert np.array_equal(_cat(x, offs, blocks).view(np.uint32), x_ref.view(np.uint32)), tag + ": apply differs"
        eta_prev = eta
    return loose


def test_resnet50_like_full():
    """Configuration 2: all 161 blocks of every worker through the oracle."""
    w = wl.get("resnet50_like")
    _run_sampled(w, w.steps, list(range(w.B)))


def test_flat_2p28_sampled():
    """Configuration 3 (the benchmark workload): first, middle and last block of
    each of the 8 workers, momentum and residuals carried over 3 steps."""
    w = wl.get("flat_2p28")
    _run_sampled(w, 3, [0, 1, 127, 255], check_props=False)


def test_skewed_blocks_sampled():
    """Configuration 4: blocks of 1..64 elements next to 8 Mi-element blocks
    (larger than the one-pass limit), 5 % exact zeros."""
    w = wl.get("skewed_blocks")
    sizes = np.diff(w.offsets)
    big = [int(b) for b in np.nonzero(sizes > 64)[0]]
    rng = np.random.default_rng(4)
    # one big block with its small neighbours, plus runs of small blocks at random places
    blocks = set()
    blocks.update(range(max(0, big[1] - 300), min(w.B, big[1] + 300)))
    for s in rng.choice(w.B - 5000, size=6, replace=False):
        blocks.update(range(int(s), int(s) + 4000))
    blocks.update([0, w.B - 1])
    _run_sampled(w, w.steps, sorted(blocks))


def test_transformer_like_sampled():
    """Configuration 5: the 51 M-element embedding block (several times the
    one-pass limit), one layer's 12 tensors and the last block through the oracle for all
    16 workers, and the whole-vector properties of every worker and of the server."""
    w = wl.get("transformer_like")
    blocks = [0] + list(range(1, 13)) + [w.B - 1]
    _run_sampled(w, w.steps, blocks)


def test_flat_2p28_momentum_free_worker_sampled():
    """The benchmark workload through the Algorithm 3 worker, with a stepsize that rises and falls."""
    w = wl.get("flat_2p28")
    _run_sampled(w, 3, [0, 128, 255], check_props=False, variant="sgd", etas=[0.05, 0.2, 0.1])


def test_flat_2p28_fused_messages_sampled():
    """The benchmark workload with one contiguous message per worker (Section 4.2)."""
    w = wl.get("flat_2p28")
    _run_sampled(w, 2, [0, 77, 255], check_props=False, variant="fused")


def test_resnet50_like_weight_decay_full():
    """Configuration 2 with the Appendix A parameter update, all blocks, random initial parameters."""
    w = wl.get("resnet50_like")
    _run_sampled(w, 2, list(range(w.B)), check_props=False, variant="wd")


def test_beyond_2p31_elements_sampled():
    """More than 2^31 elements per worker (8.6 GB per fp32 row): every index past 2^31 has to be
    formed in 64 bits.  Sampled: the first block, the block that straddles element 2^31, the tiny
    blocks and the ragged last block behind it."""
    w = wl.get("beyond_2p31")
    assert w.d > (1 << 31)
    blocks = [0, 2046, 2047] + list(range(2048, w.B))
    _run_sampled(w, w.steps, blocks, check_props=False)


@pytest.mark.parametrize("persistent,variant", [(True, "sgdm"), (False, "sgdm"), (None, "sgd"), (True, "sgd"),
                                                (False, "sgd")])
def test_blocks_around_the_one_pass_limits(persistent, variant):
    """Blocks whose tile counts sit on both sides of every default one-pass limit (768 and 1024 tiles
    for the kernels with one workgroup per tile, 2304 for the persistent one) and of earlier ones
    (1152), some ending off the tile grid, with the plan's own limits: each block must take the
    route its size calls for and give the oracle's result either way.  All blocks go through the oracle.
    persistent None: the plan's own choice (the persistent kernel for this layout), under which the
    momentum-free worker still runs one workgroup per tile and needs that kernel's limit."""
    tiles = [767, 768, 769, 1023, 1024, 1025, 1151, 1152, 1153, 2303, 2304, 2305]
    rng = np.random.default_rng(12)
    sizes = [t * 4096 + int(rng.integers(-3, 4)) for t in tiles]
    order = rng.permutation(len(sizes))
    w = wl.Workload("limit_blocks", 9, [sizes[i] for i in order], M=2, steps=2, dist=("normal", 1.0))
    dev = torch.device("cuda")
    plan = ef.ef_plan_create(w.offsets, w.M)
    if persistent is None:
        assert plan.persistent
    else:
        plan.set_persistent(persistent)
    d, B, M = w.d, w.B, w.M
    W = (d + 63) // 64
    ds = (d + 3) // 4 * 4
    g = torch.zeros((M, ds), dtype=torch.float32, device=dev)
    m = torch.zeros((M, ds), dtype=torch.float32, device=dev)
    e = torch.zeros((M, ds), dtype=torch.float32, device=dev)
    ws = torch.zeros((M, W), dtype=torch.int64, device=dev)
    wc = torch.zeros((M, B), dtype=torch.float32, device=dev)
    eta_prev = 0.0
    for t in range(w.steps):
        for i in range(M):
            w.grad(t, i, device=dev, out=g[i, :d])
        g_h, m_h, e_h = (x[:, :d].cpu().numpy() for x in (g, m, e))
        print("[limit_blocks persistent=%s] step %d on the GPU (limit %d tiles)" % (persistent, t, plan.fuse_limit), flush=True)
        if variant == "sgd":
            ef.ef_worker_step_sgd(plan, g, e, eta_prev, w.eta, ws, wc)
        else:
            ef.ef_worker_step(plan, g, m, e, w.mu, eta_prev, w.eta, ws, wc)
        torch.cuda.synchronize()
        parked, late = plan.last_fallbacks()
        assert parked == 0 and late == 0, "run-time fallbacks on an idle GPU: %d tiles, %d blocks" % (parked, late)
        for i in range(M):
            print("[limit_blocks] step %d: oracle for worker %d" % (t, i), flush=True)
            mi, ei = np.ascontiguousarray(m_h[i]), np.ascontiguousarray(e_h[i])
            if variant == "sgd":
                s_ref, c_ref = oracle.worker_step_sgd(np.ascontiguousarray(g_h[i]), ei, w.offsets, F(eta_prev), F(w.eta))
            else:
                s_ref, c_ref = oracle.worker_step(np.ascontiguousarray(g_h[i]), mi, ei, w.offsets, F(w.mu), F(eta_prev),
                                                  F(w.eta))
            tag = "limit_blocks persistent=%s %s step %d worker %d" % (persistent, variant, t, i)
            assert np.array_equal(ws[i].cpu().numpy().view(np.uint64), s_ref), tag + ": sign words differ"
            assert np.array_equal(m[i, :d].cpu().numpy().view(np.uint32), mi.view(np.uint32)), tag + ": momentum differs"
            same = check_scales(wc[i].cpu().numpy(), c_ref, tag)
            check_vector(e[i, :d].cpu().numpy(), ei, c_ref, same, w.offsets, tag + " residual")
        eta_prev = w.eta
    plan.close()
