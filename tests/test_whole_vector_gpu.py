"""Whole-vector parity at the size of the benchmark workload: EVERY block of EVERY worker, the
server and the parameter update go through the oracle, not a sample.

The GPU runs the step in the launch configuration bench.py times (all M workers in one
ef_worker_step call, default plan settings).  Every stage of Algorithm 4 is block-separable, so
the oracle is run over the vector in chunks of whole blocks: the state before the step is kept in
device copies, and chunk by chunk the pre-step state goes to the host, the oracle steps it, and
its outputs are compared with the GPU's outputs on the same element range.  The workers of a
chunk are independent, so their oracle calls (each the plain single-thread code) run side by side
on the host's cores.

Bar, as in tests/parity_util.py: sign words and momentum bit-exact; scales within 1e-6 relative;
residuals and parameters bit-exact in every block whose scale is bit-equal and within 1e-6 of the
block's scale otherwise.  State-synchronised: each step's oracle starts from the GPU's state, and
the server and the update are fed the GPU's own payloads on both sides.
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
from tests.test_parity_full_gpu import whole_vector_props, whole_vector_props_server

ORACLE_THREADS = max(1, min(16, (os.cpu_count() or 1)))


def _chunks(offs, max_elems):
    """Ranges of whole blocks [b0, b1) of at most max_elems elements (a larger block stands alone)
    that start on a 64-element boundary, so that a chunk's sign words are whole words."""
    B = len(offs) - 1
    b0 = 0
    while b0 < B:
        b1 = b0 + 1
        while b1 < B and (offs[b1 + 1] - offs[b0] <= max_elems or offs[b1] % 64 != 0):
            b1 += 1
        yield b0, b1
        b0 = b1


def _words(t, lo, hi):
    """Sign words of elements [lo, hi) from an int64 tensor [..., W]; lo is a multiple of 64, and
    the bits past hi in the last word (they belong to the next chunk) are cleared, as the oracle
    clears the padding bits of the sub-vector it is given."""
    assert lo % 64 == 0
    a = t[..., lo // 64:(hi + 63) // 64].cpu().numpy().view(np.uint64).copy()
    if hi % 64:
        a[..., -1] &= np.uint64((1 << (hi % 64)) - 1)
    return a


def _host(t, lo, hi):
    return np.ascontiguousarray(t[..., lo:hi].cpu().numpy())


def _run_whole(w, steps, max_chunk_elems, props=True):
    dev = torch.device("cuda")
    d, B, M = w.d, w.B, w.M
    W = (d + 63) // 64
    offs = w.offsets
    plan = ef.ef_plan_create(offs, M)
    ds = (d + 3) // 4 * 4
    g = torch.zeros((M, ds), dtype=torch.float32, device=dev)
    m = torch.zeros((M, ds), dtype=torch.float32, device=dev)
    e = torch.zeros((M, ds), dtype=torch.float32, device=dev)
    te = torch.zeros(d, dtype=torch.float32, device=dev)
    x = torch.zeros(d, dtype=torch.float32, device=dev)
    ws = torch.zeros((M, W), dtype=torch.int64, device=dev)
    wc = torch.zeros((M, B), dtype=torch.float32, device=dev)
    ss = torch.zeros(W, dtype=torch.int64, device=dev)
    sc = torch.zeros(B, dtype=torch.float32, device=dev)
    eta_prev = 0.0
    loose = 0
    n_scales = 0
    for t in range(steps):
        eta = w.eta
        print("[%s whole vector] step %d: gradients, GPU step" % (w.name, t), flush=True)
        for i in range(M):
            w.grad(t, i, device=dev, out=g[i, :d])
        m_pre, e_pre, te_pre, x_pre = m.clone(), e.clone(), te.clone(), x.clone()
        ws.fill_(0x5555555555555555)
        wc.fill_(-7.0)
        ss.fill_(0x5555555555555555)
        sc.fill_(-7.0)
        ef.ef_worker_step(plan, g, m, e, w.mu, eta_prev, eta, ws, wc)
        ef.ef_server_step(plan, M, ws, wc, te, eta_prev, eta, ss, sc)
        ef.ef_apply(plan, x, ss, sc, eta)
        torch.cuda.synchronize()
        if props:
            print("[%s whole vector] step %d: properties of all %d workers and the server" % (w.name, t, M), flush=True)
            for i in range(M):
                whole_vector_props(w, "%s step %d worker %d" % (w.name, t, i), g[i, :d], m_pre[i, :d], e_pre[i, :d],
                                   bool(eta_prev), ws[i], wc[i], e[i, :d])
            whole_vector_props_server(w, "%s step %d server" % (w.name, t), ws, wc, te_pre, bool(eta_prev), ss, sc, te)
        for b0, b1 in _chunks(offs, max_chunk_elems):
            lo, hi = int(offs[b0]), int(offs[b1])
            sub = (offs[b0:b1 + 1] - lo).astype(np.int64)
            print("[%s whole vector] step %d: oracle on blocks %d..%d (%d elements x %d workers + server)"
                  % (w.name, t, b0, b1 - 1, hi - lo, M), flush=True)
            g_h, m_h, e_h = _host(g, lo, hi), _host(m_pre, lo, hi), _host(e_pre, lo, hi)
            ws_h, wc_h = _words(ws, lo, hi), _host(wc, b0, b1)
            m_out, e_out = _host(m, lo, hi), _host(e, lo, hi)

            def oracle_worker(i):
                return oracle.worker_step(g_h[i], m_h[i], e_h[i], sub, F(w.mu), F(eta_prev), F(eta))

            with ThreadPoolExecutor(max_workers=ORACLE_THREADS) as pool:
                refs = list(pool.map(oracle_worker, range(M)))
            for i, (s_ref, c_ref) in enumerate(refs):
                tag = "%s step %d worker %d blocks %d..%d" % (w.name, t, i, b0, b1 - 1)
                assert np.array_equal(ws_h[i], s_ref), "%s: %d sign words differ" % (tag, int((ws_h[i] != s_ref).sum()))
                assert np.array_equal(m_out[i].view(np.uint32), m_h[i].view(np.uint32)), tag + ": momentum differs"
                same = check_scales(wc_h[i], c_ref, tag)
                loose += int((~same).sum())
                n_scales += same.size
                check_vector(e_out[i], e_h[i], c_ref, same, sub, tag + " residual")
            del g_h, m_h, e_h, m_out, e_out, refs
            # server and update on the GPU's payloads
            te_h, x_h = _host(te_pre, lo, hi), _host(x_pre, lo, hi)
            ss_ref, sc_ref = oracle.server_step(np.ascontiguousarray(ws_h), np.ascontiguousarray(wc_h), te_h, sub,
                                                F(eta_prev), F(eta))
            tag = "%s step %d server blocks %d..%d" % (w.name, t, b0, b1 - 1)
            ss_h, sc_h = _words(ss, lo, hi), _host(sc, b0, b1)
            assert np.array_equal(ss_h, ss_ref), "%s: %d sign words differ" % (tag, int((ss_h != ss_ref).sum()))
            same = check_scales(sc_h, sc_ref, tag)
            loose += int((~same).sum())
            n_scales += same.size
            check_vector(_host(te, lo, hi), te_h, sc_ref, same, sub, tag + " residual")
            oracle.apply(x_h, np.ascontiguousarray(ss_h), np.ascontiguousarray(sc_h), sub, F(eta))
            assert np.array_equal(_host(x, lo, hi).view(np.uint32), x_h.view(np.uint32)), tag + ": parameters differ"
        del m_pre, e_pre, te_pre, x_pre
        eta_prev = eta
    print("[%s whole vector] %d of %d scales differed in the last bit" % (w.name, loose, n_scales), flush=True)
    plan.close()
    return loose, n_scales


@pytest.mark.gpu
def test_flat_2p28_every_block_of_every_worker():
    """The benchmark workload (2^28 elements in 256 blocks, 8 workers), two steps (the first from
    zero state, the second with momentum, residuals and the stepsize ratio in play): all
    256 blocks x 8 workers, the server and the update against the oracle, plus the whole-vector
    properties of every worker and the server."""
    w = wl.get("flat_2p28")
    loose, n = _run_whole(w, 2, 32 << 20)
    assert loose <= max(2, n // 1000)


def test_chunks_cover_every_block_once():
    """The chunking itself, on a layout with odd block boundaries (no GPU work)."""
    rng = np.random.default_rng(3)
    sizes = rng.integers(1, 300, 500)
    offs = np.concatenate([[0], np.cumsum(sizes)])
    seen = []
    for b0, b1 in _chunks(offs, 1000):
        assert b1 > b0 and offs[b0] % 64 == 0
        seen.extend(range(b0, b1))
    assert seen == list(range(len(sizes)))
