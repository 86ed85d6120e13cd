"""The deferred-correction mode (ef_plan_set_lazy) against the ORACLE, directly, at full size.

In that mode the residual of a block larger than the one-pass limit is not written by the call
that computes it: the buffer keeps p, and e = p - Delta is formed when the next call loads the
buffer.  So the check cannot be state-synchronised step by step (the state is not there between
calls); instead the oracle runs FREE from zero state over the same gradients for all the steps,
the GPU runs the same steps in the deferred mode without any flush in between, and compared are

  * every step's payloads (worker and server sign words bit-exact, scales within 1e-6 relative;
    the second step's payload already depends on the correction applied on the fly),
  * after the last step and ef_flush: momentum bit-exact, worker residuals, server residual and
    parameters to the bar of tests/parity_util.py.

A scale that differs from the oracle's in its last bit (fp64 sums in another order; probability
about 1e-5 per block and step) moves the residual by an ulp and may flip a near-zero sign one step
later; the oracle cannot be re-synchronised here, so such a worker is only followed for its
scales from then on, and the test requires that this happens at most once.

Workloads: the B = 1 layout (one 2^28-element block, the non-block compressor of Eq. (1): all of
it takes the deferred route) with all 8 workers over the whole vector, and the transformer-like
layout on a sample of whole blocks (the 51 M-element embedding, one layer, the last tensor) with
all 16 workers.
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
from tests.test_parity_full_gpu import _bits, _cat, _pack

pytestmark = pytest.mark.gpu

THREADS = max(1, min(8, (os.cpu_count() or 1)))


def _run(w, blocks, steps):
    dev = torch.device("cuda")
    d, B, M = w.d, w.B, w.M
    W = (d + 63) // 64
    offs = w.offsets
    sizes = np.diff(offs)[blocks]
    sub = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    n = int(sub[-1])
    bsel = torch.as_tensor(blocks, device=dev)
    plan = ef.ef_plan_create(offs, M)
    plan.set_lazy(True)
    limit = plan.fuse_limit
    big = [k for k, b in enumerate(blocks) if (offs[b + 1] - 1) // 4096 - offs[b] // 4096 + 1 > limit]
    assert big, "the sample must hold a block that takes the deferred route"
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
    # per step, on the host: the sampled gradients and the GPU's payloads on the sample
    g_s, wbits, wc_s, sbits, sc_s = [], [], [], [], []
    eta_prev = 0.0
    for t in range(steps):
        print("[%s deferred vs oracle] step %d on the GPU" % (w.name, t), flush=True)
        for i in range(M):
            w.grad(t, i, device=dev, out=g[i, :d])
        g_s.append(_cat(g[:, :d], offs, blocks))
        ef.ef_worker_step(plan, g, m, e, w.mu, eta_prev, w.eta, ws, wc)
        ef.ef_server_step(plan, M, ws, wc, te, eta_prev, w.eta, ss, sc)
        ef.ef_apply(plan, x, ss, sc, w.eta)
        torch.cuda.synchronize()
        wbits.append(_bits(ws, offs, blocks))
        wc_s.append(wc[:, bsel].cpu().numpy())
        sbits.append(_bits(ss, offs, blocks))
        sc_s.append(sc[bsel].cpu().numpy())
        eta_prev = w.eta
    # the mode really was in effect: before the flush a large block's buffer holds p, not e
    k = big[0]
    before = e[0, int(offs[blocks[k]]):int(offs[blocks[k] + 1])].clone()
    ef.ef_flush(plan, e, te)
    torch.cuda.synchronize()
    assert not torch.equal(before, e[0, int(offs[blocks[k]]):int(offs[blocks[k] + 1])]), "nothing was deferred"
    del before
    m_g, e_g = _cat(m[:, :d], offs, blocks), _cat(e[:, :d], offs, blocks)
    te_g, x_g = _cat(te, offs, blocks), _cat(x, offs, blocks)

    def oracle_worker(i):
        """Free run of worker i over all steps; returns (worker still exactly followed, loose scales, m, e, scales)."""
        mi, ei = np.zeros(n, F), np.zeros(n, F)
        followed, loose, ep = True, 0, 0.0
        c_ref = None
        for t in range(steps):
            s_ref, c_ref = oracle.worker_step(np.ascontiguousarray(g_s[t][i]), mi, ei, sub, F(w.mu), F(ep), F(w.eta))
            tag = "%s deferred step %d worker %d" % (w.name, t, i)
            if followed:
                ref_bits = np.unpackbits(s_ref.view(np.uint8), bitorder="little")[:n]
                assert np.array_equal(wbits[t][i], ref_bits), "%s: %d sign bits differ" % (tag, int((wbits[t][i] != ref_bits).sum()))
                same = check_scales(wc_s[t][i], c_ref, tag)
                if not same.all():
                    loose += int((~same).sum())
                    followed = False        # the two trajectories may part by an ulp from here on
            ep = w.eta
        return followed, loose, mi, ei, c_ref

    print("[%s deferred vs oracle] oracle: %d workers x %d steps on %d elements" % (w.name, M, steps, n), flush=True)
    unfollowed = 0
    with ThreadPoolExecutor(max_workers=THREADS) as pool:
        for i, (followed, loose, mi, ei, c_ref) in enumerate(pool.map(oracle_worker, range(M))):
            tag = "%s deferred worker %d after %d steps" % (w.name, i, steps)
            if not followed:
                unfollowed += 1
                continue
            assert np.array_equal(m_g[i].view(np.uint32), mi.view(np.uint32)), tag + ": momentum differs"
            same = np.ones(len(blocks), dtype=bool)
            check_vector(e_g[i], ei, c_ref, same, sub, tag + " residual")
    assert unfollowed <= 1, "%d workers had a scale that differed in its last bit" % unfollowed
    # server and update: free run on the GPU's worker payloads
    te_o, x_o = np.zeros(n, F), np.zeros(n, F)
    ep, followed = 0.0, True
    for t in range(steps):
        ss_ref, sc_ref = oracle.server_step(_pack(wbits[t]), np.ascontiguousarray(wc_s[t]), te_o, sub, F(ep), F(w.eta))
        tag = "%s deferred step %d server" % (w.name, t)
        if followed:
            ref_bits = np.unpackbits(ss_ref.view(np.uint8), bitorder="little")[:n]
            assert np.array_equal(sbits[t], ref_bits), "%s: %d sign bits differ" % (tag, int((sbits[t] != ref_bits).sum()))
            same = check_scales(sc_s[t], sc_ref, tag)
            followed = bool(same.all())
            # the update is fed the GPU's payload on both sides
            oracle.apply(x_o, _pack(sbits[t]), np.ascontiguousarray(sc_s[t]), sub, F(w.eta))
        ep = w.eta
    if followed:
        check_vector(te_g, te_o, sc_ref, np.ones(len(blocks), dtype=bool), sub, "%s deferred server residual" % w.name)
        assert np.array_equal(x_g.view(np.uint32), x_o.view(np.uint32)), "%s deferred: parameters differ" % w.name
    plan.close()


def test_one_block_2p28_deferred_mode_against_the_oracle():
    """B = 1, d = 2^28, M = 8: the whole vector of every worker, two steps without a flush between them."""
    w = wl.get("one_block_2p28")
    _run(w, [0], 2)


def test_transformer_like_deferred_mode_against_the_oracle():
    """The 51 M-element embedding (deferred), one layer's 12 tensors (768- and 1024-tile weights:
    deferred too under this mode's 64-tile limit) and the last tensor, all 16 workers, two steps."""
    w = wl.get("transformer_like")
    _run(w, [0] + list(range(1, 13)) + [w.B - 1], 2)
