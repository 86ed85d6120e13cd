"""Helpers of the GPU parity tests: run one iteration of Algorithm 4 through
the C ABI and through the oracle from the same state and compare.

Bar (stated in the tests that use this): sign words and momentum bit-exact;
scales within 1e-6 relative; residuals and parameters bit-exact in every block
whose scale is bit-equal and within 1e-6 of the block's scale otherwise (a
scale that differs in its last bit moves p - (+-s) by one ulp of s).
"""
import numpy as np
import torch

import oracle
import paper_1905_10936_amd as ef

F = np.float32
REL = 1e-6


def to_np(t):
    a = t.detach().cpu().numpy()
    return a.view(np.uint64) if a.dtype == np.int64 else a


def block_ids(offs):
    return np.repeat(np.arange(len(offs) - 1), np.diff(offs))


def check_scales(gpu, cpu, what):
    """Returns boolean array: which scales are bit-equal.  All within REL."""
    gpu, cpu = np.asarray(gpu), np.asarray(cpu)
    same = gpu.view(np.uint32) == cpu.view(np.uint32)
    bad = np.abs(gpu.astype(np.float64) - cpu) > REL * np.abs(cpu.astype(np.float64))
    assert not bad.any(), "%s: %d scales off by more than 1e-6 relative, first block %d: gpu %r cpu %r" % (
        what, bad.sum(), np.argmax(bad), gpu.ravel()[np.argmax(bad)], cpu.ravel()[np.argmax(bad)])
    return same


def check_vector(gpu, cpu, scales_cpu, same_scale, offs, what):
    """Elementwise check of a residual/parameter vector."""
    gpu, cpu = np.asarray(gpu), np.asarray(cpu)
    neq = gpu.view(np.uint32) != cpu.view(np.uint32)
    # -0.0 and +0.0 are the same value; compare values where the bits differ
    neq &= ~((gpu == 0) & (cpu == 0))
    if not neq.any():
        return 0
    bid = block_ids(offs)
    exact_required = same_scale[bid]
    wrong = neq & exact_required
    assert not wrong.any(), "%s: %d elements differ in blocks whose scale is bit-equal; first j=%d gpu %r cpu %r" % (
        what, wrong.sum(), np.argmax(wrong), gpu[np.argmax(wrong)], cpu[np.argmax(wrong)])
    tol = REL * np.abs(scales_cpu.astype(np.float64))[bid] * 1.01 + 1e-45
    off = neq & (np.abs(gpu.astype(np.float64) - cpu) > tol)
    assert not off.any(), "%s: %d elements beyond 1e-6 of their block scale" % (what, off.sum())
    return int(neq.sum())


class GpuState:
    """Device tensors of M workers + server + parameters for one layout."""

    def __init__(self, offs, M, device="cuda", x0=None, pad=0, route="one_pass", fused=False):
        self.offs = np.asarray(offs, dtype=np.int64)
        self.d = int(self.offs[-1])
        self.B = self.offs.size - 1
        self.M = M
        self.W = (self.d + 63) // 64
        self.plan = ef.ef_plan_create(self.offs, max(M, 1))
        # which way e <- p - Delta is finished for blocks that span several tiles
        # the two kernels for single-block tiles: persistent and pipelined, or one workgroup per tile
        self.plan.set_persistent(route not in ("direct", "direct_deferred", "direct_mixed"))
        if route == "two_pass":          # every such block through the second kernel
            self.plan.tune(fuse_limit=0)
        elif route in ("deferred", "direct_deferred"):   # every wait gives up at once -> deferral list
            self.plan.tune(spin_limit=0)
        elif route in ("mixed", "direct_mixed"):         # blocks of <= 2 tiles in one pass, larger ones in two
            self.plan.tune(fuse_limit=2)
        elif route == "direct":
            pass
        elif route != "one_pass":
            raise ValueError(route)
        ds = ((self.d + 3) // 4) * 4 + 4 * pad           # row stride, multiple of 4
        self.stride = ds
        dev = torch.device(device)
        self.g = torch.zeros((M, ds), dtype=torch.float32, device=dev)
        self.m = torch.zeros((M, ds), dtype=torch.float32, device=dev)
        self.e = torch.zeros((M, ds), dtype=torch.float32, device=dev)
        self.te = torch.zeros(self.d, dtype=torch.float32, device=dev)
        self.x = torch.zeros(self.d, dtype=torch.float32, device=dev)
        if x0 is not None:
            self.x.copy_(torch.as_tensor(x0))
        self.ws = torch.zeros((M, self.W), dtype=torch.int64, device=dev)
        self.wc = torch.zeros((M, self.B), dtype=torch.float32, device=dev)
        self.ss = torch.zeros(self.W, dtype=torch.int64, device=dev)
        self.sc = torch.zeros(self.B, dtype=torch.float32, device=dev)
        # one contiguous message per worker (sign words, then scales) instead of two arrays
        self.fused = fused
        if fused:
            self.pb = ef.ef_payload_bytes(self.plan)
            self.so = ef.ef_payload_scales_offset(self.plan)
            assert self.so == 8 * self.W and self.pb % 16 == 0 and 0 <= self.pb - (self.so + 4 * self.B) < 16
            self.wmsg = torch.zeros((M, self.pb), dtype=torch.uint8, device=dev)
            self.smsg = torch.zeros(self.pb, dtype=torch.uint8, device=dev)

    def split(self, msg):
        """Host copy of fused messages [n][pb] -> (sign words [n][W], scales [n][B], padding bytes)."""
        a = to_np(msg).reshape(-1, self.pb)
        signs = np.ascontiguousarray(a[:, :self.so]).view(np.uint64)
        scales = np.ascontiguousarray(a[:, self.so:self.so + 4 * self.B]).view(np.float32)
        return signs, scales, a[:, self.so + 4 * self.B:]

    def set_grads(self, g):
        self.g[:, :self.d].copy_(torch.as_tensor(g))

    def host(self):
        d = self.d
        return dict(g=to_np(self.g[:, :d]).copy(), m=to_np(self.m[:, :d]).copy(), e=to_np(self.e[:, :d]).copy(),
                    te=to_np(self.te).copy(), x=to_np(self.x).copy())


def synced_step(st, mu, eta_prev, eta, stats=None, tag=""):
    """One iteration on the GPU through the C ABI, checked stage by stage
    against the oracle started from the same state and fed the same payloads."""
    offs, d, M = st.offs, st.d, st.M
    h = st.host()
    # poison outputs so that stale values cannot pass
    st.ws.fill_(0x5555555555555555)
    st.wc.fill_(-7.0)
    st.ss.fill_(0x5555555555555555)
    st.sc.fill_(-7.0)
    # ---- worker
    if st.fused:
        st.wmsg.fill_(0xA5)
        st.smsg.fill_(0xA5)
        ef.ef_worker_step_fused(st.plan, st.g, st.m, st.e, mu, eta_prev, eta, st.wmsg)
        torch.cuda.synchronize()
        ws, wc, padding = st.split(st.wmsg)
        assert (padding == 0xA5).all(), "%s: worker wrote into the padding of a message" % tag
    else:
        ef.ef_worker_step(st.plan, st.g, st.m, st.e, mu, eta_prev, eta, st.ws, st.wc)
        torch.cuda.synchronize()
        ws, wc = to_np(st.ws), to_np(st.wc)
    n_loose = 0
    for i in range(M):
        m_i, e_i = h["m"][i].copy(), h["e"][i].copy()
        s_ref, c_ref = oracle.worker_step(h["g"][i], m_i, e_i, offs, F(mu), F(eta_prev), F(eta))
        assert np.array_equal(ws[i], s_ref), "%s worker %d: sign words differ (%d words)" % (
            tag, i, (ws[i] != s_ref).sum())
        assert np.array_equal(to_np(st.m[i, :d]).view(np.uint32), m_i.view(np.uint32)), \
            "%s worker %d: momentum differs" % (tag, i)
        same = check_scales(wc[i], c_ref, "%s worker %d" % (tag, i))
        n_loose += int((~same).sum())
        check_vector(to_np(st.e[i, :d]), e_i, c_ref, same, offs, "%s worker %d residual" % (tag, i))
    # padding columns of the strided state must be untouched
    if st.stride > d:
        assert not to_np(st.m[:, d:]).any() and not to_np(st.e[:, d:]).any(), "%s: wrote past d" % tag
    # ---- server, fed with the GPU's worker payloads on both sides
    if st.fused:
        ef.ef_server_step_fused(st.plan, M, st.wmsg, st.te, eta_prev, eta, st.smsg)
    else:
        ef.ef_server_step(st.plan, M, st.ws, st.wc, st.te, eta_prev, eta, st.ss, st.sc)
    torch.cuda.synchronize()
    te_ref = h["te"].copy()
    ss_ref, sc_ref = oracle.server_step(np.ascontiguousarray(ws), np.ascontiguousarray(wc), te_ref, offs,
                                        F(eta_prev), F(eta))
    if st.fused:
        ss, sc, padding = st.split(st.smsg)
        ss, sc = ss[0], sc[0]
        assert (padding == 0xA5).all(), "%s: server wrote into the padding of its message" % tag
    else:
        ss, sc = to_np(st.ss), to_np(st.sc)
    assert np.array_equal(ss, ss_ref), "%s server: sign words differ (%d words)" % (tag, (ss != ss_ref).sum())
    same = check_scales(sc, sc_ref, "%s server" % tag)
    n_loose += int((~same).sum())
    check_vector(to_np(st.te), te_ref, sc_ref, same, offs, "%s server residual" % tag)
    # ---- apply, fed with the GPU's server payload on both sides
    if st.fused:
        ef.ef_apply_fused(st.plan, st.x, st.smsg, eta)
    else:
        ef.ef_apply(st.plan, st.x, st.ss, st.sc, eta)
    torch.cuda.synchronize()
    x_ref = h["x"].copy()
    oracle.apply(x_ref, np.ascontiguousarray(ss), np.ascontiguousarray(sc), offs, F(eta))
    assert np.array_equal(to_np(st.x).view(np.uint32), x_ref.view(np.uint32)), "%s apply: parameters differ" % tag
    if stats is not None:
        stats["scales_not_bit_equal"] = stats.get("scales_not_bit_equal", 0) + n_loose
    return n_loose
