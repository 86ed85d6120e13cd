"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests uses the HIP library.  Each one checks the oracle against
something that is not the oracle: hand-worked blocks, the paper's printed
closed form, the Proposition 1 energy identity, the Lemma 3 recurrence, an
exact-rational brute force, and special cases with a known answer.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from tests import exact_model as xm

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
F = np.float32


def _bits(signs, d):
    w = np.asarray(signs, dtype=np.uint64)
    j = np.arange(d)
    return ((w[j // 64] >> (j % 64).astype(np.uint64)) & np.uint64(1)).astype(np.int64)


def _read_cases(path):
    cases, cur = [], None
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *vals = line.split()
        if key == "case":
            cur = {"name": vals[0]}
            cases.append(cur)
        else:
            cur[key] = vals
    return cases


# ------------------------------------------------- P1: hand-built blocks ---

@pytest.mark.parametrize("case", _read_cases(os.path.join(GOLD, "handbuilt_blocks.txt")),
                         ids=lambda c: c["name"])
def test_compressor_handbuilt(case):
    """Section 3.2 definition of C_B, worked by hand (tests/golden)."""
    v = np.array([float(s) for s in case["v"]], dtype=F)
    offs = np.array([int(s) for s in case["offsets"]], dtype=np.int64)
    signs, scales = oracle.compress(v, offs)
    assert scales.tolist() == [float(s) for s in case["scales"]]
    assert _bits(signs, v.size).tolist() == [int(s) for s in case["bits"]]
    cb = oracle.decode(signs, scales, offs)
    assert cb.tolist() == [float(s) for s in case["cb"]]
    assert (v - cb).tolist() == [float(s) for s in case["resid"]]
    # padding bits of the last word are zero
    assert int(signs[-1]) >> (v.size % 64 or 64) == 0


def test_zero_sign_convention():
    """sign(0): +0 and -0 both encode +1 (reading for the case the paper
    leaves open in Appendix A)."""
    v = np.array([0.0, -0.0, -1.0, 1.0], dtype=F)
    signs, scales = oracle.compress(v, [0, 4])
    assert _bits(signs, 4).tolist() == [1, 1, 0, 1]
    assert scales[0] == F(0.5)


def test_payload_size_matches_bit_count():
    """Table 1: d bits + 32 B bits per direction per worker."""
    for d, sizes in ((5, [4, 1]), (64, [64]), (65, [1, 64]), (1000, [300, 700])):
        offs = np.concatenate([[0], np.cumsum(sizes)])
        s, c = oracle.compress(np.ones(d, dtype=F), offs)
        assert s.size == (d + 63) // 64 and c.size == len(sizes)
        assert s.nbytes * 8 >= d and s.nbytes * 8 - d < 64
        assert c.nbytes * 8 == 32 * len(sizes)


def test_flat_index_packing_lsb_first():
    d = 200
    v = -np.ones(d, dtype=F)
    v[[0, 63, 64, 130, 199]] = 1.0
    signs, _ = oracle.compress(v, [0, 7, 100, 200])
    assert signs.tolist() == [(1 << 0) | (1 << 63), (1 << 0), (1 << 2), (1 << 7)]


# --------------------------------- P2: the paper's constant-magnitude case ---

def _const_mag_cases():
    rows = []
    for line in open(os.path.join(GOLD, "constant_magnitude_example.txt")):
        line = line.strip()
        if line and not line.startswith("#"):
            a, b, n = line.split()
            rows.append((float(a), int(b), int(n)))
    return rows


@pytest.mark.parametrize("alpha,B,n", _const_mag_cases())
def test_constant_magnitude_example(alpha, B, n):
    """Section 3.2: equal-size blocks with |v_i| = c_b, c_b/c_{b+1} = alpha.
    Blockwise: phi = 1, i.e. C_B(v) = v exactly.  Non-block (Eq. (1)):
    delta = (1+a)(1-a^B) / (B (1-a)(1+a^B))."""
    rng = np.random.default_rng(7)
    c = np.array([alpha ** (B - 1 - b) for b in range(B)])      # increasing, ratio alpha
    sig = rng.choice([-1.0, 1.0], size=B * n)
    v = (np.repeat(c, n) * sig).astype(F)
    assert np.array_equal(v.astype(np.float64), np.repeat(c, n) * sig)  # dyadic: exact in fp32
    offs = np.arange(B + 1) * n
    signs, scales = oracle.compress(v, offs)
    assert np.array_equal(scales.astype(np.float64), c)
    assert np.array_equal(oracle.decode(signs, scales, offs), v)        # phi = 1
    # non-block compressor on the same vector: one block
    s1, c1 = oracle.compress(v, [0, B * n])
    cv = oracle.decode(s1, c1, [0, B * n]).astype(np.float64)
    v64 = v.astype(np.float64)
    delta_meas = 1.0 - np.sum((cv - v64) ** 2) / np.sum(v64 ** 2)
    delta_paper = (1 + alpha) * (1 - alpha ** B) / (B * (1 - alpha) * (1 + alpha ** B))
    assert delta_meas == pytest.approx(delta_paper, rel=1e-6)


# -------------------------------- P3: Proposition 1 energy identity + bound ---

@pytest.mark.parametrize("seed", [0, 1, 2])
def test_prop1_energy_identity(seed):
    """Proof of Proposition 1: ||C_B(v)-v||^2 = sum_b (||v_b||_2^2 - ||v_b||_1^2/d_b)
    and C_B is phi(v)-approximate with phi >= min_b 1/d_b (Definition 1)."""
    rng = np.random.default_rng(seed)
    sizes = rng.integers(1, 300, size=40)
    offs = np.concatenate([[0], np.cumsum(sizes)])
    d = int(offs[-1])
    v = (rng.standard_normal(d) * np.repeat(10.0 ** rng.uniform(-3, 1, sizes.size), sizes)).astype(F)
    v[rng.random(d) < 0.05] = 0.0
    signs, scales = oracle.compress(v, offs)
    cv = oracle.decode(signs, scales, offs).astype(np.float64)
    v64 = v.astype(np.float64)
    phi = np.inf
    for b in range(sizes.size):
        sl = slice(offs[b], offs[b + 1])
        l1, l2sq, db = np.abs(v64[sl]).sum(), (v64[sl] ** 2).sum(), sizes[b]
        lhs = ((cv[sl] - v64[sl]) ** 2).sum()
        assert lhs == pytest.approx(l2sq - l1 * l1 / db, rel=2e-6, abs=1e-6 * l2sq)
        assert scales[b] == pytest.approx(l1 / db, rel=1e-6)
        if l2sq > 0:
            phi = min(phi, l1 * l1 / (db * l2sq))
    assert phi >= 1.0 / sizes.max() - 1e-12
    assert ((cv - v64) ** 2).sum() <= (1 - phi) * (v64 ** 2).sum() * (1 + 1e-6)


def test_compressor_idempotent_and_homogeneous():
    """C_B(C_B(v)) = C_B(v) (a block of +-s has L1 mean s) and
    C_B(2^k v) = 2^k C_B(v): consequences of the definition in Section 3.2."""
    rng = np.random.default_rng(3)
    offs = np.array([0, 5, 64, 65, 200, 333])
    v = rng.standard_normal(333).astype(F)
    s, c = oracle.compress(v, offs)
    cv = oracle.decode(s, c, offs)
    s2, c2 = oracle.compress(cv, offs)
    # a block of d_b copies of +-s sums to d_b*s exactly in double (d_b*s < 2^53 ulps)
    assert np.array_equal(s, s2) and np.array_equal(c, c2)
    s3, c3 = oracle.compress(v * F(8.0), offs)
    assert np.array_equal(s, s3) and np.array_equal(c * F(8.0), c3)


# ----------------------------------------------- P9: exact-rational brute force ---

def _fr(a):
    return [Fraction(float(v)) for v in np.asarray(a).ravel()]


def _run_exact(g_steps, offs, mu, etas):
    """Exact-rational Algorithm 4 over several steps; g_steps[t][i] lists."""
    M, d = len(g_steps[0]), len(g_steps[0][0])
    m = [[Fraction(0)] * d for _ in range(M)]
    e = [[Fraction(0)] * d for _ in range(M)]
    te = [Fraction(0)] * d
    x = [Fraction(0)] * d
    trace = []
    eta_prev = Fraction(0)
    for t, eta in enumerate(etas):
        r = xm.f32(eta_prev / eta)
        pay = []
        for i in range(M):
            m[i], e[i], bits, sc = xm.worker(g_steps[t][i], m[i], e[i], offs, mu, r)
            pay.append((bits, sc))
        te, sbits, ssc = xm.server(pay, te, offs, r)
        x = xm.apply(x, sbits, ssc, offs, eta)
        trace.append((pay, sbits, ssc, [list(v) for v in m], [list(v) for v in e], list(te), list(x)))
        eta_prev = eta
    return trace


@pytest.mark.parametrize("M,mu,etas,seed", [
    (1, 0.5, [0.25, 0.25, 0.25], 0),
    (2, 0.5, [0.5, 0.25, 0.125], 1),       # r = 2 after the first step
    (3, 0.9, [0.1, 0.1], 2),               # inexact mu, eta and division by 3
    (2, 0.0, [0.1, 0.3, 0.2], 3),          # Algorithm 3 (no momentum), changing stepsize
    (3, 0.75, [0.3, 0.1, 0.2], 4),
])
def test_bruteforce_tiny(M, mu, etas, seed):
    """d <= 8, B <= 3, M <= 3: every output of every step must equal the
    exact-rational model bit for bit."""
    rng = np.random.default_rng(seed)
    offs = [0, 3, 4, 8]
    d = 8
    T = len(etas)
    g = (rng.integers(-8, 9, size=(T, M, d)) / 8.0).astype(F)
    if seed >= 2:
        g = (rng.standard_normal((T, M, d))).astype(F)
        g[rng.random((T, M, d)) < 0.15] = 0.0
    muf, etaf = F(mu), [F(v) for v in etas]
    trace = _run_exact([[_fr(g[t, i]) for i in range(M)] for t in range(T)], offs,
                       Fraction(float(muf)), [Fraction(float(v)) for v in etaf])
    m = np.zeros((M, d), F)
    e = np.zeros((M, d), F)
    te = np.zeros(d, F)
    x = np.zeros(d, F)
    eta_prev = F(0)
    for t in range(T):
        ws, wc, ss, sc = oracle.step(np.ascontiguousarray(g[t]), m, e, te, x, offs, muf, eta_prev, etaf[t])
        pay, sbits, ssc, mx, ex, tex, xx = trace[t]
        for i in range(M):
            assert int(ws[i, 0]) == xm.pack(pay[i][0])[0], (t, i)
            assert _fr(wc[i]) == pay[i][1], (t, i)
            assert _fr(m[i]) == mx[i], (t, i)
            assert _fr(e[i]) == ex[i], (t, i)
        assert int(ss[0]) == xm.pack(sbits)[0]
        assert _fr(sc) == ssc
        assert _fr(te) == tex
        assert _fr(x) == xx
        eta_prev = etaf[t]


# --------------------------------------------- P4: reconstruction invariant ---

def test_reconstruction_worker_and_server():
    """e_{t+1} = p_t - Delta_t (Algorithm 4): decode(payload) + e' gives back p,
    where p is recomputed here in float64 from the pre-step state."""
    rng = np.random.default_rng(11)
    sizes = [1, 7, 64, 100, 129, 3]
    offs = np.concatenate([[0], np.cumsum(sizes)])
    d, M = int(offs[-1]), 3
    mu, eta_prev, eta = F(0.9), F(0.2), F(0.1)
    g = rng.standard_normal((M, d)).astype(F)
    m0 = rng.standard_normal((M, d)).astype(F)
    e0 = (0.1 * rng.standard_normal((M, d))).astype(F)
    m, e = m0.copy(), e0.copy()
    ws = np.zeros((M, (d + 63) // 64), np.uint64)
    wc = np.zeros((M, len(sizes)), F)
    for i in range(M):
        ws[i], wc[i] = oracle.worker_step(g[i], m[i], e[i], offs, mu, eta_prev, eta)
        m_ref = float(mu) * m0[i].astype(np.float64) + g[i]
        p_ref = float(mu) * m_ref + g[i] + (float(eta_prev) / float(eta)) * e0[i]
        assert np.allclose(m[i], m_ref, rtol=3e-7, atol=1e-7)
        rec = oracle.decode(ws[i], wc[i], offs).astype(np.float64) + e[i]
        assert np.allclose(rec, p_ref, rtol=1e-6, atol=1e-6)
        # the bit is the sign of p wherever p is not within rounding of zero
        clear = np.abs(p_ref) > 1e-5
        assert np.array_equal(_bits(ws[i], d)[clear], (p_ref[clear] >= 0).astype(np.int64))
    te0 = (0.1 * rng.standard_normal(d)).astype(F)
    te = te0.copy()
    ss, sc = oracle.server_step(ws, wc, te, offs, eta_prev, eta)
    avg = np.mean([oracle.decode(ws[i], wc[i], offs).astype(np.float64) for i in range(M)], axis=0)
    tp_ref = avg + (float(eta_prev) / float(eta)) * te0
    rec = oracle.decode(ss, sc, offs).astype(np.float64) + te
    assert np.allclose(rec, tp_ref, rtol=1e-6, atol=1e-6)
    x0 = rng.standard_normal(d).astype(F)
    x = x0.copy()
    oracle.apply(x, ss, sc, offs, eta)
    assert np.allclose(x, x0 - float(eta) * oracle.decode(ss, sc, offs).astype(np.float64),
                       rtol=1e-6, atol=1e-7)


# -------------------------------------------- P5: Lemma 3, telescoped form ---

@pytest.mark.parametrize("mu,etas", [
    (0.9, [0.1] * 6),
    (0.9, [0.02, 0.05, 0.1, 0.1, 0.05, 0.01]),      # increasing then decreasing stepsize
    (0.0, [0.1, 0.2, 0.05, 0.05]),                  # Algorithm 3
])
def test_lemma3_error_corrected_iterate(mu, etas):
    """Lemma 3: x~_t = x_t - eta_{t-1} (e~_t + mean_i e_{t,i}) obeys
    x~_{t+1} = x~_t - eta_t mean_i (mu m_{t,i} + g_{t,i}).  The right-hand side
    is an uncompressed Nesterov-SGDM recursion run here in float64."""
    rng = np.random.default_rng(5)
    sizes = [10, 1, 200, 64, 37]
    offs = np.concatenate([[0], np.cumsum(sizes)])
    d, M = int(offs[-1]), 4
    x0 = rng.standard_normal(d).astype(F)
    x = x0.copy()
    m = np.zeros((M, d), F)
    e = np.zeros((M, d), F)
    te = np.zeros(d, F)
    m64 = np.zeros((M, d))
    xt = x0.astype(np.float64)           # the error-corrected iterate, float64 shadow
    eta_prev = F(0)
    for t, eta in enumerate(etas):
        eta = F(eta)
        g = rng.standard_normal((M, d)).astype(F)
        m64 = float(F(mu)) * m64 + g
        xt = xt - float(eta) * np.mean(float(F(mu)) * m64 + g, axis=0)
        oracle.step(g, m, e, te, x, offs, F(mu), eta_prev, eta)
        lhs = x.astype(np.float64) - float(eta) * (te.astype(np.float64) + e.astype(np.float64).mean(axis=0))
        assert np.allclose(lhs, xt, rtol=0, atol=2e-5 * (t + 1)), t
        assert np.allclose(m, m64, rtol=1e-5, atol=1e-5)
        eta_prev = eta


# --------------------------------- P6: identity-compressor case = exact SGDM ---

def test_identity_compressor_case_is_full_precision_sgdm():
    """Section 3.1: with C the identity the method is full-precision distributed
    SGD(M).  If every worker gets g = c_b * sigma (fixed +-1 pattern, dyadic c_b)
    then every compressed vector has constant magnitude per block, C_B acts as
    the identity, all residuals stay 0 and x follows Nesterov SGDM exactly."""
    rng = np.random.default_rng(9)
    sizes = [4, 16, 1, 43]
    offs = np.concatenate([[0], np.cumsum(sizes)])
    d, M = int(offs[-1]), 3
    sigma = rng.choice([-1.0, 1.0], size=d)
    c = np.repeat([0.5, 2.0, 0.25, 1.0], sizes)
    mu, eta = F(0.5), F(0.25)
    m = np.zeros((M, d), F)
    e = np.zeros((M, d), F)
    te = np.zeros(d, F)
    x = np.zeros(d, F)
    m_ref = np.zeros(d)
    x_ref = np.zeros(d)
    eta_prev = F(0)
    for t in range(5):
        gt = (c * sigma * (t + 1)).astype(F)
        g = np.tile(gt, (M, 1))
        m_ref = 0.5 * m_ref + gt
        x_ref = x_ref - 0.25 * (0.5 * m_ref + gt)
        oracle.step(g, m, e, te, x, offs, mu, eta_prev, eta)
        assert not e.any() and not te.any()
        assert np.array_equal(x.astype(np.float64), x_ref)
        assert np.array_equal(m[0].astype(np.float64), m_ref)
        eta_prev = eta


# ------------------------------------------------------------- P7: M = 1 ---

def test_single_worker_server_is_transparent_and_matches_ef_sgd():
    """M = 1: C_B is idempotent, so the server returns the worker's payload and
    its residual stays 0; with a constant stepsize and mu = 0 the iterates equal
    Algorithm 1 (EF-SGD, p = eta*g + e) up to rounding, by positive homogeneity."""
    rng = np.random.default_rng(13)
    sizes = [9, 64, 30]
    offs = np.concatenate([[0], np.cumsum(sizes)])
    d = int(offs[-1])
    eta = F(0.125)
    m = np.zeros((1, d), F)
    e = np.zeros((1, d), F)
    te = np.zeros(d, F)
    x = np.zeros(d, F)
    # Algorithm 1 in float64 with its own definition of C_B
    x1 = np.zeros(d)
    e1 = np.zeros(d)
    eta_prev = F(0)
    for t in range(6):
        g = rng.standard_normal((1, d)).astype(F)
        ws, wc, ss, sc = oracle.step(g, m, e, te, x, offs, F(0.0), eta_prev, eta)
        assert np.array_equal(ws[0], ss) and np.array_equal(wc[0], sc)
        assert not te.any()
        p1 = float(eta) * g[0] + e1
        delta1 = np.concatenate([np.abs(p1[a:b]).mean() * np.where(p1[a:b] >= 0, 1.0, -1.0)
                                 for a, b in zip(offs[:-1], offs[1:])])
        x1 = x1 - delta1
        e1 = p1 - delta1
        assert np.allclose(x, x1, rtol=0, atol=1e-5)
        assert np.allclose(float(eta) * e[0].astype(np.float64), e1, rtol=0, atol=1e-5)
        eta_prev = eta


# ------------------------------------------------------ P8: majority vote ---

@pytest.mark.parametrize("M", [3, 5, 4])
def test_equal_scales_give_majority_vote(M):
    """If all M scales of a block are equal and the server residual is 0, the
    server's sign is the majority of the workers' signs (signSGD with majority
    vote, Section 1) and its scale is s * mean_j |2 k_j - M| / M.  With M even
    an exact tie gives 0, which the zero convention encodes as +1."""
    rng = np.random.default_rng(M)
    sizes = [64, 11, 128]
    offs = np.concatenate([[0], np.cumsum(sizes)])
    d = int(offs[-1])
    s = np.array([0.5, 2.0, 0.125], F)
    bits = rng.integers(0, 2, size=(M, d))
    ws = np.zeros((M, (d + 63) // 64), np.uint64)
    for i in range(M):
        for j in np.nonzero(bits[i])[0]:
            ws[i, j // 64] |= np.uint64(1) << np.uint64(j % 64)
    wc = np.tile(s, (M, 1))
    te = np.zeros(d, F)
    ss, sc = oracle.server_step(ws, wc, te, offs, F(0.1), F(0.1))
    k = bits.sum(axis=0)
    assert np.array_equal(_bits(ss, d), (2 * k >= M).astype(np.int64))
    for b in range(3):
        sl = slice(offs[b], offs[b + 1])
        expect = float(s[b]) * np.abs(2 * k[sl] - M).mean() / M
        assert sc[b] == pytest.approx(expect, rel=1e-6)


# --------------------------------------------------------- P11: restart ---

def test_restart_from_snapshot_is_bit_identical():
    """The state of Algorithm 4 is (m_i, e_i, e~, x, eta_{t-1}); T steps equal
    T1 steps + snapshot + T-T1 steps."""
    rng = np.random.default_rng(21)
    offs = np.array([0, 50, 51, 180, 256, 300])
    d, M, T = 300, 2, 5
    g = rng.standard_normal((T, M, d)).astype(F)
    etas = [F(v) for v in (0.1, 0.1, 0.05, 0.05, 0.025)]

    def run(state, t0, t1):
        m, e, te, x, eta_prev = state
        for t in range(t0, t1):
            oracle.step(np.ascontiguousarray(g[t]), m, e, te, x, offs, F(0.9), eta_prev, etas[t])
            eta_prev = etas[t]
        return m, e, te, x, eta_prev

    z = lambda *s: np.zeros(s, F)
    full = run((z(M, d), z(M, d), z(d), z(d), F(0)), 0, T)
    half = run((z(M, d), z(M, d), z(d), z(d), F(0)), 0, 2)
    snap = tuple(np.array(a, copy=True) for a in half)
    rest = run((snap[0], snap[1], snap[2], snap[3], F(snap[4])), 2, T)
    for a, b in zip(full[:4], rest[:4]):
        assert np.array_equal(a, b)


# --------------------------------------------- phi(v) and delta (Section 3.2) ---

@pytest.mark.parametrize("alpha,B,n", _const_mag_cases())
def test_quality_constant_magnitude_example(alpha, B, n):
    """Section 3.2 example: phi = 1 and delta = (1+a)(1-a^B) / (B (1-a)(1+a^B))."""
    rng = np.random.default_rng(11)
    c = np.array([alpha ** (B - 1 - b) for b in range(B)])
    v = (np.repeat(c, n) * rng.choice([-1.0, 1.0], size=B * n)).astype(F)
    phi, delta = oracle.quality(v, np.arange(B + 1) * n)
    assert phi == pytest.approx(1.0, rel=1e-12)
    assert delta == pytest.approx((1 + alpha) * (1 - alpha ** B) / (B * (1 - alpha) * (1 + alpha ** B)), rel=1e-9)


def test_quality_one_hot_blocks_and_single_block():
    """A block with one non-zero has ratio 1/d_b (the lower bound of Proposition 1
    is attained); zero blocks are skipped; with B = 1, phi = delta."""
    sizes = [5, 1, 40, 7, 3]
    offs = np.concatenate([[0], np.cumsum(sizes)])
    v = np.zeros(int(offs[-1]), F)
    v[offs[0] + 2] = -3.0           # d_b = 5
    v[offs[2] + 39] = 0.25          # d_b = 40: the minimum
    v[offs[3]:offs[4]] = 2.0        # constant block: ratio 1
    phi, delta = oracle.quality(v, offs)
    assert phi == 1.0 / 40
    l1, l2 = 3.0 + 0.25 + 14.0, 9.0 + 0.0625 + 28.0
    assert delta == pytest.approx(l1 * l1 / (56 * l2), rel=1e-15)
    phi1, delta1 = oracle.quality(v, [0, 56])
    assert phi1 == delta1 == delta
    assert oracle.quality(np.zeros(9, F), [0, 4, 9]) == (1.0, 1.0)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_quality_is_the_approximation_constant(seed):
    """Definition 1 with Proposition 1: ||C_B(v) - v||^2 <= (1 - phi(v)) ||v||^2, with equality
    when every block has the same ratio; per block the identity of the proof gives
    ||C(v_b) - v_b||^2 = (1 - ratio_b) ||v_b||^2, so phi must equal the smallest measured ratio."""
    rng = np.random.default_rng(seed)
    sizes = rng.integers(1, 200, size=30)
    offs = np.concatenate([[0], np.cumsum(sizes)])
    v = (rng.standard_normal(int(offs[-1])) * np.repeat(10.0 ** rng.uniform(-2, 2, 30), sizes)).astype(F)
    v[rng.random(v.size) < 0.3] = 0.0
    phi, delta = oracle.quality(v, offs)
    signs, scales = oracle.compress(v, offs)
    cv = oracle.decode(signs, scales, offs).astype(np.float64)
    v64 = v.astype(np.float64)
    ratios = []
    for b in range(30):
        sl = slice(offs[b], offs[b + 1])
        n2 = (v64[sl] ** 2).sum()
        if n2 > 0:
            ratios.append(1.0 - ((cv[sl] - v64[sl]) ** 2).sum() / n2)
    assert phi == pytest.approx(min(ratios), rel=1e-5)
    assert ((cv - v64) ** 2).sum() <= (1 - phi) * (v64 ** 2).sum() * (1 + 1e-6)
    s1, c1 = oracle.compress(v, [0, v.size])
    c1v = oracle.decode(s1, c1, [0, v.size]).astype(np.float64)
    assert delta == pytest.approx(1.0 - ((c1v - v64) ** 2).sum() / (v64 ** 2).sum(), rel=1e-5)
    assert phi >= 1.0 / sizes.max() and 0 < delta <= 1


# ------------------------------------------- Algorithm 3 (no momentum) ---

def test_sgd_worker_is_momentum_worker_at_mu_zero():
    """Section 4.1: Algorithm 4 with mu = 0 is dist-EF-blockSGD (Algorithm 3).
    Run both workers over several steps with a changing stepsize; payloads and
    residuals agree (zeros compared by value: 0*m + g turns a -0 into +0)."""
    rng = np.random.default_rng(5)
    offs = np.array([0, 1, 9, 64, 65, 300])
    d = 300
    m, e4, e3 = np.zeros(d, F), np.zeros(d, F), np.zeros(d, F)
    eta_prev = F(0)
    for eta in (F(0.1), F(0.3), F(0.05), F(0.05)):
        g = rng.standard_normal(d).astype(F)
        g[rng.random(d) < 0.1] = 0.0
        s4, c4 = oracle.worker_step(g, m, e4, offs, F(0), eta_prev, eta)
        s3, c3 = oracle.worker_step_sgd(g, e3, offs, eta_prev, eta)
        assert np.array_equal(s4, s3) and np.array_equal(c4, c3)
        assert np.array_equal(e4, e3) and np.array_equal(m, g)
        eta_prev = eta


@pytest.mark.parametrize("seed", [0, 1])
def test_sgd_worker_bruteforce(seed):
    rng = np.random.default_rng(seed + 40)
    offs = [0, 2, 3, 9]
    e = np.zeros(9, F)
    ee = _fr(e)
    eta_prev = F(0)
    for eta in (F(0.1), F(0.3), F(0.07)):
        g = rng.standard_normal(9).astype(F)
        r = xm.f32(Fraction(float(eta_prev)) / Fraction(float(eta)))
        ee, bits, sc = xm.worker_sgd(_fr(g), ee, offs, r)
        signs, scales = oracle.worker_step_sgd(g, e, offs, eta_prev, eta)
        assert [int(b) for b in _bits(signs, 9)] == bits and _fr(scales) == sc and _fr(e) == ee
        eta_prev = eta


# ------------------------------------- Appendix A: weight decay outside C ---

def test_apply_wd_reduces_to_apply_without_decay():
    """lambda = 0 and a zero decay momentum: the Appendix A update is the plain
    x <- x - eta*Delta of Algorithm 4, bit for bit."""
    rng = np.random.default_rng(31)
    offs = np.array([0, 7, 64, 200])
    x0 = rng.standard_normal(200).astype(F)
    signs, scales = oracle.compress(rng.standard_normal(200).astype(F), offs)
    xa, xb, mt = x0.copy(), x0.copy(), np.zeros(200, F)
    oracle.apply(xa, signs, scales, offs, F(0.1))
    oracle.apply_wd(xb, mt, signs, scales, offs, F(0.1), F(0.9), F(0.0))
    assert np.array_equal(xa, xb) and not mt.any()


def test_apply_wd_zero_payload_is_momentum_weight_decay():
    """With a zero payload the update is m~ <- mu m~ + lam x, x <- x - eta (mu m~ + lam x):
    run in float64 on dyadic values, where every fp32 operation is exact."""
    offs = np.array([0, 4, 9])
    d = 9
    x = (np.arange(d) - 4).astype(F)               # small integers
    mt = np.zeros(d, F)
    signs = np.zeros(1, np.uint64)
    scales = np.zeros(2, F)
    xr, mr = x.astype(np.float64), np.zeros(d)
    for _ in range(4):
        mr = 0.5 * mr + 0.25 * xr
        xr = xr - 0.5 * (0.5 * mr + 0.25 * xr)
        oracle.apply_wd(x, mt, signs, scales, offs, F(0.5), F(0.5), F(0.25))
        assert np.array_equal(x.astype(np.float64), xr) and np.array_equal(mt.astype(np.float64), mr)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_apply_wd_bruteforce(seed):
    """Appendix A update against the exact-rational model, inexact constants."""
    rng = np.random.default_rng(seed)
    offs = [0, 3, 4, 8]
    x = rng.standard_normal(8).astype(F)
    mt = (0.1 * rng.standard_normal(8)).astype(F)
    signs, scales = oracle.compress(rng.standard_normal(8).astype(F), offs)
    bits = [int(b) for b in _bits(signs, 8)]
    eta, mu, lam = F(0.1), F(0.9), F(5e-4)
    xe, me = xm.apply_wd(_fr(x), _fr(mt), bits, _fr(scales), offs, Fraction(float(eta)), Fraction(float(mu)),
                         Fraction(float(lam)))
    oracle.apply_wd(x, mt, signs, scales, offs, eta, mu, lam)
    assert _fr(x) == xe and _fr(mt) == me


# ------------------------------------------------------- argument checks ---

def test_oracle_rejects_bad_partitions():
    v = np.ones(4, F)
    for offs in ([0, 2, 2, 4], [1, 4], [0, 3], [0, 5], [0, 3, 2, 4]):
        with pytest.raises(oracle.OracleError):
            oracle.compress(v, offs)


# ------------------------------------ large blocks: exactly rounded sums ---

def test_scale_of_a_large_block_against_the_exactly_rounded_sum():
    """Section 3.2: scale_b = ||v_Gb||_1 / d_b.  For blocks of 10^5 to 10^6 elements with magnitudes
    spread over many binades, math.fsum gives the correctly rounded fp64 value of the L1 norm; the
    oracle's ascending fp64 sum may differ from it by at most n * 2^-53 relative, so the fp32 scale
    is the correctly rounded one or its neighbour, and is the correctly rounded one whenever the
    exact quotient is not within that distance of a rounding boundary."""
    import math
    rng = np.random.default_rng(2024)
    sizes = [100003, 1 << 20, 250000]
    offs = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    v = (rng.standard_normal(int(offs[-1])) * 10.0 ** rng.uniform(-6, 3, int(offs[-1]))).astype(F)
    _, scales = oracle.compress(v, offs)
    for b, n in enumerate(sizes):
        seg = np.abs(v[offs[b]:offs[b + 1]].astype(np.float64))
        exact = math.fsum(seg.tolist()) / n
        want = np.float32(exact)
        got = scales[b]
        assert abs(float(got) - exact) <= abs(exact) * (2.0 ** -24 + n * 2.0 ** -53)
        ulp = np.spacing(want)
        assert abs(float(got) - float(want)) <= float(ulp)
        # away from a rounding boundary the two must be the same float
        lo, hi = float(want) - float(ulp) / 2, float(want) + float(ulp) / 2
        if min(exact - lo, hi - exact) > abs(exact) * n * 2.0 ** -52:
            assert got == want
