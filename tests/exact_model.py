"""Brute-force model of Algorithm 4 in exact rational arithmetic.

Independent of oracle/ and of the HIP library: pure-Python loops over
fractions.Fraction, with an explicit round-to-nearest-even to binary32 (or
binary64) after every operation the algorithm writes.  Only usable on tiny
inputs; it exists so that the oracle can be checked against something that is
not the oracle.
"""
from fractions import Fraction


def _round_to(q, mant_bits, emin):
    """Round the rational q to a binary float with `mant_bits` significand bits
    (including the hidden one) and minimum normal exponent `emin`, ties to even.
    Returns a Fraction.  Overflow is not handled (inputs are tiny)."""
    q = Fraction(q)
    if q == 0:
        return Fraction(0)
    s = -1 if q < 0 else 1
    a = -q if q < 0 else q
    # exponent e with 2^e <= a < 2^(e+1)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    elif Fraction(2) ** (e + 1) <= a:
        e += 1
    e = max(e, emin)
    ulp = Fraction(2) ** (e - (mant_bits - 1))
    n = a / ulp
    k = n.numerator // n.denominator
    rem = n - k
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (k & 1)):
        k += 1
    return s * k * ulp


def f32(q):
    return _round_to(q, 24, -126)


def f64(q):
    return _round_to(q, 53, -1022)


def block_of(j, offs):
    for b in range(len(offs) - 1):
        if offs[b] <= j < offs[b + 1]:
            return b
    raise IndexError(j)


def compress(p, offs):
    """C_B: per block (||p_b||_1 / d_b, bits) with bit = (p >= 0).  The L1 sum
    runs in binary64 in ascending order; the scale is rounded to binary32."""
    B = len(offs) - 1
    bits = [1 if v >= 0 else 0 for v in p]
    scales = []
    for b in range(B):
        acc = Fraction(0)
        for j in range(offs[b], offs[b + 1]):
            acc = f64(acc + abs(p[j]))
        scales.append(f32(f64(acc / (offs[b + 1] - offs[b]))))
    return bits, scales


def decode(bits, scales, offs):
    return [scales[block_of(j, offs)] if bits[j] else -scales[block_of(j, offs)]
            for j in range(len(bits))]


def worker(g, m, e, offs, mu, r):
    d = len(g)
    m_new = [f32(f32(mu * m[j]) + g[j]) for j in range(d)]
    p = [f32(f32(f32(mu * m_new[j]) + g[j]) + f32(r * e[j])) for j in range(d)]
    bits, scales = compress(p, offs)
    delta = decode(bits, scales, offs)
    e_new = [f32(p[j] - delta[j]) for j in range(d)]
    return m_new, e_new, bits, scales


def server(payloads, te, offs, r):
    M = len(payloads)
    d = len(te)
    acc = [Fraction(0)] * d
    for bits, scales in payloads:
        delta = decode(bits, scales, offs)
        acc = [f32(acc[j] + delta[j]) for j in range(d)]
    tp = [f32(f32(acc[j] / M) + f32(r * te[j])) for j in range(d)]
    bits, scales = compress(tp, offs)
    delta = decode(bits, scales, offs)
    te_new = [f32(tp[j] - delta[j]) for j in range(d)]
    return te_new, bits, scales


def apply(x, bits, scales, offs, eta):
    delta = decode(bits, scales, offs)
    return [f32(x[j] - f32(eta * delta[j])) for j in range(len(x))]


def pack(bits):
    words = [0] * ((len(bits) + 63) // 64)
    for j, b in enumerate(bits):
        if b:
            words[j // 64] |= 1 << (j % 64)
    return words


def apply_wd(x, mt, bits, scales, offs, eta, mu, lam):
    """Appendix A: mt <- mu*mt + lam*x ; x <- x - eta*(Delta + mu*mt + lam*x)."""
    delta = decode(bits, scales, offs)
    x_new, m_new = [], []
    for j in range(len(x)):
        lx = f32(lam * x[j])
        mn = f32(f32(mu * mt[j]) + lx)
        u = f32(f32(delta[j] + f32(mu * mn)) + lx)
        m_new.append(mn)
        x_new.append(f32(x[j] - f32(eta * u)))
    return x_new, m_new


def worker_sgd(g, e, offs, r):
    """Algorithm 3 worker: p = g + r e."""
    d = len(g)
    p = [f32(g[j] + f32(r * e[j])) for j in range(d)]
    bits, scales = compress(p, offs)
    delta = decode(bits, scales, offs)
    return [f32(p[j] - delta[j]) for j in range(d)], bits, scales
