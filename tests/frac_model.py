"""A second, independently written evaluation of the paper's definitions with Python Fractions.

Used only to cross-check the C++ oracle by brute force on tiny cases.  It follows the paper's
equations (Sec. 2.3 quantizer, Sec. 3 FMAq, App. D recursion) on exact rationals; it is NOT how
the oracle computes (that one uses integer magnitudes in a common unit) and it is far too slow
for anything but a handful of steps.
"""
from fractions import Fraction as F


def e4m3_value(code):
    s = -1 if code & 0x80 else 1
    e = (code >> 3) & 15
    m = code & 7
    if e == 0:
        return s * F(m, 8) * F(1, 64)
    return s * (1 + F(m, 8)) * F(2) ** (e - 7)


def code_value(code, E, M, bias):
    """8-bit code, 1 sign / E exponent / M mantissa bits: subnormals at e = 0, every code finite."""
    s = -1 if code & 0x80 else 1
    e = (code >> M) & ((1 << E) - 1)
    m = code & ((1 << M) - 1)
    if e == 0:
        return s * F(m, 2 ** M) * F(2) ** (1 - bias)
    return s * (1 + F(m, 2 ** M)) * F(2) ** (e - bias)


def floor_log2(x):
    """floor(log2 x) for a positive Fraction."""
    e = x.numerator.bit_length() - x.denominator.bit_length()
    if F(2) ** e > x:
        e -= 1
    assert F(2) ** e <= x < F(2) ** (e + 1)
    return e


def rne_int(x):
    fl = x.numerator // x.denominator
    r = x - fl
    if r > F(1, 2) or (r == F(1, 2) and fl % 2 == 1):
        return fl + 1
    return fl


NO_UNDERFLOW = 0x100


def quant(x, E, M, b, rnd):
    """rnd: 0 floor, 1 nearest-even; | NO_UNDERFLOW drops the flush-to-zero case."""
    no_uf = bool(rnd & NO_UNDERFLOW)
    rnd &= ~NO_UNDERFLOW
    r_of = F(2) ** (2 ** E - b - 1) * (2 - F(1, 2 ** M))
    r_uf = F(2) ** (-b)
    sgn = -1 if x < 0 else 1
    ax = abs(x)
    if ax >= r_of:
        return sgn * r_of, "OF"
    if ax == 0:
        return F(0), ""
    if ax < r_uf and not no_uf:
        return F(0), "UF"
    e = floor_log2(ax)
    frac = (ax / F(2) ** e - 1) * 2 ** M
    m = rne_int(frac) if rnd == 1 else frac.numerator // frac.denominator
    return sgn * F(2) ** e * (1 + F(m, 2 ** M)), ""


def fmaq(a_code, b_code, s, qp, qa, in_a=None, in_b=None):
    va = e4m3_value(a_code) if in_a is None else code_value(a_code, *in_a)
    vb = e4m3_value(b_code) if in_b is None else code_value(b_code, *in_b)
    xw = va * vb
    p, _ = quant(xw, *qp)
    t = p + s
    z, ev = quant(t, *qa)
    of = ev == "OF"
    uf = (xw != 0 and p == 0) or ev == "UF"
    return z, of, uf


def chain(a_codes, b_codes, qp, qa, in_a=None, in_b=None):
    s = F(0)
    evs = []
    for a, b in zip(a_codes, b_codes):
        s, of, uf = fmaq(a, b, s, qp, qa, in_a, in_b)
        evs.append((of, uf))
    return s, evs


def chain_chunk16(a_codes, b_codes, qp, qa, with_events=False):
    """Two-level order: chains of 16 from zero, then a chain over the chunk sums (no Q_prod there).
    With events: (value, [(OF, UF) per step k], [(OF, UF) per chunk j])."""
    t = F(0)
    ev1, ev2 = [], []
    for k0 in range(0, len(a_codes), 16):
        c, evs = chain(a_codes[k0:k0 + 16], b_codes[k0:k0 + 16], qp, qa)
        ev1.extend(evs)
        t, ev = quant(t + c, *qa)
        ev2.append((ev == "OF", ev == "UF"))
    return (t, ev1, ev2) if with_events else t


def ste_diff(a_code, b_code, s, qp, qa, eps2, eps1=None, in_a=None, in_b=None):
    """STE^DIFF of one step (Sec. 4 / App. D): 1 iff |FMAq(x, w, s) - s| / (|x w| + eps1) > eps2, as the ratio
    it is written as.  eps1 = None is the limit eps1 -> 0+: a zero product makes the ratio 0 (the numerator is 0
    too: Q_acc(0 + s) = s for s on the accumulator's grid)."""
    va = e4m3_value(a_code) if in_a is None else code_value(a_code, *in_a)
    vb = e4m3_value(b_code) if in_b is None else code_value(b_code, *in_b)
    xw = va * vb
    z, _, _ = fmaq(a_code, b_code, s, qp, qa, in_a, in_b)
    num = abs(z - s)
    if eps1 is None:
        if xw == 0:
            assert num == 0
            return 0
        ratio = num / abs(xw)
    else:
        ratio = num / (abs(xw) + F(eps1))
    return 1 if ratio > F(eps2) else 0


def chain_diff(a_codes, b_codes, qp, qa, eps2, eps1=None, in_a=None, in_b=None):
    """(value, [STE^DIFF per step]) of a sequential chain."""
    s = F(0)
    out = []
    for a, b in zip(a_codes, b_codes):
        out.append(ste_diff(a, b, s, qp, qa, eps2, eps1, in_a, in_b))
        s, _, _ = fmaq(a, b, s, qp, qa, in_a, in_b)
    return s, out
