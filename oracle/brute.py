"""Definition-level brute force for tiny inputs -- TEST INFRASTRUCTURE ONLY.

Independent of ``se_oracle.c``: exact rational arithmetic (``fractions.Fraction``) with
an explicit round-to-nearest-even to binary32 after every fp32 operation, and no member
lists -- every worker scans all workers and keeps those sharing its group, as the SESGD
update equation (Sec. 3.2) is written.  Meant for a handful of columns (n <= 8 for every group size; a few larger n to pin the
summation order of groups of more than 8).
"""
from __future__ import annotations

from fractions import Fraction

import numpy as np

_MASK = 0xFFFFFFFF


def rn32(q: Fraction) -> Fraction:
    """Round an exact rational to the nearest binary32 value, ties to even.  Handles
    subnormals; raises on overflow (never reached by the tests)."""
    if q == 0:
        return Fraction(0)
    sign = -1 if q < 0 else 1
    a = abs(q)
    # exponent e with 2^e <= a < 2^(e+1)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    elif Fraction(2) ** (e + 1) <= a:
        e += 1
    e = max(e, -126)                      # subnormal range shares the exponent -126
    ulp = Fraction(2) ** (e - 23)
    scaled = a / ulp                      # exact
    lo = scaled.numerator // scaled.denominator
    rem = scaled - lo
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (lo & 1)):
        lo += 1
    out = lo * ulp
    if out >= Fraction(2) ** 128:
        raise OverflowError("binary32 overflow")
    return sign * out


def f32(x) -> Fraction:
    """Exact value of a float that is already representable in binary32."""
    return Fraction(float(np.float32(x)))


def fma32(a: Fraction, b: Fraction, c: Fraction) -> Fraction:
    return rn32(a * b + c)


def add32(a: Fraction, b: Fraction) -> Fraction:
    return rn32(a + b)


def mul32(a: Fraction, b: Fraction) -> Fraction:
    return rn32(a * b)


BLOCK = 8


def sum_in_order(vals) -> Fraction:
    """The library's fixed summation order on a list of binary32 values (ascending worker id):
    consecutive blocks of 8 are each added up left to right, then the block sums are added up
    left to right, with one rounding per addition."""
    parts = []
    for b in range(0, len(vals), BLOCK):
        part = vals[b]
        for q in vals[b + 1:b + BLOCK]:
            part = add32(part, q)
        parts.append(part)
    total = parts[0]
    for part in parts[1:]:
        total = add32(total, part)
    return total


def _mix32(z: int) -> int:
    z ^= z >> 16
    z = (z * 0x6A09E667) & _MASK
    z ^= z >> 15
    z = (z * 0xBB67AE85) & _MASK
    z ^= z >> 16
    return z


def brute_key(seed: int, it: int, n: int, i: int) -> int:
    golden = 0x9E3779B9
    h = golden
    for w in (seed & _MASK, (seed >> 32) & _MASK, it & _MASK, (it >> 32) & _MASK, n, i):
        h = _mix32(((h ^ w) + golden) & _MASK)
    return h


def brute_group_of(seed: int, n: int, m: int, it: int) -> list:
    """Sort the workers by (key, id) and cut the order into consecutive blocks of m."""
    order = sorted(range(n), key=lambda i: (brute_key(seed, it, n, i), i))
    group_of = [0] * n
    for pos, i in enumerate(order):
        group_of[i] = pos // m
    return group_of


def brute_step(x, g, v, group_of, m, lr, mu):
    """x, g: [n][P] nested lists/arrays of binary32-representable numbers; v the same or
    None.  Returns (x_new, v_new) as float32 arrays.  For every worker i on its own:
    x_new[i] = (1/m) * sum (in the fixed order) over all j, ascending, with
    group_of[j] == group_of[i] of xhat[j], where xhat[j] = x[j] - lr*v'[j] and
    v'[j] = mu*v[j] + g[j]."""
    n = len(x)
    P = len(x[0])
    lr_q, mu_q = f32(lr), f32(mu)
    inv_m = rn32(Fraction(1) / f32(m))
    x_new = np.zeros((n, P), np.float32)
    v_new = None if v is None else np.zeros((n, P), np.float32)
    for e in range(P):
        vprime, xhat = [], []
        for j in range(n):
            gg = f32(g[j][e])
            vp = gg if v is None else fma32(mu_q, f32(v[j][e]), gg)
            vprime.append(vp)
            xhat.append(fma32(-lr_q, vp, f32(x[j][e])))
        for i in range(n):
            s = sum_in_order([xhat[j] for j in range(n) if group_of[j] == group_of[i]])
            x_new[i, e] = np.float32(float(mul32(s, inv_m)))
            if v is not None:
                v_new[i, e] = np.float32(float(vprime[i]))
    return x_new, v_new


def brute_ring_step(x, g, v, lr, mu):
    """Mean gradient over all workers, then the same momentum/SGD update on each."""
    n = len(x)
    P = len(x[0])
    lr_q, mu_q = f32(lr), f32(mu)
    inv_n = rn32(Fraction(1) / f32(n))
    x_new = np.zeros((n, P), np.float32)
    v_new = None if v is None else np.zeros((n, P), np.float32)
    for e in range(P):
        gbar = mul32(sum_in_order([f32(g[j][e]) for j in range(n)]), inv_n)
        for i in range(n):
            vp = gbar if v is None else fma32(mu_q, f32(v[i][e]), gbar)
            x_new[i, e] = np.float32(float(fma32(-lr_q, vp, f32(x[i][e]))))
            if v is not None:
                v_new[i, e] = np.float32(float(vp))
    return x_new, v_new


def brute_step_ex(x, g, v, group_of, m, lr, mu, wd=0.0, grad_avg=False):
    """General form: weight decay d = wd*x + gsrc folded into the momentum update; with
    grad_avg the gradients (not the parameters) are averaged inside the group and every
    worker updates on its own."""
    n = len(x)
    P = len(x[0])
    lr_q, mu_q, wd_q = f32(lr), f32(mu), f32(wd)
    inv_m = rn32(Fraction(1) / f32(m))
    x_new = np.zeros((n, P), np.float32)
    v_new = None if v is None else np.zeros((n, P), np.float32)
    for e in range(P):
        if grad_avg:
            for i in range(n):
                s = sum_in_order([f32(g[j][e]) for j in range(n) if group_of[j] == group_of[i]])
                gbar = mul32(s, inv_m)
                d = gbar if wd_q == 0 else fma32(wd_q, f32(x[i][e]), gbar)
                vp = d if v is None else fma32(mu_q, f32(v[i][e]), d)
                x_new[i, e] = np.float32(float(fma32(-lr_q, vp, f32(x[i][e]))))
                if v is not None:
                    v_new[i, e] = np.float32(float(vp))
        else:
            xhat, vprime = [], []
            for j in range(n):
                gg = f32(g[j][e])
                d = gg if wd_q == 0 else fma32(wd_q, f32(x[j][e]), gg)
                vp = d if v is None else fma32(mu_q, f32(v[j][e]), d)
                vprime.append(vp)
                xhat.append(fma32(-lr_q, vp, f32(x[j][e])))
            for i in range(n):
                s = sum_in_order([xhat[j] for j in range(n) if group_of[j] == group_of[i]])
                x_new[i, e] = np.float32(float(mul32(s, inv_m)))
                if v is not None:
                    v_new[i, e] = np.float32(float(vprime[i]))
    return x_new, v_new


def brute_global_average(x):
    n = len(x)
    P = len(x[0])
    inv_n = rn32(Fraction(1) / f32(n))
    out = np.zeros((n, P), np.float32)
    for e in range(P):
        s = sum_in_order([f32(x[j][e]) for j in range(n)])
        out[:, e] = np.float32(float(mul32(s, inv_n)))
    return out
