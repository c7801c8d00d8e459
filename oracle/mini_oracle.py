"""A second, even plainer oracle for one super-group at a time, in pure Python.

TEST INFRASTRUCTURE.  It restates the quantizer of Section 3.3 with Python
integers, numpy.float32 scalars and exact rational arithmetic for the fused
multiply-adds, and is used only to cross-check the C oracle on a few
super-groups (two implementations written separately must agree bit for bit).
It shares nothing with dq_oracle.c or with the GPU library.
"""
from fractions import Fraction

import numpy as np

f32 = np.float32
M32 = 0xFFFFFFFF


def round_to_f32(q):
    """Correctly rounded (nearest, ties to even) binary32 value of the rational q."""
    if q == 0:
        return f32(0.0)
    sign = -1 if q < 0 else 1
    a = abs(q)
    # find e with 2^e <= a < 2^(e+1)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    if Fraction(2) ** (e + 1) <= a:
        e += 1
    e_q = max(e, -126) - 23  # exponent of one unit in the last place (subnormals: fixed)
    scaled = a / (Fraction(2) ** e_q)
    n = scaled.numerator // scaled.denominator
    rem = scaled - n
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (n & 1)):
        n += 1
    return f32(sign * float(Fraction(n) * Fraction(2) ** e_q))


def fma32(a, b, c):
    return round_to_f32(Fraction(float(a)) * Fraction(float(b)) + Fraction(float(c)))


def philox(ctr, key):
    c0, c1, c2, c3 = ctr
    k0, k1 = key
    for _ in range(10):
        p0 = 0xD2511F53 * c0
        p1 = 0xCD9E8D57 * c2
        c0, c1, c2, c3 = ((p1 >> 32) ^ c1 ^ k0) & M32, p1 & M32, ((p0 >> 32) ^ c3 ^ k1) & M32, p0 & M32
        k0 = (k0 + 0x9E3779B9) & M32
        k1 = (k1 + 0xBB67AE85) & M32
    return [c0, c1, c2, c3]


def levels(b, g):
    R = 2 ** (b - 1) - 1
    pw = [1.0]
    for _ in range(R):
        pw.append(pw[-1] * g)
    T = [f32(r) if R == 1 else f32((pw[r] - 1.0) / (pw[R] - 1.0)) for r in range(R + 1)]
    T[0], T[R] = f32(0), f32(1)
    D = [f32(T[r + 1] - T[r]) for r in range(R)]
    return T, D


def bits(x):
    return int(np.array(x, f32).view(np.uint32))


def draws(seed, rnd, n, sg, rank):
    key = (seed & M32, seed >> 32)

    def call(index, stream, r16):
        return philox((index & M32, index >> 32, rnd, (stream << 16) | r16), key)

    gamma = []
    for g in range(16):
        w = call(sg * 16 + g, 0, rank)
        gamma += [(w[k >> 2] >> (8 * (k & 3))) & 0xFF for k in range(16)]
    w = call(sg, 1, rank)
    sbytes = [(w[g >> 2] >> (8 * (g & 3))) & 0xFF for g in range(16)]
    w = call(sg, 2, 0xFFFF)
    return gamma, sbytes, perm_slot(w, n, rank)


def perm_slot(w, n, rank):
    """The shared permutation of 0..n-1 at `rank`: three rounds of (odd multiply + add, then the
    k bits in reverse order) on k = ceil(log2 n) bits, repeated until the value is below n,
    then rotated by floor(w3 n / 2^32)."""
    k = (n - 1).bit_length()

    def rounds(y):
        for t in range(3):
            y = ((w[t] | 1) * y + (w[t] >> 16)) % (1 << k)
            y = int(format(y, "b").zfill(k)[::-1], 2) if k else 0
        return y

    y = rounds(rank)
    while y >= n:
        y = rounds(y)
    return (y + ((w[3] * n) >> 32)) % n


def encode_sg(b, g, n, seed, rnd, sg, rank, v):
    """v: 256 float32.  Returns (codes[256], rG[16], sf_bits)."""
    T, D = levels(b, g)
    R = len(T) - 1
    gamma, sbytes, slot = draws(seed, rnd, n, sg, rank)
    v = [f32(x) for x in v]
    M = max(abs(x) for x in v)
    mb = bits(M)
    h = (mb >> 16) + (1 if mb & 0xFFFF else 0)
    if h < 0x0D80:
        h = 0
    sf = np.array(h << 16, np.uint32).view(f32)
    inv_n = f32(1.0) / f32(n)
    s_n = inv_n * f32(1.0 / 256.0)
    codes, rG = [], []
    for gi in range(16):
        o = (f32((slot + gi) % n) + f32(1.0 / 512.0)) * inv_n
        vg = v[gi * 16:(gi + 1) * 16]
        m = max(abs(x) for x in vg)
        rg = 0
        if h:
            t = min(m * (f32(255.0) / sf), f32(255.0))
            fl = np.floor(t)
            us = (f32(sbytes[gi]) + f32(0.5)) * f32(1.0 / 256.0)
            rg = int(fl) + (1 if us < t - fl else 0)
        rG.append(rg)
        for k, x in enumerate(vg):
            sign = bits(x) >> 31
            r = 0
            if rg:
                xn = min(abs(x) * (f32(1.0) / m), f32(1.0))
                u = fma32(f32(gamma[gi * 16 + k]), s_n, o)
                lo = max(i for i in range(R + 1) if T[i] <= xn)
                r = lo if lo == R else lo + (1 if fma32(u, D[lo], T[lo]) < xn else 0)
            codes.append((sign << (b - 1)) | r)
    return codes, rG, h


def decode_sg(b, g, codes, rG, sf_bits, local=None):
    T, _ = levels(b, g)
    R = len(T) - 1
    sf = np.array(sf_bits << 16, np.uint32).view(f32)
    step = sf / f32(255.0)
    out = []
    for i, cd in enumerate(codes):
        sfg = f32(rG[i // 16]) * step
        t = T[cd & R]
        if (cd >> (b - 1)) & 1:
            t = -t
        out.append(t * sfg if local is None else fma32(t, sfg, f32(local[i])))
    return np.array(out, f32)
