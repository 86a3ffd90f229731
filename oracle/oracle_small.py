"""A second, even slower statement of the operator, for vectors of a few thousand
coordinates: Python integers, `fractions.Fraction` and `math.fsum` instead of
C++ arithmetic, a bit string instead of a byte buffer.

TEST INFRASTRUCTURE ONLY.  It exists so that the C++ oracle is checked against
something written differently (exact rational sums, Python's arbitrary
precision integers for the Philox multiplies, a sort over tuples for the
selection); it follows the same passages of the paper: Algorithm 1 (worker
lines of a synchronisation step), Section 2.2 (Top_k / Rand_k), Definition 1
example 1 (QSGD), Definition 2 (Sign), Lemma 1's proof (norm over the kept
values), Lemma 3 with m = 1 (l1 scaling), Corollary 1 (per-block application).
"""
from __future__ import annotations

import math
import struct
from fractions import Fraction

import numpy as np

f32 = np.float32


def philox4x32_10(ctr, key):
    """Philox4x32 with ten rounds (Salmon et al., SC'11), on Python integers."""
    c = [int(x) & 0xFFFFFFFF for x in ctr]
    k = [int(x) & 0xFFFFFFFF for x in key]
    for _ in range(10):
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & 0xFFFFFFFF, (p0 >> 32) ^ c[3] ^ k[1], p0 & 0xFFFFFFFF]
        k = [(k[0] + 0x9E3779B9) & 0xFFFFFFFF, (k[1] + 0xBB67AE85) & 0xFFFFFFFF]
    return c


def random_word(seed, worker, rnd, stream, i):
    ctr = [i >> 2, worker, rnd & 0xFFFFFFFF, (rnd >> 32) | (stream << 30)]
    return philox4x32_10(ctr, [seed & 0xFFFFFFFF, seed >> 32])[i & 3]


def _bits(x):
    return struct.unpack("<I", struct.pack("<f", float(x)))[0]


def _round_fraction_to_double(q: Fraction) -> float:
    """Nearest-even double of a non-negative rational (Python's int/int division is correctly rounded)."""
    return q.numerator / q.denominator


def cube_root_fixed(x: float) -> float:
    """The cube root as the method takes it for m = 3: a start value from the binary exponent, then eight Newton
    steps y <- (2 y + x / y^2) / 3, every operation one IEEE double operation (Python floats are)."""
    if not x > 0.0:
        return 0.0
    mant, e = math.frexp(x)                       # x = mant * 2^e, 0.5 <= mant < 1: binary exponent E = e - 1
    E = e - 1
    q, r = divmod(E, 3)                           # floor division: r in {0, 1, 2}
    y = math.ldexp(1.0, q) * (1.0, 1.2599210498948732, 1.5874010519681994)[r]
    for _ in range(8):
        t = y * y
        u = x / t
        w = 2.0 * y
        y = (w + u) / 3.0
    return y


def compress(m, delta, d, seg_offset, seg_k, s, sparsifier, quantizer, seed, worker, rnd, dense=False):
    m = np.asarray(m, dtype=f32)
    delta = np.asarray(delta, dtype=f32)
    v = (m + delta).astype(f32)
    L = len(seg_k)
    w_idx = max(1, (d - 1).bit_length())
    qsgd = quantizer in (0, 4)                      # 4: the scaled operator of Lemma 2
    w_lev = (s - 1).bit_length() if qsgd else 0
    sel, levels, negs, gvals, scales, counts = [], [], [], [], [], []
    for l in range(L):
        lo, hi, k = int(seg_offset[l]), int(seg_offset[l + 1]), int(seg_k[l])
        if sparsifier == 0:
            ranked = sorted(range(lo, hi), key=lambda i: (-(_bits(v[i]) & 0x7FFFFFFF), i))
        else:
            ranked = sorted(range(lo, hi), key=lambda i: (-random_word(seed, worker, rnd, 0, i), i))
        S = sorted(ranked[:k])
        vs = [v[i] for i in S]
        if qsgd:
            total = sum(Fraction(float(x)) ** 2 for x in vs)
            N = f32(math.sqrt(_round_fraction_to_double(total)))
            N_sent = N
            if quantizer == 4:
                beta = min(k / (s * s), math.sqrt(k) / s)
                N_sent = f32(N / f32(1.0 + beta))
            n_sent = 0
            for i, x in zip(S, vs):
                lev = 0
                if N > 0:
                    a = f32(abs(x)) / N
                    t = min(f32(a * f32(s)), f32(s))
                    fl = f32(math.floor(float(t)))
                    frac = f32(t - fl)
                    u = f32(random_word(seed, worker, rnd, 1, i) >> 8) * f32(2.0 ** -24)
                    lev = int(fl) + (1 if u < frac else 0)
                neg = bool(x < 0)
                g = f32(0)
                if lev:
                    g = f32(f32(N_sent * f32(lev)) / f32(s))
                    g = -g if neg else g
                    n_sent += 1
                sel.append(i); levels.append(lev); negs.append(neg); gvals.append(g)
            scales.append(N_sent); counts.append(n_sent)
        elif quantizer == 3:                            # no quantiser
            for i, x in zip(S, vs):
                sel.append(i); levels.append(1); negs.append(bool(x < 0)); gvals.append(f32(x))
            scales.append(f32(0)); counts.append(k)
        else:
            if quantizer == 1:
                total = sum(Fraction(float(abs(x))) for x in vs)
                c = f32(_round_fraction_to_double(total) / float(k))
            elif quantizer == 2:                        # ||v_S||_2 / k
                total = sum(Fraction(float(x)) ** 2 for x in vs)
                c = f32(math.sqrt(_round_fraction_to_double(total)) / float(k))
            elif quantizer == 5:                        # ||v_S||_3 / k (Lemma 3, m = 3)
                total = sum(Fraction(float(abs(x))) ** 3 for x in vs)
                c = f32(cube_root_fixed(_round_fraction_to_double(total)) / float(k))
            else:                                       # ||v_S||_4 / k (Lemma 3, m = 4)
                total = sum(Fraction(float(x)) ** 4 for x in vs)
                c = f32(math.sqrt(math.sqrt(_round_fraction_to_double(total))) / float(k))
            for i, x in zip(S, vs):
                neg = bool(x < 0)
                sel.append(i); levels.append(1); negs.append(neg); gvals.append(-c if neg else c)
            scales.append(c); counts.append(k)

    # message as a list of bits, least significant bit of each field first
    bits = []

    def put(value, width):
        bits.extend((value >> b) & 1 for b in range(width))

    def align32():
        while len(bits) % 32:
            bits.append(0)

    nnz = sum(counts)
    if dense:
        # the index-free format of an operator that keeps every coordinate: one code per coordinate, in order;
        # a QSGD level is written as it is (0..s, in the bits needed to write s), then the sign bit
        assert all(int(seg_k[l]) == int(seg_offset[l + 1]) - int(seg_offset[l]) for l in range(L))
        put(d, 32)
        for sc in scales:
            put(_bits(sc), 32)
        w_code = (s.bit_length() + 1) if qsgd else 32 if quantizer == 3 else 1
        for lev, neg, g in zip(levels, negs, gvals):
            if quantizer == 3:
                put(_bits(g), 32)
                continue
            if qsgd:
                put(lev, s.bit_length())
            put(int(neg), 1)
        payload_bits = 32 + 32 * L + d * w_code
    else:
        put(nnz, 32)
        for sc in scales:
            put(_bits(sc), 32)
        if qsgd and L > 1:
            for c_ in counts:
                put(c_, 32)
        for i, lev in zip(sel, levels):
            if lev:
                put(i, w_idx)
        align32()
        for lev, neg, g in zip(levels, negs, gvals):
            if lev:
                if quantizer == 3:
                    put(_bits(g), 32)
                    continue
                if qsgd:
                    put(lev - 1, w_lev)
                put(int(neg), 1)
        header = 32 + 32 * L + (32 * L if qsgd and L > 1 else 0)
        payload_bits = header + nnz * (w_idx + (w_lev + 1 if qsgd else 32 if quantizer == 3 else 1))
    while len(bits) % 64:
        bits.append(0)
    msg = np.packbits(np.array(bits, dtype=np.uint8), bitorder="little")

    m_out = v.copy()
    for i, lev, g in zip(sel, levels, gvals):
        if lev:
            m_out[i] = f32(v[i] - g)
    return dict(m_out=m_out, msg=msg, bits=payload_bits, sel_idx=np.array(sel, dtype=np.uint32),
                sel_level=np.array(levels, dtype=np.uint16), sel_neg=np.array(negs, dtype=np.uint8),
                scales=np.array(scales, dtype=f32), g_val=np.array(gvals, dtype=f32))
