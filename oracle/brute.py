"""Scalar-loop brute force of the same path (Sec. III-C, Algorithm 1), for tiny inputs only.

TEST INFRASTRUCTURE ONLY.  It pins oracle/cocktail_oracle.py: no numpy vector
operation appears here.  Floating-point steps of the quantiser are evaluated in
exact rational arithmetic and rounded to binary32 / binary16 by an explicit
round-to-nearest-even routine, so a vectorised IEEE implementation and this one
can only agree if both follow the same sequence of correctly-rounded operations.
"""
from __future__ import annotations

import math
from fractions import Fraction
from typing import List, Sequence


def round_binary(x: Fraction, precision: int, emin: int, emax: int) -> Fraction:
    """Round an exact rational to the nearest value of a binary format (ties to even).

    precision: significand bits including the hidden one (24 for binary32, 11 for binary16);
    emin: exponent of the smallest normal (-126 / -14); emax: of the largest (127 / 15).
    Values above the largest finite number are not expected here (asserted).
    """
    if x == 0:
        return Fraction(0)
    sign = -1 if x < 0 else 1
    a = abs(x)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    elif Fraction(2) ** (e + 1) <= a:
        e += 1
    e = max(e, emin)                                   # subnormals share the exponent emin
    quantum = Fraction(2) ** (e - (precision - 1))
    n = a / quantum
    lo = n.numerator // n.denominator
    rem = n - lo
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and lo % 2 == 1):
        lo += 1
    r = lo * quantum
    assert r < Fraction(2) ** (emax + 1), "overflow not modelled"
    return sign * r


def rn32(x: Fraction) -> Fraction:
    return round_binary(x, 24, -126, 127)


def rn16(x: Fraction) -> Fraction:
    return round_binary(x, 11, -14, 15)


def rint_even(x: Fraction) -> int:
    lo = x.numerator // x.denominator
    rem = x - lo
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and lo % 2 == 1):
        lo += 1
    return lo


def quantize_group(xs: Sequence[float], bits: int):
    """One group of one token.  xs: python floats holding fp16 values.  Returns (codes, scale, zero) with
    scale/zero as python floats (exactly representable in fp16)."""
    qmax = (1 << bits) - 1
    fx = [Fraction(x) for x in xs]
    mn, mx = min(fx), max(fx)
    r = rn32(mx - mn)
    scale = rn16(rn32(r / qmax))
    if scale == 0:
        return [0] * len(xs), 0.0, float(mn)
    inv = rn32(1 / scale)
    codes = []
    for x in fx:
        t = rn32(rn32(x - mn) * inv)
        codes.append(min(max(rint_even(t), 0), qmax))
    return codes, float(scale), float(mn)


def plan(seq_len: int, chunk: int, bits: Sequence[int]):
    n = seq_len // chunk
    order = []
    for want in (2, 4, 8, 16):
        for i in range(n):
            if bits[i] == want:
                order.append(i)
    tok = {2: [], 4: [], 8: [], 16: []}
    for i in order:
        for r in range(chunk):
            tok[bits[i]].append(i * chunk + r)
    for t in range(n * chunk, seq_len):
        tok[16].append(t)
    return order, [tok[2], tok[4], tok[8], tok[16]]


def fp16_bytes(x: float) -> bytes:
    import struct
    return struct.pack("<e", x)


def build_class_bytes(kv: List[List[List[float]]], tokens: Sequence[int], bits: int, group: int) -> bytes:
    """Packed bytes of one class for one sequence.  kv[h][t][d] python floats (fp16 values);
    `tokens` = original token indices of the class in cache order."""
    hkv = len(kv)
    d = len(kv[0][0]) if kv[0] else 0
    n = len(tokens)
    if n == 0:
        return b""
    nblk = (n + 63) // 64
    rowb = d * 2 if bits == 16 else d * bits // 8
    metab = 0 if bits == 16 else 4 * (d // group)
    bb = 64 * (rowb + metab)
    out = bytearray(hkv * nblk * bb)
    for h in range(hkv):
        for r, t in enumerate(tokens):
            x = kv[h][t]
            blk, i = divmod(r, 64)
            base = (h * nblk + blk) * bb
            if bits == 16:
                row = b"".join(fp16_bytes(v) for v in x)
            else:
                per = 32 // bits
                words = [0] * (d // per)
                meta = b""
                for g in range(d // group):
                    codes, sc, ze = quantize_group(x[g * group:(g + 1) * group], bits)
                    meta += fp16_bytes(sc) + fp16_bytes(ze if ze != 0 else 0.0)
                    for j, c in enumerate(codes):
                        ch = g * group + j
                        wi, within = divmod(ch, per)
                        shift = (within // 2) * bits + (16 if within % 2 else 0)
                        words[wi] |= c << shift
                row = b"".join(int(w).to_bytes(4, "little") for w in words)
                mo = base + 64 * rowb + i * metab
                out[mo:mo + metab] = meta
            for p in range(rowb // 16):
                o = base + (p * 64 + i) * 16
                out[o:o + 16] = row[p * 16:(p + 1) * 16]
    return bytes(out)


def dequant_token(x: Sequence[float], bits: int, group: int) -> List[float]:
    if bits == 16:
        return [float(v) for v in x]
    out = []
    for g in range(len(x) // group):
        codes, sc, ze = quantize_group(x[g * group:(g + 1) * group], bits)
        out += [ze + c * sc for c in codes]
    return out


def attention(q: Sequence[float], k_rows: List[List[float]], v_rows: List[List[float]], sm_scale: float):
    """Single-query softmax attention with plain loops (float64)."""
    s = []
    for kr in k_rows:
        acc = 0.0
        for a, b in zip(q, kr):
            acc += a * b
        s.append(acc * sm_scale)
    m = max(s)
    e = [math.exp(v - m) for v in s]
    tot = math.fsum(e)
    d = len(v_rows[0])
    out = [math.fsum(e[t] * v_rows[t][j] for t in range(len(s))) / tot for j in range(d)]
    return out, m + math.log(tot)
