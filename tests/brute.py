"""Pure-Python exact-arithmetic brute force for tiny ring All-Reduce cases.

Independent of oracle/ (no import, no shared helper): values are decoded to
exact rationals, added exactly, and rounded to the target binary format by
explicit round-to-nearest-even on the rational.  The fold order is the closed
form of the ring: for block c the sum starts with the rank after c in the ring
and ends with rank c, rounding to the wire type after every addition
(accumulation itself goes through binary32 first).
"""
from fractions import Fraction

# (exponent bits, fraction bits)
FMT = {"fp32": (8, 23), "bf16": (8, 7), "fp16": (5, 10)}


def decode(bits, fmt):
    """bits -> ('num', Fraction, sign) | ('inf', sign) | ('nan',)"""
    eb, fb = FMT[fmt]
    sign = (bits >> (eb + fb)) & 1
    e = (bits >> fb) & ((1 << eb) - 1)
    m = bits & ((1 << fb) - 1)
    bias = (1 << (eb - 1)) - 1
    if e == (1 << eb) - 1:
        return ("nan",) if m else ("inf", sign)
    if e == 0:
        v = Fraction(m, 1 << fb) * Fraction(2) ** (1 - bias)
    else:
        v = (1 + Fraction(m, 1 << fb)) * Fraction(2) ** (e - bias)
    return ("num", -v if sign else v, sign)


def encode(x, sign_if_zero, fmt):
    """Round the exact rational x to fmt, ties to even; returns the bit pattern."""
    eb, fb = FMT[fmt]
    bias = (1 << (eb - 1)) - 1
    emax = (1 << eb) - 2 - bias
    emin = 1 - bias
    if x == 0:
        return sign_if_zero << (eb + fb)
    sign = 1 if x < 0 else 0
    a = -x if sign else x
    # exponent E with 2^E <= a < 2^(E+1)
    E = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** E > a:
        E -= 1
    if Fraction(2) ** (E + 1) <= a:
        E += 1
    E = max(E, emin)                       # subnormals share emin's spacing
    ulp = Fraction(2) ** (E - fb)
    q = a / ulp                            # in units of one ulp
    n = q.numerator // q.denominator
    rem = q - n
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (n & 1)):
        n += 1
    # n counts ulps: n < 2^fb subnormal, 2^fb <= n < 2^(fb+1) normal, == 2^(fb+1) carries
    if n == (1 << (fb + 1)):
        n >>= 1
        E += 1
    if n < (1 << fb):                      # subnormal (only possible at emin)
        return (sign << (eb + fb)) | n
    if E > emax:
        return (sign << (eb + fb)) | (((1 << eb) - 1) << fb)   # infinity
    return (sign << (eb + fb)) | ((E + bias) << fb) | (n - (1 << fb))


def add_round(a_bits, b_bits, src_fmt, dst_fmt):
    """round_dst(a + b) with a, b given in src_fmt; IEEE rules for specials and zeros."""
    a, b = decode(a_bits, src_fmt), decode(b_bits, src_fmt)
    eb, fb = FMT[dst_fmt]
    nan = (((1 << eb) - 1) << fb) | (1 << (fb - 1))
    if a[0] == "nan" or b[0] == "nan":
        return nan
    if a[0] == "inf" or b[0] == "inf":
        if a[0] == "inf" and b[0] == "inf":
            if a[1] != b[1]:
                return nan
            return (a[1] << (eb + fb)) | (((1 << eb) - 1) << fb)
        s = a[1] if a[0] == "inf" else b[1]
        return (s << (eb + fb)) | (((1 << eb) - 1) << fb)
    x = a[1] + b[1]
    # exact zero result: -0 only when both operands are negative (incl. -0 + -0)
    zero_sign = 1 if (a[2] == 1 and b[2] == 1) else 0
    return encode(x, zero_sign, dst_fmt)


def widen(bits, fmt):
    """Exact conversion of a wire value to binary32 bits (every wire value is representable)."""
    d = decode(bits, fmt)
    if d[0] == "nan":
        return 0x7FC00000
    if d[0] == "inf":
        return (d[1] << 31) | 0x7F800000
    return encode(d[1], d[2], "fp32")


def hop(incoming_bits, local_bits, fmt):
    """One ring hop: widen both to binary32, add with one rounding, round to the wire type."""
    s32 = add_round(widen(incoming_bits, fmt), widen(local_bits, fmt), "fp32", "fp32")
    d = decode(s32, "fp32")
    eb, fb = FMT[fmt]
    if d[0] == "nan":
        return (((1 << eb) - 1) << fb) | (1 << (fb - 1))
    if d[0] == "inf":
        return (d[1] << (eb + fb)) | (((1 << eb) - 1) << fb)
    return encode(d[1], d[2], fmt)


def hop_int32(a, b):
    s = (a + b) & 0xFFFFFFFF
    return s - (1 << 32) if s >= (1 << 31) else s


def block_ranges(count, W):
    B = -(-count // W)
    return [(min(c * B, count), min((c + 1) * B, count)) for c in range(W)]


def fold_order(c, ring):
    """Ranks in the order their values enter block c's sum."""
    W = len(ring)
    p = ring.index(c)
    return [ring[(p + k) % W] for k in range(1, W + 1)]


def allreduce(inputs, fmt, ring=None):
    """inputs: W lists of bit patterns (or Python ints for fmt == 'int32').
    Returns the list every rank must hold afterwards."""
    W = len(inputs)
    count = len(inputs[0])
    ring = list(range(W)) if ring is None else list(ring)
    out = [None] * count
    for c, (lo, hi) in enumerate(block_ranges(count, W)):
        order = fold_order(c, ring)
        for i in range(lo, hi):
            acc = inputs[order[0]][i]
            for r in order[1:]:
                acc = hop_int32(acc, inputs[r][i]) if fmt == "int32" else hop(acc, inputs[r][i], fmt)
            out[i] = acc
    return out


def reduce(inputs, fmt, root, ring=None):
    """Ring Reduce to `root`: every element summed in the order next(root), ..., root."""
    W = len(inputs)
    ring = list(range(W)) if ring is None else list(ring)
    order = fold_order(root, ring)
    out = []
    for i in range(len(inputs[0])):
        acc = inputs[order[0]][i]
        for r in order[1:]:
            acc = hop_int32(acc, inputs[r][i]) if fmt == "int32" else hop(acc, inputs[r][i], fmt)
        out.append(acc)
    return out


def sum_fp32acc(bits_in_order, fmt):
    """Binary32 running sum of the given wire values, in order, rounded to fmt once at the end."""
    acc = widen(bits_in_order[0], fmt)
    for b in bits_in_order[1:]:
        acc = add_round(acc, widen(b, fmt), "fp32", "fp32")
    d = decode(acc, "fp32")
    eb, fb = FMT[fmt]
    if d[0] == "nan":
        return (((1 << eb) - 1) << fb) | (1 << (fb - 1))
    if d[0] == "inf":
        return (d[1] << (eb + fb)) | (((1 << eb) - 1) << fb)
    return encode(d[1], d[2], fmt)


def allreduce_fp32acc(inputs, fmt, ring=None):
    W = len(inputs)
    count = len(inputs[0])
    ring = list(range(W)) if ring is None else list(ring)
    out = [None] * count
    for c, (lo, hi) in enumerate(block_ranges(count, W)):
        order = fold_order(c, ring)
        for i in range(lo, hi):
            out[i] = sum_fp32acc([inputs[r][i] for r in order], fmt)
    return out
