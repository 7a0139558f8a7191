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
FMT = {"fp32": (8, 23), "bf16": (8, 7), "fp16": (5, 10), "fp64": (11, 52)}
# integer wire types: (bits, signed)
INT = {"int32": (32, True), "int64": (64, True), "uint8": (8, False)}


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
    """One ring hop: widen both to binary32, add with one rounding, round to the wire type
    (fp64: one binary64 addition)."""
    if fmt == "fp64":
        return add_round(incoming_bits, local_bits, "fp64", "fp64")
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
                acc = node_int(acc, inputs[r][i], "sum", fmt) if fmt in INT else hop(acc, inputs[r][i], fmt)
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
            acc = node_int(acc, inputs[r][i], "sum", fmt) if fmt in INT else hop(acc, inputs[r][i], fmt)
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


# ---------------------------------------------------------------------------
# other operators, the tree order, rounding once: exact arithmetic as above
# ---------------------------------------------------------------------------
def _special(fmt, kind, sign=0):
    eb, fb = FMT[fmt]
    top = ((1 << eb) - 1) << fb
    if kind == "nan":
        return top | (1 << (fb - 1))
    return (sign << (eb + fb)) | top


def mul_round(a_bits, b_bits, src_fmt, dst_fmt):
    """round_dst(a * b) with IEEE rules for specials: 0 * inf = NaN, sign = xor of the signs."""
    a, b = decode(a_bits, src_fmt), decode(b_bits, src_fmt)
    if a[0] == "nan" or b[0] == "nan":
        return _special(dst_fmt, "nan")
    sa = a[1] if a[0] == "inf" else a[2]
    sb = b[1] if b[0] == "inf" else b[2]
    sign = sa ^ sb
    if a[0] == "inf" or b[0] == "inf":
        other = b if a[0] == "inf" else a
        if other[0] == "num" and other[1] == 0:
            return _special(dst_fmt, "nan")
        return _special(dst_fmt, "inf", sign)
    return encode(a[1] * b[1], sign, dst_fmt)


def pick_extreme(a_bits, b_bits, fmt, want_max):
    """maximum / minimum of IEEE 754-2019 (clause 9.6): NaN if either is NaN; -0 < +0."""
    a, b = decode(a_bits, fmt), decode(b_bits, fmt)
    if a[0] == "nan" or b[0] == "nan":
        return _special(fmt, "nan")

    def key(d):     # (value as a comparable, sign of zero as tie break): larger key = larger number
        if d[0] == "inf":
            return (2, 0, 0) if d[1] == 0 else (-2, 0, 0)
        return (0, d[1], -d[2])

    ka, kb = key(a), key(b)
    if ka == kb:
        return a_bits
    a_larger = ka > kb
    return a_bits if (a_larger == want_max) else b_bits


def node(a_bits, b_bits, fmt, op):
    """One hop / tree node with per-result rounding to fmt; operands and result are fmt bit patterns."""
    if op == "sum":
        return hop(a_bits, b_bits, fmt)
    if op == "prod":
        p32 = mul_round(widen(a_bits, fmt), widen(b_bits, fmt), "fp32", "fp32")
        d = decode(p32, "fp32")
        if d[0] == "nan":
            return _special(fmt, "nan")
        if d[0] == "inf":
            return _special(fmt, "inf", d[1])
        return encode(d[1], d[2], fmt)
    return pick_extreme(a_bits, b_bits, fmt, op == "max")


def node_int(a, b, op, fmt="int32"):
    """Integer hop: sum and product wrap modulo 2^bits (two's complement when signed)."""
    bits, signed = INT[fmt]
    if op in ("max", "min"):
        return max(a, b) if op == "max" else min(a, b)
    s = (a + b if op == "sum" else a * b) & ((1 << bits) - 1)
    return s - (1 << bits) if signed and s >= (1 << (bits - 1)) else s


def node_int32(a, b, op):
    return node_int(a, b, op, "int32")


def node64(a, b, op):
    """One fp64 hop: a single IEEE binary64 operation, nothing to widen or narrow."""
    if op == "sum":
        return add_round(a, b, "fp64", "fp64")
    if op == "prod":
        return mul_round(a, b, "fp64", "fp64")
    return pick_extreme(a, b, "fp64", op == "max")


def node32(a32, b32, op):
    """The same on binary32 bit patterns without narrowing (for rounding once)."""
    if op == "sum":
        return add_round(a32, b32, "fp32", "fp32")
    if op == "prod":
        return mul_round(a32, b32, "fp32", "fp32")
    return pick_extreme(a32, b32, "fp32", op == "max")


def narrow(x32, fmt):
    d = decode(x32, "fp32")
    if d[0] == "nan":
        return _special(fmt, "nan")
    if d[0] == "inf":
        return _special(fmt, "inf", d[1])
    return encode(d[1], d[2], fmt)


def combine(vals, fmt, op="sum", order="ring", rounding="each"):
    """vals: wire bit patterns (ints for int32) in the order they enter.  Ring: left fold.
    Tree: neighbours first, level by level, an odd last value moves up unchanged."""
    if fmt in INT:
        f = lambda a, b: node_int(a, b, op, fmt)
    elif fmt == "fp64":
        f = lambda a, b: node64(a, b, op)
        rounding = "each"          # the wire type is the accumulation type: nothing to round later
    elif rounding == "each":
        f = lambda a, b: node(a, b, fmt, op)
    else:
        vals = [widen(v, fmt) for v in vals]
        f = lambda a, b: node32(a, b, op)
    vals = list(vals)
    if order == "ring":
        acc = vals[0]
        for v in vals[1:]:
            acc = f(acc, v)
    else:
        while len(vals) > 1:
            nxt = [f(vals[k], vals[k + 1]) for k in range(0, len(vals) - 1, 2)]
            if len(vals) & 1:
                nxt.append(vals[-1])
            vals = nxt
        acc = vals[0]
    if fmt not in INT and rounding != "each":
        acc = narrow(acc, fmt)
    return acc


def allreduce_var(inputs, fmt, op="sum", ring=None, order="ring", rounding="each"):
    """What every rank must hold after the All-Reduce variant."""
    W = len(inputs)
    count = len(inputs[0])
    ring = list(range(W)) if ring is None else list(ring)
    out = [None] * count
    for c, (lo, hi) in enumerate(block_ranges(count, W)):
        who = fold_order(c, ring) if order == "ring" else ring
        for i in range(lo, hi):
            out[i] = combine([inputs[r][i] for r in who], fmt, op, order, rounding)
    return out
