"""Pins for the oracle's other reduction operators (product, maximum, minimum)
and for its tree-order variants (CPU only): exact-rational brute force, the
hand-derived fixtures under golden/, library routines where a case reduces to
one, order independence where the operator has it, and the error bound of the
tree against the correctly rounded exact sum."""
import os
import random

import numpy as np
import pytest
import torch

import brute
from oracle import ring_oracle as orc
from test_oracle_ring import CODE, GOLDEN, _bits, _from_values, _random_wire, _to_values

OPS = {"sum": orc.SUM, "prod": orc.PROD, "max": orc.MAX, "min": orc.MIN}
ORDERS = {"ring": orc.ORDER_RING, "tree": orc.ORDER_TREE}
ROUNDINGS = {"each": orc.ROUND_EACH, "once": orc.ROUND_ONCE}
NAN_MASK = {"fp32": (0x7FFFFFFF, 0x7F800000), "bf16": (0x7FFF, 0x7F80), "fp16": (0x7FFF, 0x7C00),
            "fp64": (0x7FFFFFFFFFFFFFFF, 0x7FF0000000000000)}


def _same(got_bits, want_bits, dtype):
    """bit equality where any NaN equals any NaN"""
    if dtype == "int32":
        return list(got_bits) == list(want_bits)
    m, inf = NAN_MASK[dtype]
    return all(g == w or ((g & m) > inf and (w & m) > inf) for g, w in zip(got_bits, want_bits))


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [line.split() for line in f if line.strip() and not line.startswith("#")]


def _sym(tok, dtype):
    """golden-file symbol -> wire bit pattern"""
    if tok == "nan":
        return _bits(_from_values([np.nan], dtype), dtype)[0]
    v = {"+inf": np.inf, "-inf": -np.inf, "inf": np.inf, "+0": 0.0, "-0": -0.0}.get(tok)
    if v is None:
        v = float(tok)
    return _bits(_from_values([v], dtype), dtype)[0]


def _wire_of_bits(bits, dtype):
    if dtype == "fp32":
        return np.array(bits, dtype=np.uint32).view(np.float32)
    if dtype == "fp64":
        return np.array(bits, dtype=np.uint64).view(np.float64)
    if dtype == "int32":
        return np.array(bits, dtype=np.int32)
    return np.array(bits, dtype=np.uint16)


# ------------------------------------------------------------ brute force
@pytest.mark.parametrize("dtype", ["fp32", "bf16", "fp16", "int32"])
@pytest.mark.parametrize("op", ["prod", "max", "min"])
def test_ring_with_other_operators_matches_brute_force(dtype, op):
    rng = np.random.Generator(np.random.Philox(300))
    rnd = random.Random(300)
    for W in (1, 2, 3, 5):
        for count in (0, 1, 7, 33):
            ring = list(range(W))
            rnd.shuffle(ring)
            ins = [_random_wire(rng, count, dtype) for _ in range(W)]
            for use_ring in (None, ring):
                want = brute.allreduce_var([_bits(a, dtype) for a in ins], dtype, op=op, ring=use_ring)
                for chunk in (0, 3):
                    out = orc.allreduce(ins, CODE[dtype], ring=use_ring, chunk_elems=chunk, op=OPS[op])
                    for o in out:
                        assert _same(_bits(o, dtype), want, dtype), (dtype, op, W, count, use_ring)
                # the closed-form variant with (ring order, per-result rounding) is the same result
                var = orc.allreduce_var(ins, CODE[dtype], op=OPS[op], ring=use_ring)
                assert _same(_bits(var[W - 1], dtype), want, dtype)


@pytest.mark.parametrize("dtype", ["fp32", "bf16", "fp16", "int32"])
@pytest.mark.parametrize("order,rounding", [("tree", "each"), ("tree", "once"), ("ring", "once")])
def test_variants_match_brute_force(dtype, order, rounding):
    rng = np.random.Generator(np.random.Philox(301))
    rnd = random.Random(301)
    for op in ("sum", "prod", "max"):
        for W in (1, 2, 3, 5, 6, 7):
            count = 2 * W + 3
            ring = list(range(W))
            rnd.shuffle(ring)
            ins = [_random_wire(rng, count, dtype) for _ in range(W)]
            want = brute.allreduce_var([_bits(a, dtype) for a in ins], dtype, op=op, ring=ring, order=order,
                                       rounding=rounding)
            out = orc.allreduce_var(ins, CODE[dtype], op=OPS[op], ring=ring, order=ORDERS[order],
                                    rounding=ROUNDINGS[rounding])
            for o in out:
                assert _same(_bits(o, dtype), want, dtype), (dtype, op, order, rounding, W)


def test_tree_shape_is_neighbours_first():
    """Symbolic check of the brute force's own tree (which the oracle is compared with):
    W = 5 gives ((v0 v1)(v2 v3)) v4, W = 6 gives ((v0 v1)(v2 v3))(v4 v5)."""
    def shape(W):
        vals = [str(k) for k in range(W)]
        while len(vals) > 1:
            nxt = ["(" + vals[k] + vals[k + 1] + ")" for k in range(0, len(vals) - 1, 2)]
            if len(vals) & 1:
                nxt.append(vals[-1])
            vals = nxt
        return vals[0]
    assert shape(5) == "(((01)(23))4)"
    assert shape(6) == "(((01)(23))(45))"
    assert shape(8) == "(((01)(23))((45)(67)))"
    # with values 2^k as int32 "sum" the tree and the ring agree (integers are associative) ...
    ins = [np.array([1 << k], dtype=np.int32) for k in range(6)]
    assert orc.allreduce_var(ins, orc.INT32, order=orc.ORDER_TREE)[0][0] == 63
    # ... and a float case tells the shapes apart: bf16 (256, 1, 1, 1, 1): neighbours first keeps
    # 1 + 1 = 2 alive: (256+1)+(1+1) = 256+2 = 258, then + 1 = 259 -> ties to 260 (even); a left
    # fold would lose every 1: 256
    # (five elements, one per block: element 4 is block 4, whose ring sum starts at rank 0)
    ins = [_from_values([v] * 5, "bf16") for v in (256.0, 1.0, 1.0, 1.0, 1.0)]
    assert np.all(_to_values(orc.allreduce_var(ins, orc.BF16, order=orc.ORDER_TREE)[0], "bf16") == 260.0)
    assert _to_values(orc.allreduce_var(ins, orc.BF16, ring=[0, 1, 2, 3, 4])[4], "bf16")[4] == 256.0


# ------------------------------------------------------------ golden fixtures
@pytest.mark.parametrize("row", _rows("prod_range_w4.txt"), ids=lambda r: r[0])
def test_product_overflow_underflow_example(row):
    dtype, e = row[0], int(row[1])
    n = 8
    B = 2.0 ** e
    ranks = [_from_values([v] * n, dtype) for v in (B, B, 1.0 / B, 1.0 / B)]
    out = orc.allreduce(ranks, CODE[dtype], op=orc.PROD)
    for r in range(4):
        for c in range(4):
            want = _sym(row[2 + c], dtype)
            assert _same(_bits(out[r][2 * c:2 * c + 2], dtype), [want, want], dtype), (dtype, r, c)
    tree = orc.allreduce_var(ranks, CODE[dtype], op=orc.PROD, order=orc.ORDER_TREE)
    assert _same(_bits(tree[0], dtype), [_sym(row[6], dtype)] * n, dtype)


@pytest.mark.parametrize("row", _rows("tree_cancellation_w4.txt"), ids=lambda r: r[0])
def test_tree_cancellation_example(row):
    dtype, M = row[0], float(row[1])
    ranks = [_from_values([v] * 12, dtype) for v in (M, 1.0, -M, 1.0)]
    each = orc.allreduce_var(ranks, CODE[dtype], order=orc.ORDER_TREE, rounding=orc.ROUND_EACH)
    once = orc.allreduce_var(ranks, CODE[dtype], order=orc.ORDER_TREE, rounding=orc.ROUND_ONCE)
    for r in range(4):
        assert np.all(_to_values(each[r], dtype) == float(row[2]))
        assert np.all(_to_values(once[r], dtype) == float(row[3]))


@pytest.mark.parametrize("dtype", ["fp32", "bf16", "fp16", "fp64"])
def test_maximum_minimum_of_special_operands(dtype):
    rows = _rows("minmax_specials.txt")
    a = _wire_of_bits([_sym(r[0], dtype) for r in rows], dtype)
    b = _wire_of_bits([_sym(r[1], dtype) for r in rows], dtype)
    for op, col in ((orc.MAX, 2), (orc.MIN, 3)):
        want = [_sym(r[col], dtype) for r in rows]
        assert _same(_bits(orc.hop_op(a, b, CODE[dtype], op), dtype), want, dtype)
        # through the ring, two ranks: incoming = rank 1's value for block 0, rank 0's for block 1
        out = orc.allreduce([a, b], CODE[dtype], op=op)
        assert _same(_bits(out[0], dtype), want, dtype) and _same(_bits(out[1], dtype), want, dtype)


# ------------------------------------------------------------ library routines
@pytest.mark.parametrize("dtype", ["fp32", "fp16", "bf16", "int32"])
def test_two_ranks_equal_the_library_elementwise_operation(dtype):
    rng = np.random.Generator(np.random.Philox(302))
    n = 200_000
    if dtype == "int32":
        x, y = (rng.integers(-2**31, 2**31, size=n, dtype=np.int64).astype(np.int32) for _ in range(2))
        lib = {"prod": (x.astype(np.int64) * y.astype(np.int64)).astype(np.int32),   # wraps
               "max": np.maximum(x, y), "min": np.minimum(x, y)}
    else:
        # random bit patterns cover subnormals, infinities, NaNs and both zeros
        x, y = (_random_wire(rng, n, dtype) for _ in range(2))
        if dtype == "bf16":
            tx, ty = (torch.from_numpy(v.view(np.int16).copy()).view(torch.bfloat16) for v in (x, y))
            back = lambda t: t.view(torch.int16).numpy().view(np.uint16)
            lib = {"prod": back(tx * ty), "max": back(torch.maximum(tx, ty)), "min": back(torch.minimum(tx, ty))}
        else:
            fx, fy = (v if dtype == "fp32" else v.view(np.float16) for v in (x, y))
            with np.errstate(all="ignore"):
                lib = {"prod": fx * fy, "max": np.maximum(fx, fy), "min": np.minimum(fx, fy)}
            if dtype == "fp16":
                lib = {k: v.view(np.uint16) for k, v in lib.items()}
    for name, want in lib.items():
        got = orc.allreduce([x, y], CODE[dtype], op=OPS[name])[0]
        gb, wb = _bits(got, dtype), _bits(np.ascontiguousarray(want), dtype)
        if name in ("max", "min") and dtype != "int32":
            # libraries do not promise the sign of a zero chosen among zeros: compare those as values
            m, _ = NAN_MASK[dtype]
            gb = [0 if (g & m) == 0 else g for g in gb]
            wb = [0 if (w & m) == 0 else w for w in wb]
        assert _same(gb, wb, dtype), (dtype, name)


@pytest.mark.parametrize("dtype", ["fp32", "bf16", "fp16", "int32"])
def test_maximum_minimum_do_not_depend_on_order(dtype):
    rng = np.random.Generator(np.random.Philox(303))
    W, n = 7, 3001
    ins = [_random_wire(rng, W * n, dtype) for _ in range(W)]
    ring = [3, 1, 4, 0, 6, 2, 5]
    for op in (orc.MAX, orc.MIN):
        base = orc.allreduce(ins, CODE[dtype], op=op)[0]
        for other in (orc.allreduce(ins, CODE[dtype], ring=ring, op=op)[2],
                      orc.allreduce_var(ins, CODE[dtype], op=op, order=orc.ORDER_TREE)[0],
                      orc.allreduce_var(ins, CODE[dtype], op=op, ring=ring, order=orc.ORDER_TREE,
                                        rounding=orc.ROUND_ONCE)[5]):
            assert _same(_bits(base, dtype), _bits(other, dtype), dtype)
        if dtype != "int32":
            # on finite inputs it is the library's reduction over the rank axis
            vals = np.array([_to_values(_from_values(rng.standard_normal(n), dtype), dtype) for _ in range(W)])
            fin = [_from_values(v, dtype) for v in vals]
            got = _to_values(orc.allreduce(fin, CODE[dtype], op=op)[0], dtype)
            assert np.array_equal(got, vals.max(axis=0) if op == orc.MAX else vals.min(axis=0))


def test_powers_of_two_multiply_exactly():
    rng = np.random.Generator(np.random.Philox(304))
    W, n = 8, 4000
    for dtype, lim in (("fp32", 15), ("bf16", 15), ("fp16", 1)):
        exps = rng.integers(-lim, lim + 1, size=(W, n))
        ins = [_from_values(np.exp2(e.astype(np.float64)), dtype) for e in exps]
        for out in (orc.allreduce(ins, CODE[dtype], op=orc.PROD)[0],
                    orc.allreduce_var(ins, CODE[dtype], op=orc.PROD, order=orc.ORDER_TREE)[0]):
            assert np.array_equal(_to_values(out, dtype), np.exp2(exps.sum(axis=0).astype(np.float64)))


def test_sum_operator_is_the_plain_ring_and_entry_points_agree():
    rng = np.random.Generator(np.random.Philox(305))
    W, n = 4, 500
    ring = [2, 0, 3, 1]
    for dtype in ("bf16", "fp16", "fp32", "int32"):
        ins = [_random_wire(rng, W * n, dtype) if dtype == "int32" else _from_values(rng.standard_normal(W * n), dtype)
               for _ in range(W)]
        # (ring order, per-result rounding, sum) is the ring All-Reduce itself
        a = orc.allreduce(ins, CODE[dtype], ring=ring)
        b = orc.allreduce_var(ins, CODE[dtype], ring=ring)
        assert np.array_equal(a[0], b[0])
        # (ring order, rounding once, sum) is the binary32-accumulation variant
        assert np.array_equal(orc.allreduce_fp32acc(ins, CODE[dtype], ring=ring)[0],
                              orc.allreduce_var(ins, CODE[dtype], ring=ring, rounding=orc.ROUND_ONCE)[0])
        for op in (orc.PROD, orc.MAX):
            for order in (orc.ORDER_RING, orc.ORDER_TREE):
                ar = orc.allreduce_var(ins, CODE[dtype], op=op, ring=ring, order=order)
                rs = orc.reduce_scatter_var(ins, CODE[dtype], op=op, ring=ring, order=order)
                for r in range(W):
                    assert np.array_equal(ar[r], ar[0])
                    assert np.array_equal(rs[r], ar[0][r * n:(r + 1) * n])
                    red = orc.reduce_var(ins, CODE[dtype], r, op=op, ring=ring, order=order)
                    assert np.array_equal(red[r * n:(r + 1) * n], ar[0][r * n:(r + 1) * n])
            # ring replay with the operator: Reduce-Scatter and Reduce agree with the All-Reduce
            ar = orc.allreduce(ins, CODE[dtype], ring=ring, op=op)
            rs = orc.reduce_scatter(ins, CODE[dtype], ring=ring, op=op)
            for r in range(W):
                assert np.array_equal(rs[r], ar[0][r * n:(r + 1) * n])
                red = orc.reduce(ins, CODE[dtype], r, ring=ring, op=op)
                assert np.array_equal(red[r * n:(r + 1) * n], ar[0][r * n:(r + 1) * n])


def test_three_rank_tree_is_the_left_fold_of_the_block_that_starts_at_ring_zero():
    """For W = 3 the tree (v0 v1) v2 over ring order is the ring's own left fold for the block
    whose sum starts at ring[0], i.e. block ring[2]."""
    rng = np.random.Generator(np.random.Philox(306))
    ring = [1, 2, 0]
    n = 999
    for dtype in ("bf16", "fp16", "fp32"):
        ins = [_from_values(rng.standard_normal(3 * n), dtype) for _ in range(3)]
        tree = orc.allreduce_var(ins, CODE[dtype], ring=ring, order=orc.ORDER_TREE)[0]
        ringres = orc.allreduce(ins, CODE[dtype], ring=ring)[0]
        c = ring[2]
        assert np.array_equal(tree[c * n:(c + 1) * n], ringres[c * n:(c + 1) * n])
        assert not np.array_equal(tree, ringres)


# ------------------------------------------------------------ error bounds
@pytest.mark.parametrize("dtype,fb", [("bf16", 7), ("fp16", 10)])
@pytest.mark.parametrize("W", [4, 8, 16])
def test_tree_sum_error_bounds(dtype, fb, W):
    """Rounding once (binary32 intermediates): within 2 ulp of the correctly rounded exact sum,
    the tolerance stated for reordered variants (in fact within one ulp).
    Per-node rounding: the pairwise-summation bound |got - exact| <= ((1+u)^d - 1) * sum|x|,
    d = ceil(log2 W) levels, u = half an ulp of 1 -- tighter than the ring's W-1 roundings in a
    row, but not a 2-ulp statement: like the ring itself it is checked bit for bit instead."""
    rng = np.random.Generator(np.random.Philox(310 + W))
    count = 20_000
    ins = [_from_values(rng.standard_normal(count), dtype) for _ in range(W)]
    vals = np.array([_to_values(a, dtype) for a in ins])
    exact = vals.sum(axis=0)
    ref = _to_values(_from_values(exact, dtype), dtype)
    once = _to_values(orc.allreduce_var(ins, CODE[dtype], order=orc.ORDER_TREE, rounding=orc.ROUND_ONCE)[0], dtype)
    big = np.maximum(np.abs(ref), np.abs(vals).max(axis=0))
    ulp = np.exp2(np.floor(np.log2(np.maximum(big, 1e-30))) - fb)
    assert np.all(np.abs(once - ref) <= 2 * ulp)
    assert np.all(np.abs(once - ref) <= np.exp2(np.floor(np.log2(np.maximum(np.abs(ref), 1e-30))) - fb))
    each = _to_values(orc.allreduce_var(ins, CODE[dtype], order=orc.ORDER_TREE, rounding=orc.ROUND_EACH)[0], dtype)
    u = 2.0 ** -(fb + 1)
    d = int(np.ceil(np.log2(W)))
    assert np.all(np.abs(each - exact) <= ((1 + u) ** d - 1) * np.abs(vals).sum(axis=0))
    # per-node rounding in tree order loses less than the ring's W-1 roundings in a row, on average
    ring = _to_values(orc.allreduce(ins, CODE[dtype])[0], dtype)
    assert np.abs(each - exact).mean() < np.abs(ring - exact).mean()
    assert np.abs(once - exact).mean() <= np.abs(each - exact).mean()


@pytest.mark.parametrize("W", [4, 8, 16])
def test_tree_sum_fp32_within_relative_tolerance(W):
    rng = np.random.Generator(np.random.Philox(320 + W))
    count = 50_000
    ins = [rng.uniform(-1, 1, count).astype(np.float32) for _ in range(W)]
    vals = np.array([a.astype(np.float64) for a in ins])
    exact = vals.sum(axis=0)
    got = orc.allreduce_var(ins, orc.FP32, order=orc.ORDER_TREE)[0].astype(np.float64)
    assert np.all(np.abs(got - exact) <= 1e-6 * np.abs(vals).sum(axis=0))


# ------------------------------------------------------------ planted mistakes
def test_pins_catch_planted_mistakes():
    """A maximum that returns the non-NaN operand, a maximum that ignores the sign of zero, a
    tree that folds from the left, and a product that rounds through the wire type twice are
    each told apart from the oracle by the fixtures above."""
    rows = _rows("minmax_specials.txt")
    dtype = "fp32"
    a = _wire_of_bits([_sym(r[0], dtype) for r in rows], dtype)
    b = _wire_of_bits([_sym(r[1], dtype) for r in rows], dtype)
    want = _wire_of_bits([_sym(r[2], dtype) for r in rows], dtype)
    with np.errstate(all="ignore"):
        wrong_nan = np.fmax(a, b)                                  # drops NaN operands
    assert np.isnan(want).sum() > np.isnan(wrong_nan).sum()
    wrong_zero = np.where(a >= b, a, b)                            # picks a for (-0, +0)
    assert not np.array_equal(np.signbit(wrong_zero), np.signbit(want))
    ins = [_from_values([v] * 5, "bf16") for v in (256.0, 1.0, 1.0, 1.0, 1.0)]
    left_fold = orc.allreduce_var(ins, orc.BF16, ring=[0, 1, 2, 3, 4])[4]
    assert _to_values(left_fold, "bf16")[4] != 260.0
