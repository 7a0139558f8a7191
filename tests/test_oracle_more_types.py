"""Pins for the further wire types of the oracle (CPU only): fp64, int64, uint8 --
exact-rational / big-integer brute force, library routines for two ranks, exact
integer sums, order independence of the integer types, and the invariants."""
import random

import numpy as np
import pytest

import brute
from oracle import ring_oracle as orc
from test_oracle_ring import CODE, _bits, _from_values, _random_wire, _to_values

OPS = {"sum": orc.SUM, "prod": orc.PROD, "max": orc.MAX, "min": orc.MIN}
TYPES = ["fp64", "int64", "uint8"]


def _rand(rng, n, dtype):
    if dtype == "fp64":
        # wide exponent spread, a few specials: infinities, NaN, zeros of both signs, subnormals
        v = rng.standard_normal(n) * np.exp2(rng.integers(-40, 41, size=n).astype(np.float64))
        pick = rng.random(n)
        v = np.where(pick < 0.02, np.inf, v)
        v = np.where((pick >= 0.02) & (pick < 0.04), -np.inf, v)
        v = np.where((pick >= 0.04) & (pick < 0.06), np.nan, v)
        v = np.where((pick >= 0.06) & (pick < 0.08), -0.0, v)
        v = np.where((pick >= 0.08) & (pick < 0.10), 5e-324 * rng.integers(1, 1000, size=n), v)
        return v.astype(np.float64)
    return _random_wire(rng, n, dtype)


def _same(got, want, dtype):
    if dtype != "fp64":
        return list(got) == list(want)
    nan = lambda b: (b & 0x7FFFFFFFFFFFFFFF) > 0x7FF0000000000000
    return all(g == w or (nan(g) and nan(w)) for g, w in zip(got, want))


@pytest.mark.parametrize("dtype", TYPES)
@pytest.mark.parametrize("op", ["sum", "prod", "max", "min"])
def test_ring_matches_brute_force(dtype, op):
    rng = np.random.Generator(np.random.Philox(400))
    rnd = random.Random(400)
    for W in (1, 2, 3, 5):
        for count in (0, 1, 7, 33):
            ring = list(range(W))
            rnd.shuffle(ring)
            ins = [_rand(rng, count, dtype) for _ in range(W)]
            for use_ring in (None, ring):
                want = brute.allreduce_var([_bits(a, dtype) for a in ins], dtype, op=op, ring=use_ring)
                for chunk in (0, 3):
                    for o in orc.allreduce(ins, CODE[dtype], ring=use_ring, chunk_elems=chunk, op=OPS[op]):
                        assert _same(_bits(o, dtype), want, dtype), (dtype, op, W, count, use_ring, chunk)
                tree = brute.allreduce_var([_bits(a, dtype) for a in ins], dtype, op=op, ring=use_ring, order="tree")
                got = orc.allreduce_var(ins, CODE[dtype], op=OPS[op], ring=use_ring, order=orc.ORDER_TREE)
                assert _same(_bits(got[0], dtype), tree, dtype)
                # the wire type is its own accumulation type: rounding once changes nothing
                once = orc.allreduce_var(ins, CODE[dtype], op=OPS[op], ring=use_ring, order=orc.ORDER_TREE,
                                         rounding=orc.ROUND_ONCE)
                assert _same(_bits(once[0], dtype), tree, dtype)


@pytest.mark.parametrize("dtype", TYPES)
def test_two_ranks_equal_the_library_elementwise_operation(dtype):
    rng = np.random.Generator(np.random.Philox(401))
    n = 100_000
    x, y = _rand(rng, n, dtype), _rand(rng, n, dtype)
    with np.errstate(all="ignore"):
        lib = {"sum": x + y, "prod": x * y, "max": np.maximum(x, y), "min": np.minimum(x, y)}   # integer types wrap
    for name, want in lib.items():
        got = orc.allreduce([x, y], CODE[dtype], op=OPS[name])[0]
        gb, wb = _bits(got, dtype), _bits(np.ascontiguousarray(want), dtype)
        if dtype == "fp64" and name in ("max", "min"):
            zero = lambda b: 0 if (b & 0x7FFFFFFFFFFFFFFF) == 0 else b   # the library may pick either zero
            gb, wb = [zero(b) for b in gb], [zero(b) for b in wb]
        assert _same(gb, wb, dtype), (dtype, name)


@pytest.mark.parametrize("dtype", ["int64", "uint8"])
def test_integer_types_equal_big_integer_arithmetic_in_any_order(dtype):
    rng = np.random.Generator(np.random.Philox(402))
    W, n = 7, 501
    bits, signed = brute.INT[dtype]
    ins = [_rand(rng, W * n, dtype) for _ in range(W)]
    cols = [[int(a[i]) for a in ins] for i in range(W * n)]
    def wrap(v):
        v &= (1 << bits) - 1
        return v - (1 << bits) if signed and v >= (1 << (bits - 1)) else v
    prod = lambda c: wrap(int(np.prod(np.array(c, dtype=object))))
    want = {"sum": [wrap(sum(c)) for c in cols], "prod": [prod(c) for c in cols],
            "max": [max(c) for c in cols], "min": [min(c) for c in cols]}
    ring = [3, 1, 4, 0, 6, 2, 5]
    for name, w in want.items():
        for out in (orc.allreduce(ins, CODE[dtype], op=OPS[name])[0],
                    orc.allreduce(ins, CODE[dtype], ring=ring, chunk_elems=17, op=OPS[name])[3],
                    orc.allreduce_var(ins, CODE[dtype], op=OPS[name], ring=ring, order=orc.ORDER_TREE)[6]):
            assert [int(v) for v in out] == w, (dtype, name)


def test_fp64_small_integers_sum_exactly_and_bound_against_exact_sum():
    rng = np.random.Generator(np.random.Philox(403))
    ints = [rng.integers(-1000, 1001, size=3000) for _ in range(16)]
    out = orc.allreduce([v.astype(np.float64) for v in ints], orc.FP64)[0]
    assert np.array_equal(out, np.sum(ints, axis=0).astype(np.float64))
    # W - 1 roundings of at most half an ulp of the largest partial each
    W, n = 8, 20_000
    vals = [rng.standard_normal(n) for _ in range(W)]
    got = orc.allreduce(vals, orc.FP64)[0]
    import fractions
    for i in range(0, n, 997):
        exact = sum(fractions.Fraction(v[i]) for v in vals)
        order = [(i // (n // W) + 1 + k) % W for k in range(W)]
        acc, big = 0.0, 0.0
        for r in order:
            acc += vals[r][i]
            big = max(big, abs(acc))
        assert acc == got[i]                                     # numpy's own doubles, same order
        assert abs(fractions.Fraction(got[i]) - exact) <= (W - 1) * fractions.Fraction(np.spacing(big)) / 2


@pytest.mark.parametrize("dtype", TYPES)
def test_invariants(dtype):
    rng = np.random.Generator(np.random.Philox(404))
    W, n = 6, 700
    ring = [5, 0, 3, 1, 4, 2]
    ins = [_rand(rng, W * n, dtype) if dtype != "fp64" else rng.standard_normal(W * n) for _ in range(W)]
    ar = orc.allreduce(ins, CODE[dtype], ring=ring, chunk_elems=64)
    for r in range(W):
        assert np.array_equal(ar[r], ar[0])
    rs = orc.reduce_scatter(ins, CODE[dtype], ring=ring)
    ag = orc.all_gather(rs, CODE[dtype], ring=ring, chunk_elems=9)
    for r in range(W):
        assert np.array_equal(rs[r], ar[0][r * n:(r + 1) * n])
        assert np.array_equal(ag[r], ar[0])
        assert np.array_equal(orc.reduce(ins, CODE[dtype], r, ring=ring)[r * n:(r + 1) * n], rs[r])
    assert all(np.array_equal(o, ins[2]) for o in orc.broadcast(ins[2], CODE[dtype], W, 2, ring=ring))
    a2a = orc.alltoall(ins, CODE[dtype])
    for r in range(W):
        for q in range(W):
            assert np.array_equal(a2a[r][q * n:(q + 1) * n], ins[q][r * n:(r + 1) * n])
    # the binary32-accumulation entry points do not exist for these types
    with pytest.raises(ValueError):
        orc.allreduce_fp32acc(ins, CODE[dtype])
