"""Pins for the binary32-accumulation variant (CPU only): exact-rational brute
force, equality with the ring where the two coincide, and the 2-ulp bound
against the correctly rounded exact sum."""
import random

import numpy as np
import pytest

import brute
from oracle import ring_oracle as orc
from test_oracle_ring import CODE, _bits, _from_values, _random_wire, _to_values


@pytest.mark.parametrize("dtype", ["fp32", "bf16", "fp16"])
def test_fp32acc_matches_brute_force_on_tiny_inputs(dtype):
    rng = np.random.Generator(np.random.Philox(90))
    rnd = random.Random(90)
    for W in (1, 2, 3, 5):
        for count in (0, 1, 7, 40):
            ring = list(range(W))
            rnd.shuffle(ring)
            ins = [_random_wire(rng, count, dtype) for _ in range(W)]
            for use_ring in (None, ring):
                want = brute.allreduce_fp32acc([_bits(a, dtype) for a in ins], dtype, ring=use_ring)
                out = orc.allreduce_fp32acc(ins, CODE[dtype], ring=use_ring)
                for o in out:
                    assert _bits(o, dtype) == want, (dtype, W, count, use_ring)


@pytest.mark.parametrize("dtype", ["fp32", "int32"])
def test_fp32acc_equals_the_ring_for_four_byte_types(dtype):
    rng = np.random.Generator(np.random.Philox(91))
    W, n = 7, 1001
    ins = [_random_wire(rng, W * n, dtype) for _ in range(W)]
    ring = [3, 1, 4, 0, 6, 2, 5]
    a = orc.allreduce(ins, CODE[dtype], ring=ring)[0]
    b = orc.allreduce_fp32acc(ins, CODE[dtype], ring=ring)[0]
    assert np.array_equal(_bits(a, dtype), _bits(b, dtype)) if dtype == "fp32" else np.array_equal(a, b)


@pytest.mark.parametrize("dtype", ["bf16", "fp16"])
def test_fp32acc_two_ranks_equals_the_ring_and_entry_points_agree(dtype):
    rng = np.random.Generator(np.random.Philox(92))
    a, b = (_from_values(rng.standard_normal(5000), dtype) for _ in range(2))
    assert np.array_equal(orc.allreduce_fp32acc([a, b], CODE[dtype])[0], orc.allreduce([a, b], CODE[dtype])[0])
    W, n = 4, 600
    ins = [_from_values(rng.standard_normal(W * n), dtype) for _ in range(W)]
    ring = [2, 0, 3, 1]
    ar = orc.allreduce_fp32acc(ins, CODE[dtype], ring=ring)
    rs = orc.reduce_scatter_fp32acc(ins, CODE[dtype], ring=ring)
    for r in range(W):
        assert np.array_equal(ar[r], ar[0])
        assert np.array_equal(rs[r], ar[0][r * n:(r + 1) * n])
        red = orc.reduce_fp32acc(ins, CODE[dtype], r, ring=ring)
        assert np.array_equal(red[r * n:(r + 1) * n], ar[0][r * n:(r + 1) * n])


@pytest.mark.parametrize("dtype,fb", [("bf16", 7), ("fp16", 10)])
@pytest.mark.parametrize("W", [4, 8, 16])
def test_fp32acc_within_two_ulp_of_the_correctly_rounded_exact_sum(dtype, fb, W):
    rng = np.random.Generator(np.random.Philox(93 + W))
    count = 20_000
    ins = [_from_values(rng.standard_normal(count), dtype) for _ in range(W)]
    got = _to_values(orc.allreduce_fp32acc(ins, CODE[dtype])[0], dtype)
    vals = np.array([_to_values(a, dtype) for a in ins])
    exact = vals.sum(axis=0)                                   # float64: exact for these magnitudes
    ref = _to_values(_from_values(exact, dtype), dtype)        # rounded once by the library conversion
    # ulp of the largest magnitude met on the way (bounds every prefix sum)
    big = np.maximum(np.abs(ref), np.abs(np.cumsum(vals, axis=0)).max(axis=0))
    ulp = np.exp2(np.floor(np.log2(np.maximum(big, 1e-30))) - fb)
    assert np.all(np.abs(got - ref) <= 2 * ulp)
    # and it is at least as close to the exact sum as the per-hop ring is, on average
    ring = _to_values(orc.allreduce(ins, CODE[dtype])[0], dtype)
    assert np.abs(got - exact).mean() <= np.abs(ring - exact).mean()


def test_fp32acc_small_integers_exact():
    rng = np.random.Generator(np.random.Philox(94))
    for dtype in ("fp32", "bf16", "fp16", "int32"):
        ints = [rng.integers(-8, 9, size=2000) for _ in range(16)]
        out = orc.allreduce_fp32acc([_from_values(v, dtype) for v in ints], CODE[dtype])[0]
        assert np.array_equal(_to_values(out, dtype), np.sum(ints, axis=0).astype(np.float64))
