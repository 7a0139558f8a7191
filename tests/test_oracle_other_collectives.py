"""Pins for the oracle's Reduce, Broadcast and All-to-All (CPU only)."""
import random

import numpy as np
import pytest

import brute
from oracle import ring_oracle as orc
from test_oracle_ring import CODE, _bits, _from_values, _golden_rows, _random_wire, _to_values


@pytest.mark.parametrize("dtype", ["fp32", "bf16", "fp16", "int32"])
def test_reduce_matches_brute_force_on_tiny_inputs(dtype):
    rng = np.random.Generator(np.random.Philox(70))
    rnd = random.Random(70)
    for W in (1, 2, 3, 4, 5):
        for count in (0, 1, 5, 33):
            ring = list(range(W))
            rnd.shuffle(ring)
            ins = [_random_wire(rng, count, dtype) for _ in range(W)]
            lists = [a.tolist() if dtype == "int32" else _bits(a, dtype) for a in ins]
            for root in range(W):
                for use_ring in (None, ring):
                    want = brute.reduce(lists, dtype, root, ring=use_ring)
                    for chunk in (0, 2):
                        got = orc.reduce(ins, CODE[dtype], root, ring=use_ring, chunk_elems=chunk)
                        got = got.tolist() if dtype == "int32" else _bits(got, dtype)
                        assert got == want, (dtype, W, count, root, use_ring, chunk)


@pytest.mark.parametrize("dtype,M,blocks", _golden_rows())
def test_reduce_on_the_cancellation_example(dtype, M, blocks):
    # reducing to root c sums in the order c+1, ..., c: the value block c of the All-Reduce holds
    ranks = [_from_values([v] * 8, dtype) for v in (M, 1.0, -M, 1.0)]
    for root in range(4):
        out = _to_values(orc.reduce(ranks, CODE[dtype], root), dtype)
        assert np.all(out == blocks[root])


@pytest.mark.parametrize("dtype", ["fp32", "bf16", "fp16", "int32"])
def test_reduce_agrees_with_allreduce_block_of_the_root_and_with_exact_sums(dtype):
    rng = np.random.Generator(np.random.Philox(71))
    W, n = 6, 500
    ring = [4, 2, 0, 5, 3, 1]
    ins = [_random_wire(rng, W * n, dtype) for _ in range(W)]
    ar = orc.allreduce(ins, CODE[dtype], ring=ring)[0]
    for root in range(W):
        red = orc.reduce(ins, CODE[dtype], root, ring=ring)
        a, b = red[root * n:(root + 1) * n], ar[root * n:(root + 1) * n]
        if dtype == "int32":
            assert np.array_equal(a, b)
        else:
            va, vb = _to_values(a, dtype), _to_values(b, dtype)
            assert np.array_equal(np.isnan(va), np.isnan(vb)) and np.array_equal(va[~np.isnan(va)], vb[~np.isnan(vb)])
    ints = [rng.integers(-8, 9, size=999) for _ in range(W)]
    out = orc.reduce([_from_values(v, dtype) for v in ints], CODE[dtype], 3, ring=ring)
    assert np.array_equal(_to_values(out, dtype), np.sum(ints, axis=0).astype(np.float64))


@pytest.mark.parametrize("dtype", ["fp32", "bf16", "fp16"])
def test_reduce_two_ranks_is_the_library_add(dtype):
    rng = np.random.Generator(np.random.Philox(72))
    a = _from_values(rng.standard_normal(10_001), dtype)
    b = _from_values(rng.standard_normal(10_001) * 1e-2, dtype)
    want = orc.allreduce([a, b], CODE[dtype])[0]        # pinned to numpy / torch adds elsewhere
    for root in (0, 1):
        assert np.array_equal(orc.reduce([a, b], CODE[dtype], root), want)


@pytest.mark.parametrize("dtype", ["fp32", "bf16", "fp16", "int32"])
def test_broadcast_and_alltoall_are_their_definitions(dtype):
    rng = np.random.Generator(np.random.Philox(73))
    for W in (1, 2, 5, 16):
        n = 37
        ins = [_random_wire(rng, W * n, dtype) for _ in range(W)]
        for root in (0, W - 1):
            ring = list(range(W))
            random.Random(W).shuffle(ring)
            for o in orc.broadcast(ins[root], CODE[dtype], W, root, ring=ring):
                assert np.array_equal(_bits(o, dtype), _bits(ins[root], dtype))
        out = orc.alltoall(ins, CODE[dtype])
        # block transpose: stack to (rank, block, n), swap the first two axes
        cube = np.stack([a.reshape(W, n) for a in ins])
        want = cube.transpose(1, 0, 2)
        for r in range(W):
            assert np.array_equal(out[r].reshape(W, n).view(np.uint8), want[r].view(np.uint8))
        # applying it twice gives the input back
        back = orc.alltoall(out, CODE[dtype])
        assert all(np.array_equal(_bits(x, dtype), _bits(y, dtype)) for x, y in zip(back, ins))
