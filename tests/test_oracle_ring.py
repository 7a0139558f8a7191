"""Pins for the oracle's ring replay (CPU only): block tables, fold order,
brute force on tiny inputs, closed forms, invariants, library special cases."""
import os
import random

import numpy as np
import pytest
import torch

import brute
from oracle import ring_oracle as orc

CODE = {"fp32": orc.FP32, "bf16": orc.BF16, "fp16": orc.FP16, "int32": orc.INT32,
        "fp64": orc.FP64, "int64": orc.INT64, "uint8": orc.UINT8}
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _from_values(vals, dtype):
    """float values -> wire array, using library conversions (not the oracle's)."""
    v = np.asarray(vals, dtype=np.float64)
    if dtype == "fp32":
        return v.astype(np.float32)
    if dtype == "fp16":
        return v.astype(np.float16).view(np.uint16)
    if dtype == "bf16":
        return torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    if dtype == "fp64":
        return v.copy()
    if dtype == "int64":
        return v.astype(np.int64)
    if dtype == "uint8":
        return v.astype(np.int64).astype(np.uint8)      # wraps modulo 256
    return v.astype(np.int32)


def _to_values(a, dtype):
    if dtype == "fp16":
        return a.view(np.float16).astype(np.float64)
    if dtype == "bf16":
        return torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16).double().numpy()
    return a.astype(np.float64)


def _bits(a, dtype):
    if dtype == "fp32":
        return [int(x) for x in a.view(np.uint32)]
    if dtype == "fp64":
        return [int(x) for x in a.view(np.uint64)]
    return [int(x) for x in a]


# ------------------------------------------------------------ block tables
@pytest.mark.parametrize("W", list(range(2, 17)))
def test_block_tables_by_set_simulation(W):
    """Simulate who has contributed to which block, using only the send/recv
    tables: after Reduce-Scatter rank r's block r holds every rank once, in the
    order next(r) ... r; after All-Gather every rank holds every finished block."""
    rnd = random.Random(100 + W)
    for trial in range(4):
        ring = list(range(W))
        if trial:
            rnd.shuffle(ring)
        nxt = {ring[k]: ring[(k + 1) % W] for k in range(W)}
        held = [[(r,) for _ in range(W)] for r in range(W)]     # held[r][block] = contributors, in order
        touched = [set() for _ in range(W)]
        for s in range(W - 1):
            tab = [orc.ring_step(W, ring, orc.PHASE_RS, s, r) for r in range(W)]
            msgs = {}
            for r in range(W):
                sb, _ = tab[r]
                assert tab[nxt[r]][1] == sb          # what r sends is what next(r) expects
                msgs[nxt[r]] = held[r][sb]
            for r in range(W):
                rb = tab[r][1]
                assert rb not in touched[r]          # own data of a block is used once
                touched[r].add(rb)
                assert r not in msgs[r]
                held[r][rb] = msgs[r] + (r,)
        for r in range(W):
            p = ring.index(r)
            assert list(held[r][r]) == [ring[(p + k) % W] for k in range(1, W + 1)]
            assert len(touched[r]) == W - 1 and ring[(p - 1) % W] not in touched[r]
        done = [{r: held[r][r]} for r in range(W)]
        for s in range(W - 1):
            tab = [orc.ring_step(W, ring, orc.PHASE_AG, s, r) for r in range(W)]
            msgs = {}
            for r in range(W):
                sb, _ = tab[r]
                assert tab[nxt[r]][1] == sb and sb in done[r]
                msgs[nxt[r]] = (sb, done[r][sb])
            for r in range(W):
                b, v = msgs[r]
                assert b == tab[r][1] and b not in done[r]
                done[r][b] = v
        for r in range(W):
            assert sorted(done[r]) == list(range(W))
            assert all(done[r][b] == held[b][b] for b in range(W))


def test_identity_ring_tables_match_closed_form():
    for W in (2, 4, 8, 16):
        for r in range(W):
            for s in range(W - 1):
                assert orc.ring_step(W, None, orc.PHASE_RS, s, r) == ((r - s - 1) % W, (r - s - 2) % W)
                assert orc.ring_step(W, None, orc.PHASE_AG, s, r) == ((r - s) % W, (r - s - 1) % W)


def test_ring_step_rejects_bad_arguments():
    for args in [(4, [0, 1, 2, 2], 0, 0, 0), (4, None, 0, 3, 0), (4, None, 2, 0, 0), (4, None, 0, 0, 4), (0, None, 0, 0, 0)]:
        with pytest.raises((ValueError, AssertionError)):
            orc.ring_step(*args)


# ------------------------------------------------------------ worked example
def _golden_rows():
    rows = []
    with open(os.path.join(GOLDEN, "cancellation_w4.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                t = line.split()
                rows.append((t[0], float(t[1]), [float(x) for x in t[2:6]]))
    return rows


@pytest.mark.parametrize("dtype,M,blocks", _golden_rows())
def test_cancellation_example(dtype, M, blocks):
    n = 16
    ranks = [_from_values([v] * n, dtype) for v in (M, 1.0, -M, 1.0)]
    out = orc.allreduce(ranks, CODE[dtype])
    want = np.repeat(np.array(blocks), n // 4)
    for o in out:
        assert np.array_equal(_to_values(o, dtype), want)
    # the brute force agrees, and other conventions would not: the example discriminates
    got_brute = brute.allreduce([_bits(r, dtype) for r in ranks], dtype)
    assert got_brute == _bits(out[0], dtype)
    start_at_c = []
    for c in range(4):
        order = [(c + k) % 4 for k in range(4)]
        acc = _bits(ranks[order[0]], dtype)[0]
        for r in order[1:]:
            acc = brute.hop(acc, _bits(ranks[r], dtype)[0], dtype)
        start_at_c.append(acc)
    assert start_at_c != [_bits(out[0], dtype)[c * 4] for c in range(4)]
    rev = brute.allreduce([_bits(r, dtype) for r in ranks], dtype, ring=[0, 3, 2, 1])
    assert rev != got_brute


# ------------------------------------------------------------ brute force
def _random_wire(rng, n, dtype):
    if dtype == "int32":
        return rng.integers(-2**31, 2**31, size=n, dtype=np.int64).astype(np.int32)
    if dtype == "int64":
        return rng.integers(-2**63, 2**63 - 1, size=n, dtype=np.int64, endpoint=True)
    if dtype == "uint8":
        return rng.integers(0, 256, size=n, dtype=np.int64).astype(np.uint8)
    # moderate exponent spread so that most additions round; a few huge / tiny values
    mant = rng.standard_normal(n) * np.exp2(rng.integers(-3, 4, size=n))
    if dtype == "fp16":
        mant = np.where(rng.random(n) < 0.1, mant * 1e4, mant)       # overflow region
        mant = np.where(rng.random(n) < 0.1, mant * 1e-7, mant)      # subnormal region
    return _from_values(mant, dtype)


@pytest.mark.parametrize("dtype", ["fp32", "bf16", "fp16", "int32"])
def test_allreduce_matches_brute_force_on_tiny_inputs(dtype):
    rng = np.random.Generator(np.random.Philox(7))
    rnd = random.Random(7)
    for W in (1, 2, 3, 4, 5):
        for count in (0, 1, 2, 3, 5, 8, 13, 64):
            ring = list(range(W))
            rnd.shuffle(ring)
            for use_ring in (None, ring):
                ins = [_random_wire(rng, count, dtype) for _ in range(W)]
                want = brute.allreduce([_bits(a, dtype) if dtype != "int32" else a.tolist() for a in ins],
                                       dtype, ring=use_ring)
                for chunk in (0, 1, 3):
                    out = orc.allreduce(ins, CODE[dtype], ring=use_ring, chunk_elems=chunk)
                    for o in out:
                        got = o.tolist() if dtype == "int32" else _bits(o, dtype)
                        assert got == want, (dtype, W, count, use_ring, chunk)


# ------------------------------------------------------------ closed forms
@pytest.mark.parametrize("dtype", ["fp32", "bf16", "fp16", "int32"])
@pytest.mark.parametrize("W", [2, 3, 8, 16])
def test_small_integer_inputs_give_exact_sums(dtype, W):
    # |v| <= 8 and W <= 16 keep every partial sum an integer below 2^8, exact in all four types
    rng = np.random.Generator(np.random.Philox(W))
    count = 1000 + W
    ints = [rng.integers(-8, 9, size=count) for _ in range(W)]
    out = orc.allreduce([_from_values(v, dtype) for v in ints], CODE[dtype])
    want = np.sum(ints, axis=0).astype(np.float64)
    for o in out:
        assert np.array_equal(_to_values(o, dtype), want)
    # constants: every rank 1 -> W ; rank r filled with r+1 -> W(W+1)/2
    ones = orc.allreduce([_from_values(np.ones(count), dtype) for _ in range(W)], CODE[dtype])
    assert np.all(_to_values(ones[0], dtype) == W)
    ramp = orc.allreduce([_from_values(np.full(count, r + 1.0), dtype) for r in range(W)], CODE[dtype])
    assert np.all(_to_values(ramp[W - 1], dtype) == W * (W + 1) / 2)


def test_int32_equals_wrapped_int64_sum_for_any_ring_and_chunk():
    rng = np.random.Generator(np.random.Philox(5))
    W, count = 7, 10_003
    ins = [rng.integers(-2**31, 2**31, size=count, dtype=np.int64).astype(np.int32) for _ in range(W)]
    want = (np.sum([a.astype(np.int64) for a in ins], axis=0) & 0xFFFFFFFF).astype(np.uint32).view(np.int32)
    for ring in (None, [3, 1, 4, 0, 6, 2, 5]):
        for chunk in (0, 17, 4096):
            for o in orc.allreduce(ins, orc.INT32, ring=ring, chunk_elems=chunk):
                assert np.array_equal(o, want)


# ------------------------------------------------------------ library special case
@pytest.mark.parametrize("dtype", ["fp32", "bf16", "fp16"])
def test_two_ranks_equal_library_elementwise_add(dtype):
    rng = np.random.Generator(np.random.Philox(9))
    n = 200_001
    a = _from_values(rng.standard_normal(n) * 100, dtype)
    b = _from_values(rng.standard_normal(n) * 0.37, dtype)
    out = orc.allreduce([a, b], CODE[dtype])
    if dtype == "fp32":
        want = (a + b).view(np.uint32)
        got = [o.view(np.uint32) for o in out]
    elif dtype == "fp16":
        want = (a.view(np.float16) + b.view(np.float16)).view(np.uint16)
        got = out
    else:
        ta = torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16)
        tb = torch.from_numpy(b.view(np.int16).copy()).view(torch.bfloat16)
        want = (ta + tb).view(torch.int16).numpy().view(np.uint16)
        got = out
    assert np.array_equal(got[0], want) and np.array_equal(got[1], want)


# ------------------------------------------------------------ invariants
@pytest.mark.parametrize("dtype", ["fp32", "bf16", "fp16", "int32"])
def test_invariants(dtype):
    rng = np.random.Generator(np.random.Philox(13))
    W, n = 6, 999                          # block = 999 elements, vector = 5994
    ring = [2, 0, 5, 1, 4, 3]
    if dtype == "int32":
        ins = [rng.integers(-1000, 1001, size=W * n).astype(np.int32) for _ in range(W)]
    else:
        ins = [_from_values(rng.standard_normal(W * n) * 1e-3, dtype) for _ in range(W)]
    keep = [a.copy() for a in ins]
    ar = orc.allreduce(ins, CODE[dtype], ring=ring, chunk_elems=100)
    assert all(np.array_equal(a, b) for a, b in zip(ins, keep))          # inputs untouched
    assert all(np.array_equal(ar[0], o) for o in ar[1:])                 # every rank identical
    # result does not depend on the chunk size
    for chunk in (0, 1, 7, 998, 999, 5000):
        assert np.array_equal(orc.allreduce(ins, CODE[dtype], ring=ring, chunk_elems=chunk)[0], ar[0])
    # All-Reduce == All-Gather after Reduce-Scatter (count divisible by W: same block map)
    rs = orc.reduce_scatter(ins, CODE[dtype], ring=ring, chunk_elems=64)
    for r in range(W):
        assert np.array_equal(rs[r], ar[0][r * n:(r + 1) * n])
    ag = orc.all_gather(rs, CODE[dtype], ring=ring, chunk_elems=64)
    assert all(np.array_equal(o, ar[0]) for o in ag)
    # All-Gather alone is concatenation
    parts = [a[:n] for a in ins]
    for o in orc.all_gather(parts, CODE[dtype], ring=ring):
        assert np.array_equal(o, np.concatenate(parts))
    # W = 1 is the identity
    assert np.array_equal(orc.allreduce([ins[0]], CODE[dtype])[0], ins[0])


@pytest.mark.parametrize("dtype,ulp_bits", [("fp32", 23), ("bf16", 7), ("fp16", 10)])
def test_ring_result_within_rounding_bound_of_exact_sum(dtype, ulp_bits):
    """|ring - exact| <= (W-1) * half an ulp of the largest partial sum (a loose
    form of 'within the numerical tolerance of BF16', Section 5.3 'Model Accuracy')."""
    rng = np.random.Generator(np.random.Philox(17))
    W, count = 8, 8000
    ins = [_from_values(rng.standard_normal(count), dtype) for _ in range(W)]
    out = _to_values(orc.allreduce(ins, CODE[dtype])[0], dtype)
    vals = np.array([_to_values(a, dtype) for a in ins])
    exact = vals.sum(axis=0)
    biggest = np.abs(vals).sum(axis=0)                       # bounds every partial sum
    half_ulp = np.exp2(np.floor(np.log2(biggest)) - ulp_bits - 1)
    assert np.all(np.abs(out - exact) <= (W - 1) * half_ulp)
    assert np.any(out != exact) or dtype == "fp32"          # rounding really happens in 16 bits


def test_float_result_depends_on_ring_order_as_the_fold_predicts():
    # relabelling the ring changes which rank starts each block's sum
    ins = [_from_values([v] * 8, "bf16") for v in (256.0, 1.0, -256.0, 1.0)]
    a = _to_values(orc.allreduce(ins, orc.BF16, ring=[0, 1, 2, 3])[0], "bf16")
    b = _to_values(orc.allreduce(ins, orc.BF16, ring=[0, 3, 2, 1])[0], "bf16")
    assert a.tolist() == [2, 2, 2, 2, 0, 0, 1, 1]
    want_b = brute.allreduce([_bits(x, "bf16") for x in ins], "bf16", ring=[0, 3, 2, 1])
    assert _bits(orc.allreduce(ins, orc.BF16, ring=[0, 3, 2, 1])[0], "bf16") == want_b
    assert a.tolist() != b.tolist()


def test_specials_propagate():
    inf, nan = np.inf, np.nan
    cols = np.array([[inf, 1, 1, 1], [inf, -inf, 0, 0], [nan, 1, 2, 3], [65504, 65504, 0, 0],
                     [-0.0, -0.0, -0.0, -0.0], [0.0, -0.0, -0.0, -0.0], [6e-8, 6e-8, 0, 0]]).T
    ins = [_from_values(cols[r], "fp16") for r in range(4)]
    out = orc.allreduce(ins, orc.FP16)[0].view(np.float16)
    # count = 7, W = 4 -> blocks of 2: every element still sees all four ranks
    assert out[0] == inf and np.isnan(out[1]) and np.isnan(out[2]) and out[3] == inf
    assert out[4] == 0 and np.signbit(out[4]) and out[5] == 0 and not np.signbit(out[5])
    assert out[6] == np.float16(6e-8) + np.float16(6e-8)     # subnormal kept, not flushed
