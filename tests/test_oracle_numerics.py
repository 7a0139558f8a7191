"""Pins for the oracle's conversions and its single hop (CPU only).

The wire-type conversions are checked against numpy's float16 and torch's
bfloat16 (library routines), the hop against exact rational arithmetic
(tests/brute.py) and against correctly rounded sums computed in float64.
"""
import numpy as np
import pytest
import torch

import brute
from oracle import ring_oracle as orc


def _rand_f32_patterns(n, seed):
    rng = np.random.Generator(np.random.Philox(seed))
    return rng.integers(0, 1 << 32, size=n, dtype=np.uint64).astype(np.uint32)


def _torch_bf16_bits(x_f32):
    return torch.from_numpy(x_f32.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def _is_nan16(b, fmt):
    return (b & 0x7FFF) > (0x7F80 if fmt == "bf16" else 0x7C00)


# ---------------------------------------------------------------- conversions
def test_bf16_widen_all_patterns():
    allp = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    got = orc.bf16_to_f32(allp).view(np.uint32)
    want = torch.from_numpy(allp.view(np.int16).copy()).view(torch.bfloat16).float().numpy().view(np.uint32)
    assert np.array_equal(got, want)


def test_f16_widen_all_patterns():
    allp = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    got = orc.f16_to_f32(allp)
    want = allp.view(np.float16).astype(np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got.view(np.uint32)[~nan], want.view(np.uint32)[~nan])


def _edge_f32():
    e = [0x00000000, 0x80000000, 0x00000001, 0x007FFFFF, 0x00800000, 0x7F7FFFFF, 0x7F800000, 0xFF800000,
         0x7FC00000, 0x7F800001, 0xFFFFFFFF, 0x3F800000, 0x3F808000, 0x3F818000, 0x3F807FFF, 0x3F808001,
         0x7F7F8000, 0x7F7F7FFF, 0x477FE000, 0x477FF000, 0x477FEFFF, 0x33800000, 0x33000000, 0x33000001,
         0x387FC000, 0x387FE000, 0x38800000, 0x387FFFFF, 0x32FFFFFF]
    return np.array(e, dtype=np.uint32)


def test_f32_to_bf16_matches_torch():
    pats = np.concatenate([_rand_f32_patterns(3_000_000, 11), _edge_f32(),
                           # every tie and near-tie in a few binades
                           (np.arange(0x3F800000, 0x3F800000 + (1 << 18), dtype=np.uint32))])
    x = pats.view(np.float32)
    got, want = orc.f32_to_bf16(x), _torch_bf16_bits(x)
    nan = np.isnan(x)
    assert np.all(_is_nan16(got[nan], "bf16")) and np.all(_is_nan16(want[nan], "bf16"))
    assert np.array_equal(got[~nan], want[~nan])


def test_f32_to_f16_matches_numpy():
    # random patterns, plus dense coverage of the binary16 normal, subnormal and overflow ranges
    dense = []
    for e in (0x33000000, 0x33800000, 0x38000000, 0x38800000, 0x3F800000, 0x47000000, 0x47800000):
        dense.append(np.arange(e - (1 << 16), e + (1 << 16), dtype=np.uint32))
    pats = np.concatenate([_rand_f32_patterns(3_000_000, 12), _edge_f32(), *dense])
    x = pats.view(np.float32)
    got = orc.f32_to_f16(x)
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    nan = np.isnan(x)
    assert np.all(_is_nan16(got[nan], "fp16"))
    assert np.array_equal(got[~nan], want[~nan])


def test_bf16_epsilon_is_two_to_minus_seven():
    # Section 5.3 "Model Accuracy" quotes 7.8125e-3 as BF16 machine epsilon: the
    # gap between 1 and the next bf16 value, i.e. a 1 + 7 bit significand.
    one = orc.f32_to_bf16(np.array([1.0], np.float32))[0]
    nxt = orc.bf16_to_f32(np.array([one + 1], np.uint16))[0]
    assert nxt - 1.0 == 7.8125e-3 == 2.0 ** -7
    # half of it is a tie and rounds back to 1 (even), just above half rounds up
    assert orc.f32_to_bf16(np.array([1.0 + 2.0 ** -8], np.float32))[0] == one
    assert orc.f32_to_bf16(np.array([1.0 + 2.0 ** -8 + 2.0 ** -20], np.float32))[0] == one + 1


# ------------------------------------------------------------------------ hop
def test_hop_fp16_is_correctly_rounded_sum():
    rng = np.random.Generator(np.random.Philox(21))
    a = rng.integers(0, 1 << 16, size=4_000_000, dtype=np.uint32).astype(np.uint16)
    b = rng.integers(0, 1 << 16, size=4_000_000, dtype=np.uint32).astype(np.uint16)
    got = orc.hop(a, b, orc.FP16)
    # binary16 sums are exact in float64, and numpy rounds float64 -> float16 once
    with np.errstate(over="ignore", invalid="ignore"):
        want = (a.view(np.float16).astype(np.float64) + b.view(np.float16).astype(np.float64)).astype(np.float16)
    want = want.view(np.uint16)
    nan = _is_nan16(want, "fp16")
    assert np.array_equal(_is_nan16(got, "fp16"), nan)
    assert np.array_equal(got[~nan], want[~nan])


def test_hop_bf16_matches_library_add():
    rng = np.random.Generator(np.random.Philox(22))
    a = rng.integers(0, 1 << 16, size=4_000_000, dtype=np.uint32).astype(np.uint16)
    b = rng.integers(0, 1 << 16, size=4_000_000, dtype=np.uint32).astype(np.uint16)
    got = orc.hop(a, b, orc.BF16)
    ta = torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16)
    tb = torch.from_numpy(b.view(np.int16).copy()).view(torch.bfloat16)
    want = (ta + tb).view(torch.int16).numpy().view(np.uint16)
    nan = _is_nan16(want, "bf16")
    assert np.array_equal(_is_nan16(got, "bf16"), nan)
    assert np.array_equal(got[~nan], want[~nan])


def test_hop_fp32_matches_numpy_add():
    a = _rand_f32_patterns(2_000_000, 23).view(np.float32)
    b = _rand_f32_patterns(2_000_000, 24).view(np.float32)
    got = orc.hop(a, b, orc.FP32)
    with np.errstate(over="ignore", invalid="ignore"):
        want = a + b
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got.view(np.uint32)[~nan], want.view(np.uint32)[~nan])


def _interesting_pairs(fmt, n, seed):
    """Bit-pattern pairs with close exponents (so sums round, cancel, go subnormal or overflow)."""
    eb, fb = brute.FMT[fmt]
    rng = np.random.Generator(np.random.Philox(seed))
    emax = (1 << eb) - 1
    out = []
    for _ in range(n):
        mode = rng.integers(0, 4)
        if mode == 0:       # anywhere
            e1, e2 = rng.integers(0, emax + 1), rng.integers(0, emax + 1)
        elif mode == 1:     # near each other
            e1 = rng.integers(0, emax); e2 = min(emax - 1, max(0, e1 + rng.integers(-fb - 3, fb + 4)))
        elif mode == 2:     # subnormal neighbourhood
            e1, e2 = rng.integers(0, 4), rng.integers(0, 4)
        else:               # overflow neighbourhood
            e1, e2 = emax - 1 - rng.integers(0, 2), emax - 1 - rng.integers(0, 3)
        m1, m2 = rng.integers(0, 1 << fb), rng.integers(0, 1 << fb)
        if rng.integers(0, 3) == 0:
            m2 = m1 if rng.integers(0, 2) else (m1 ^ 1)
        s1, s2 = rng.integers(0, 2), rng.integers(0, 2)
        out.append(((int(s1) << (eb + fb)) | (int(e1) << fb) | int(m1),
                    (int(s2) << (eb + fb)) | (int(e2) << fb) | int(m2)))
    return out


@pytest.mark.parametrize("fmt,code", [("bf16", orc.BF16), ("fp16", orc.FP16), ("fp32", orc.FP32)])
def test_hop_matches_exact_rational_arithmetic(fmt, code):
    pairs = _interesting_pairs(fmt, 6000, 31)
    # signed zeros, infinities, NaN
    eb, fb = brute.FMT[fmt]
    sgn = 1 << (eb + fb)
    inf = ((1 << eb) - 1) << fb
    specials = [0, sgn, inf, sgn | inf, inf | 1, 1, sgn | 1, (1 << fb), inf - 1, sgn | (inf - 1)]
    pairs += [(x, y) for x in specials for y in specials]
    if fmt == "fp32":
        a = np.array([p[0] for p in pairs], dtype=np.uint32).view(np.float32)
        b = np.array([p[1] for p in pairs], dtype=np.uint32).view(np.float32)
        got = orc.hop(a, b, code).view(np.uint32)
        nanmask = inf
        is_nan = lambda v: (v & 0x7FFFFFFF) > nanmask
    else:
        a = np.array([p[0] for p in pairs], dtype=np.uint16)
        b = np.array([p[1] for p in pairs], dtype=np.uint16)
        got = orc.hop(a, b, code)
        is_nan = lambda v: (v & (sgn - 1)) > inf
    for (x, y), g in zip(pairs, got):
        w = brute.hop(x, y, fmt)
        if is_nan(w):
            assert is_nan(int(g)), (hex(x), hex(y))
        else:
            assert int(g) == w, (fmt, hex(x), hex(y), hex(int(g)), hex(w))


def test_hop_int32_wraps():
    a = np.array([2**31 - 1, -2**31, 5, -7, 2**31 - 1], dtype=np.int32)
    b = np.array([1, -1, -9, 7, 2**31 - 1], dtype=np.int32)
    got = orc.hop(a, b, orc.INT32)
    want = ((a.astype(np.int64) + b.astype(np.int64)) & 0xFFFFFFFF).astype(np.uint32).view(np.int32)
    assert np.array_equal(got, want)
    assert [brute.hop_int32(int(x), int(y)) for x, y in zip(a, b)] == want.tolist()
