"""Pins for the oracle's storage conversions and its reduce-and-average step
(AllReduce = sum over participants, Section 2.3; DDP averages, Section 3.2.1)."""
import struct
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle

FP32, FP16, BF16 = oracle.DT_FP32, oracle.DT_FP16, oracle.DT_BF16
U = 2.0 ** -24          # unit roundoff of binary32


# ---- storage conversions against independent library routines -------------
def test_fp16_widening_all_patterns_against_struct():
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.to_f32(bits.view(np.float16), FP16)
    want = np.array(struct.unpack("<65536e", bits.tobytes()), dtype=np.float64)
    same = (got.astype(np.float64) == want) | (np.isnan(got) & np.isnan(want))
    assert same.all()


def test_fp16_round_trip_all_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    back = oracle.from_f32(oracle.to_f32(bits.view(np.float16), FP16), FP16).view(np.uint16)
    finite = ~np.isnan(bits.view(np.float16))
    assert (back[finite] == bits[finite]).all()       # subnormals included
    assert np.isnan(back[~finite].view(np.float16)).all()


def test_bf16_widening_and_round_trip_all_patterns_against_torch():
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.to_f32(bits, BF16)
    want = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).float().numpy()
    assert (got.view(np.uint32) == want.view(np.uint32)).all()
    back = oracle.from_f32(got, BF16)
    finite = ~np.isnan(got)
    assert (back[finite] == bits[finite]).all()
    assert np.isnan(oracle.to_f32(back[~finite], BF16)).all()


def test_bf16_rounding_against_torch_on_ties_and_random_bits():
    rng = np.random.default_rng(7)
    hi = np.arange(65536, dtype=np.uint32) << 16
    lows = [0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF]
    pats = np.concatenate([hi | np.uint32(lo) for lo in lows]
                          + [rng.integers(0, 2**32, size=1_000_000, dtype=np.uint64).astype(np.uint32)])
    x = pats.view(np.float32)
    got = oracle.from_f32(x, BF16)
    want = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    finite = ~np.isnan(x)
    assert (got[finite] == want[finite]).all()
    assert np.isnan(oracle.to_f32(got[~finite], BF16)).all()


def test_fp16_rounding_against_torch_on_random_bits():
    rng = np.random.default_rng(8)
    x = rng.integers(0, 2**32, size=1_000_000, dtype=np.uint64).astype(np.uint32).view(np.float32)
    x = np.concatenate([x, (rng.standard_normal(200_000) * 1e-6).astype(np.float32)])  # subnormal range
    got = oracle.from_f32(x, FP16).view(np.uint16)
    want = torch.from_numpy(x.copy()).to(torch.float16).view(torch.int16).numpy().view(np.uint16)
    finite = ~np.isnan(x)
    assert (got[finite] == want[finite]).all()


# ---- reduce: exact closed forms -------------------------------------------
@pytest.mark.parametrize("R", [1, 2, 3, 5, 8, 16, 32])
@pytest.mark.parametrize("dtype,bound", [(FP32, 200_000), (FP16, 60), (BF16, 60)])
def test_integer_inputs_equal_exact_arithmetic(R, dtype, bound):
    """Integer-valued inputs whose sum stays below 2^24: every binary32
    partial sum is exact whatever the order, so the result must be the
    integer sum divided by R, rounded once."""
    rng = np.random.default_rng(R * 10 + dtype)
    ints = rng.integers(-bound, bound + 1, size=(R, 4097))
    if dtype == FP32:
        flats = [ints[r].astype(np.float32) for r in range(R)]
    elif dtype == FP16:
        flats = [ints[r].astype(np.float16) for r in range(R)]
    else:
        flats = [(ints[r].astype(np.float32).view(np.uint32) >> 16).astype(np.uint16) for r in range(R)]
        assert (oracle.to_f32(flats[0], BF16) == ints[0]).all()   # |v| <= 60 fits 8 bits
    got = oracle.to_f32(oracle.reduce_average(flats, dtype), dtype)
    total = ints.sum(axis=0)
    for j in range(0, 4097, 97):      # exact rationals on a sample
        q = Fraction(int(total[j]), R)
        if dtype == FP32:
            want = np.float32(q.numerator / q.denominator)    # see note below
        elif dtype == FP16:
            want = np.float32(np.float16(q.numerator / q.denominator))
        else:
            want = oracle.to_f32(oracle.from_f32(np.array([q.numerator / q.denominator], dtype=np.float64).astype(np.float32), BF16), BF16)[0]
        assert got[j] == want
    # note: float64 division of integers below 2^24 by R <= 32 is within 2^-53
    # relative of the rational; a binary32 (or narrower) rounding boundary is a
    # dyadic rational at distance >= 1/(R 2^k) from it, far more than that, so
    # rounding the float64 quotient equals rounding the rational.
    if R & (R - 1) == 0 and dtype == FP32:
        assert (got.astype(np.float64) == total / R).all()    # exact for power-of-two R


@pytest.mark.parametrize("dtype", [FP32, FP16, BF16])
def test_single_replica_is_identity(dtype):
    rng = np.random.default_rng(3)
    x = (rng.standard_normal(10_000) * 1e-2).astype(np.float32)
    if dtype == FP16:
        x = x.astype(np.float16)
    elif dtype == BF16:
        x = (x.view(np.uint32) >> 16).astype(np.uint16)
    got = oracle.reduce_average([x], dtype)
    assert got.tobytes() == x.tobytes()


def test_equal_replicas_average_to_themselves():
    rng = np.random.default_rng(4)
    x = rng.standard_normal(5000).astype(np.float32)
    # x + x is exact, and halving is exact: only R = 2 has this property
    # (x + x + x already rounds)
    assert (oracle.reduce_average([x, x], FP32) == x).all()


@pytest.mark.parametrize("R", [2, 3, 8, 32])
def test_against_float64_definition_within_summation_bound(R):
    """|fixed-order binary32 result - exact mean| <= gamma_R * mean|x|,
    gamma_R = R u / (1 - R u): (R-1) additions and one division."""
    rng = np.random.default_rng(R)
    flats = [(rng.standard_normal(50_000) * 1e-2).astype(np.float32) for _ in range(R)]
    got = oracle.reduce_average(flats, FP32).astype(np.float64)
    exact = np.sum([f.astype(np.float64) for f in flats], axis=0) / R
    scale = np.sum([np.abs(f.astype(np.float64)) for f in flats], axis=0) / R
    gamma = R * U / (1 - R * U)
    assert (np.abs(got - exact) <= gamma * scale + 1e-300).all()
    # and the error is real (not float64 in disguise) for R > 2
    if R > 2:
        assert np.abs(got - exact).max() > 0


def test_sum_order_is_r_ascending():
    """(2^24 + 1) + (-2^24): ascending order gives 2^24 + 1 -> rounds to 2^24
    first, then 0; the reverse order would give 1."""
    a = np.array([2.0 ** 24], dtype=np.float32)
    b = np.array([1.0], dtype=np.float32)
    c = np.array([-(2.0 ** 24)], dtype=np.float32)
    assert oracle.reduce_average([a, b, c, np.zeros(1, np.float32)], FP32)[0] == 0.0
    assert oracle.reduce_average([c, a, b, np.zeros(1, np.float32)], FP32)[0] == 0.25


def test_division_not_reciprocal_multiplication():
    """R = 3: the average is s / 3 correctly rounded.  Multiplying by
    float32(1/3) differs from that on many inputs; the oracle must match the
    division."""
    rng = np.random.default_rng(11)
    flats = [rng.integers(-1000, 1000, size=20_000).astype(np.float32) for _ in range(3)]
    s = flats[0].astype(np.float64) + flats[1] + flats[2]
    want = (s / 3.0).astype(np.float32)          # exact sum, one rounding (see note above)
    got = oracle.reduce_average(flats, FP32)
    assert (got == want).all()
    recip = (s.astype(np.float32) * np.float32(1.0 / 3.0)).astype(np.float32)
    assert (recip != want).any()


def test_fp16_two_replicas_all_patterns_against_exact():
    """Every fp16 pattern averaged with a fixed partner.  a + c is exact in
    float64; where the binary32 sum is exact as well the result must be the
    once-rounded exact mean, elsewhere it may differ by the double rounding,
    at most one fp16 step."""
    bits = np.arange(65536, dtype=np.uint16)
    a = bits.view(np.float16)
    finite = np.isfinite(a)
    for partner in (np.float16(0.3711), np.float16(-1.5e-5), np.float16(1024.0)):
        c = np.full(65536, partner, dtype=np.float16)
        got = oracle.reduce_average([a, c], FP16)
        with np.errstate(over="ignore", invalid="ignore"):
            exact = (a.astype(np.float64) + c.astype(np.float64)) / 2.0
            want = exact.astype(np.float16)
            s32 = a.astype(np.float32) + c.astype(np.float32)
        sum_exact = finite & (s32.astype(np.float64) == exact * 2.0)
        assert (got[sum_exact] == want[sum_exact]).all()
        rest = finite & ~sum_exact
        step = np.abs(got[rest].view(np.int16).astype(np.int32) - want[rest].view(np.int16).astype(np.int32))
        assert (step <= 1).all()


def test_fp16_subnormal_inputs_are_not_flushed():
    tiny = np.array([2.0 ** -24, 3 * 2.0 ** -24, -(2.0 ** -23)], dtype=np.float16)
    zero = np.zeros(3, dtype=np.float16)
    got = oracle.reduce_average([tiny, tiny], FP16)
    assert (got == tiny).all()
    got = oracle.reduce_average([tiny, zero], FP16).astype(np.float64)
    # halves of subnormals: 2^-25 ties to even (0), 1.5 * 2^-24 ties to even (2^-23), -2^-24 exact
    assert got.tolist() == [0.0, 2.0 ** -23, -(2.0 ** -24)]


def test_nonfinite_values_propagate():
    x = np.array([np.inf, np.nan, 1.0, -np.inf], dtype=np.float32)
    y = np.array([1.0, 1.0, np.inf, np.inf], dtype=np.float32)
    got = oracle.reduce_average([x, y], FP32)
    assert np.isposinf(got[0]) and np.isnan(got[1]) and np.isposinf(got[2]) and np.isnan(got[3])
