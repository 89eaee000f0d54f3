"""Pins for the oracle's lower-precision transport (Section 6.2.3: gradients
need not be communicated in the parameter's type): 16-bit replica copies,
binary32 accumulation, binary32 averages."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads
from conftest import read_golden

FP32, FP16, BF16 = oracle.DT_FP32, oracle.DT_FP16, oracle.DT_BF16
U = 2.0 ** -24


def store(x, dtype):
    return oracle.from_f32(np.asarray(x, dtype=np.float32), dtype)


def test_hand_worked_example():
    g = read_golden("transport_example.txt")
    assert g["transport"] == "fp16" and int(g["R"]) == 2
    x0 = np.array([float(v) for v in g["replica0"].split()], dtype=np.float16)
    x1 = np.array([float(v) for v in g["replica1"].split()], dtype=np.float16)
    want32 = np.array([float(v) for v in g["average_f32"].split()], dtype=np.float32)
    want16 = np.array([float(v) for v in g["average_all_fp16"].split()], dtype=np.float16)
    got = oracle.reduce_average_transport([x0, x1], FP16)
    assert got.dtype == np.float32 and got.tobytes() == want32.tobytes()
    assert oracle.reduce_average([x0, x1], FP16).tobytes() == want16.tobytes()
    cin = np.array([float(v) for v in g["compress_in"].split()], dtype=np.float32)
    cout = np.array([float(v) for v in g["compress_out"].split()], dtype=np.float16)
    assert oracle.compress(cin, FP16).tobytes() == cout.tobytes()


@pytest.mark.parametrize("transport", [FP16, BF16])
@pytest.mark.parametrize("R", [1, 2, 3, 8, 16])
def test_rounding_the_result_gives_the_pinned_all_16_bit_result(transport, R):
    """reduce_average (pinned on its own) is the same sum and division followed
    by one rounding to the storage format; so rounding the transport result
    must reproduce it bit for bit, and with the output type equal to the
    transport type the two functions coincide."""
    rng = np.random.default_rng(100 * R + transport)
    flats = [store(rng.standard_normal(5000) * 1e-2, transport) for _ in range(R)]
    y32 = oracle.reduce_average_transport(flats, transport)
    assert y32.dtype == np.float32
    assert oracle.from_f32(y32, transport).tobytes() == oracle.reduce_average(flats, transport).tobytes()
    assert oracle.reduce_average_transport(flats, transport, transport).tobytes() == \
        oracle.reduce_average(flats, transport).tobytes()
    # and the binary32 result carries more than the 16-bit one whenever rounding bites
    assert (oracle.to_f32(oracle.from_f32(y32, transport), transport) != y32).any() or R == 1


@pytest.mark.parametrize("transport,bound", [(FP16, 2048), (BF16, 128)])
@pytest.mark.parametrize("R", [1, 2, 3, 5, 8, 32])
def test_integer_inputs_equal_exact_arithmetic(transport, bound, R):
    """Integers that the transport format holds exactly, sums below 2^24: every
    partial sum is exact in any order, the result is the integer sum divided
    by R rounded once to binary32."""
    rng = np.random.default_rng(7 * R + transport)
    ints = rng.integers(-bound, bound + 1, size=(R, 2049))
    flats = [store(ints[r], transport) for r in range(R)]
    assert all((oracle.to_f32(f, transport) == ints[r]).all() for r, f in enumerate(flats))
    got = oracle.reduce_average_transport(flats, transport)
    total = ints.sum(axis=0)
    for j in range(0, 2049, 31):
        q = Fraction(int(total[j]), R)
        # (float64 quotient of integers below 2^24 by R <= 32, then rounded to binary32: equal to
        # rounding the rational, see the note in test_oracle_reduce.py)
        assert got[j] == np.float32(q.numerator / q.denominator)
    if R & (R - 1) == 0:
        assert (got.astype(np.float64) == total / R).all()


@pytest.mark.parametrize("transport", [FP16, BF16])
@pytest.mark.parametrize("R", [2, 3, 8, 32])
def test_against_float64_definition_within_summation_bound(transport, R):
    rng = np.random.default_rng(R + 50 * transport)
    flats = [store(rng.standard_normal(20000) * 1e-3, transport) for _ in range(R)]
    exact = sum(oracle.to_f32(f, transport).astype(np.float64) for f in flats) / R
    scale = sum(np.abs(oracle.to_f32(f, transport).astype(np.float64)) for f in flats) / R
    got = oracle.reduce_average_transport(flats, transport).astype(np.float64)
    # R - 1 additions and one division in binary32 on exactly representable inputs
    assert (np.abs(got - exact) <= R * U * scale + 1e-45).all()


@pytest.mark.parametrize("transport,eps", [(FP16, 2.0 ** -11), (BF16, 2.0 ** -8)])
def test_compress_is_one_correct_rounding(transport, eps):
    rng = np.random.default_rng(3)
    x = (rng.standard_normal(100000) * 1e-2).astype(np.float32)
    x = x[np.abs(x) > 1e-4]                       # normal range of both formats
    c = oracle.to_f32(oracle.compress(x, transport), transport)
    assert (np.abs(c.astype(np.float64) - x.astype(np.float64)) <= eps * np.abs(x.astype(np.float64))).all()
    if transport == FP16:
        assert oracle.compress(x, FP16).tobytes() == x.astype(np.float16).tobytes()
    with pytest.raises(ValueError):
        oracle.compress(x, FP32)


def test_synchronize_transport_on_the_tiny_list():
    """Buckets are those of a 16-bit model (a bucket is what is communicated);
    the values are the float64 mean of what was sent, within the bound; with
    never-marked parameters the outputs are zeros of the output type."""
    numel = workloads.numel_of(workloads.tiny_shapes())
    n, R, cap = len(numel), 4, 16384
    sent = [[oracle.compress(workloads.gaussian_grad(70, r, 0, p, numel[p], 1.0), BF16) for p in range(n)]
            for r in range(R)]
    outs, asg, log = oracle.synchronize_transport(numel, [BF16] * n, cap, sent)
    ref = oracle.assign_buckets(numel, [BF16] * n, cap)
    assert asg.bucket_of.tolist() == ref.bucket_of.tolist() and asg.offset_of.tolist() == ref.offset_of.tolist()
    assert log == oracle.launch_schedule(ref, list(range(n - 1, -1, -1)))
    for p in range(n):
        assert outs[p].dtype == np.float32 and outs[p].size == numel[p]
        exact = sum(oracle.to_f32(sent[r][p], BF16).astype(np.float64) for r in range(R)) / R
        scale = sum(np.abs(oracle.to_f32(sent[r][p], BF16).astype(np.float64)) for r in range(R)) / R
        assert (np.abs(outs[p].astype(np.float64) - exact) <= R * U * scale).all()
        # rounding to the transport type gives the all-16-bit synchronization (pinned elsewhere)
    all16, _, _ = oracle.synchronize(numel, [BF16] * n, cap, sent)
    for p in range(n):
        assert oracle.from_f32(outs[p], BF16).tobytes() == all16[p].tobytes()
    order = [7, 6, 4, 3, 1]                        # 5, 2, 0 never marked
    outs2, _, _ = oracle.synchronize_transport(numel, [BF16] * n, cap, sent, order)
    for p in (5, 2, 0):
        assert outs2[p].dtype == np.float32 and not outs2[p].any()
    for p in order:
        assert outs2[p].tobytes() == outs[p].tobytes()
