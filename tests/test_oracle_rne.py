"""Pins for the narrowing oracle (oracle/rne.c): hand-derived vectors, an
independent integer formulation, torch's CPU cast, and ordering properties."""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

from oracle import rne

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "rne_vectors.txt")


def integer_rne(u):
    """Second, independent formulation: add half an ulp (minus one when the
    kept LSB is even) and truncate; NaNs get the quiet bit."""
    u = u.astype(np.uint64)
    is_nan = (u & 0x7FFFFFFF) > 0x7F800000
    r = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    r = np.where(is_nan, (u >> 16) | 0x40, r)
    return (r & 0xFFFF).astype(np.uint16)


def torch_cast(u):
    t = torch.from_numpy(u.view(np.int32)).view(torch.float32).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def test_hand_vectors():
    ins, outs = [], []
    for line in open(GOLDEN):
        line = line.split("#")[0].split()
        if line:
            ins.append(int(line[0], 16))
            outs.append(int(line[1], 16))
    assert len(ins) >= 20
    got = rne.narrow(np.array(ins, dtype=np.uint32))
    assert [hex(x) for x in got] == [hex(x) for x in outs]


def _edge_patterns():
    hi = np.arange(1 << 16, dtype=np.uint32) << 16
    lows = np.array([0x0000, 0x0001, 0x0002, 0x3FFF, 0x4000, 0x7FFE, 0x7FFF, 0x8000, 0x8001,
                     0x8002, 0xBFFF, 0xC000, 0xFFFE, 0xFFFF, 0x1234, 0xEDCB], dtype=np.uint32)
    return (hi[:, None] | lows[None, :]).reshape(-1)


def test_exhaustive_edge_patterns_vs_integer_formula_and_torch():
    u = _edge_patterns()  # every bf16 prefix x every interesting low half
    got = rne.narrow(u)
    assert np.array_equal(got, integer_rne(u))
    not_nan = (u & 0x7FFFFFFF) <= 0x7F800000
    assert np.array_equal(got[not_nan], torch_cast(u[not_nan]))


def test_all_2_pow_32_patterns():
    """Every fp32 bit pattern: definitional oracle == integer formulation, and
    == torch's CPU cast wherever the input is not a NaN."""
    step = 1 << 20  # small blocks stay in cache and avoid page-fault churn

    def block(b):
        u = np.arange(b * step, (b + 1) * step, dtype=np.uint64).astype(np.uint32)
        got = rne.narrow(u)
        ok = np.array_equal(got, integer_rne(u))
        not_nan = (u & 0x7FFFFFFF) <= 0x7F800000
        ok = ok and np.array_equal(got[not_nan], torch_cast(u[not_nan]))
        return ok

    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        res = list(ex.map(block, range((1 << 32) // step)))
    assert all(res), [i for i, r in enumerate(res) if not r]


def test_nearest_and_monotone():
    rng = np.random.default_rng(0)
    u = rng.integers(0, 0x7F800000, size=200000, dtype=np.uint32)  # positive finite
    u.sort()
    got = rne.narrow(u)
    # monotone: ordering of positive floats is the ordering of their bit patterns
    assert np.all(np.diff(got.astype(np.int64)) >= 0)
    # nearest: the error is at most half the gap between the bracketing bf16 values
    x = u.view(np.float32).astype(np.float64)
    lo = ((u >> 16) << 16).view(np.float32).astype(np.float64)
    hi_bits = ((u >> 16) + 1) << 16
    finite_hi = hi_bits < 0x7F800000
    hi = np.where(finite_hi, hi_bits.astype(np.uint32).view(np.float32).astype(np.float64), 2.0 ** 128)
    y_bits = got.astype(np.uint32) << 16
    y = np.where(y_bits < 0x7F800000, y_bits.view(np.float32).astype(np.float64), 2.0 ** 128)
    assert np.all(np.abs(y - x) <= (hi - lo) / 2)
    # sign symmetry
    neg = rne.narrow(u | np.uint32(0x80000000))
    assert np.array_equal(neg, got | np.uint16(0x8000))


def test_nan_never_becomes_inf_and_keeps_sign():
    rng = np.random.default_rng(1)
    payload = rng.integers(1, 1 << 23, size=100000, dtype=np.uint32)
    sign = rng.integers(0, 2, size=100000, dtype=np.uint32) << 31
    u = sign | np.uint32(0x7F800000) | payload
    got = rne.narrow(u)
    assert np.all((got & 0x7FFF) > 0x7F80)
    assert np.array_equal(got >> 15, (u >> 31).astype(np.uint16))
    assert np.all(got & 0x0040)


def test_identity_conversions_copy_bits():
    a = np.arange(100, dtype=np.uint16)
    b = rne.convert(a, "bf16", "bf16")
    assert np.array_equal(a, b) and b is not a
