"""Pins for the CPU oracle: it is checked against what the mathematics fixes,
never against itself and never against the HIP library.

  * closed forms and special cases (identity, constants, cancellation, -0);
  * an order discriminator only left-to-right summation passes;
  * exact rational brute force on tiny inputs (fractions.Fraction);
  * an integer-arithmetic model of IEEE-754 roundTiesToEven (tests/ieee_model.py);
  * library routines on special cases (float64 adds, torch's bf16 cast);
  * hand-derived fixtures under tests/golden/.
The "mutant" tests at the end show that plausible mistakes (tree order, bf16
accumulation, truncation, fused or distributed scaling) fail these pins.
"""
import os
import random
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from tests import ieee_model as M

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def f32(bits):
    return np.array(bits, dtype=np.uint32).view(np.float32)


def bits32(x):
    return np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)


ODT = {"f32": oracle.F32, "bf16": oracle.BF16, "f16": oracle.F16, "e4m3": oracle.FP8_E4M3, "e5m2": oracle.FP8_E5M2}
FP8_FMT = {"e4m3": M.E4M3, "e5m2": M.E5M2}


def col(bits, dtype):
    """One-element buffer per input from a list of bit patterns."""
    if dtype == oracle.F32:
        return [np.array([b], dtype=np.uint32).view(np.float32) for b in bits]
    if dtype in (oracle.FP8_E4M3, oracle.FP8_E5M2):
        return [np.array([b], dtype=np.uint8) for b in bits]
    return [np.array([b], dtype=np.uint16) for b in bits]


def out_bits(arr):
    return int(arr.view(np.uint32)[0]) if arr.dtype == np.float32 else int(arr[0])


# ----------------------------------------------------------------- fixtures

def _load_cases(name, nfields):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = [p.strip() for p in line.split(";", nfields - 1)]
            assert len(parts) == nfields, line
            rows.append(parts)
    return rows


def _model_sum(dtype, in_bits):
    """Exact model of the in-order fp32 sum with one final narrowing."""
    if dtype == "f32":
        acc = in_bits[0]
        for b in in_bits[1:]:
            acc = M.add_rne(acc, b)
        return acc
    if dtype in FP8_FMT:
        acc = M.widen_fp8_to_f32(in_bits[0], FP8_FMT[dtype])
        for b in in_bits[1:]:
            acc = M.add_rne(acc, M.widen_fp8_to_f32(b, FP8_FMT[dtype]))
        return M.narrow_f32_to_fp8(acc, FP8_FMT[dtype])
    if dtype == "f16":
        acc = M.widen_f16_to_f32(in_bits[0])
        for b in in_bits[1:]:
            acc = M.add_rne(acc, M.widen_f16_to_f32(b))
        return M.narrow_f32_to_f16(acc)
    acc = in_bits[0] << 16
    for b in in_bits[1:]:
        acc = M.add_rne(acc, b << 16)
    return M.narrow_f32_to_bf16(acc)


@pytest.mark.parametrize("row", _load_cases("reduce_sum_cases.txt", 4), ids=lambda r: r[3][:40])
def test_golden_reduce_sum(row):
    dt, ins, exp, _why = row
    in_bits = [int(x, 16) for x in ins.split()]
    exp = int(exp, 16)
    dtype = ODT[dt]
    # the fixture itself must agree with exact rational arithmetic
    fmt = {"f32": M.BINARY32, "bf16": M.BFLOAT16, "f16": M.BINARY16, "e4m3": M.E4M3, "e5m2": M.E5M2}[dt]
    kinds = [M.decode(b, fmt)[0] for b in in_bits]
    if all(k == "num" for k in kinds) and (dt in FP8_FMT or exp not in (0x7F800000, 0x7F80, 0x7C00)):
        assert _model_sum(dt, in_bits) == exp
    got = out_bits(oracle.reduce_sum(col(in_bits, dtype), dtype))
    assert got == exp, "%s: got %x want %x" % (row[3], got, exp)


@pytest.mark.parametrize("row", _load_cases("combine_avg_cases.txt", 6), ids=lambda r: r[5][:40])
def test_golden_combine_avg(row):
    dt, a, b, s, exp, _why = row
    a, b, s, exp = (int(v, 16) for v in (a, b, s, exp))
    dtype = ODT[dt]
    scale = f32([s])[0]
    if dt in FP8_FMT:
        A, B = M.widen_fp8_to_f32(a, FP8_FMT[dt]), M.widen_fp8_to_f32(b, FP8_FMT[dt])
    elif dt == "f32":
        A, B = a, b
    elif dt == "f16":
        A, B = M.widen_f16_to_f32(a), M.widen_f16_to_f32(b)
    else:
        A, B = a << 16, b << 16
    t = M.add_rne(A, B)
    if M.decode(t, M.BINARY32)[0] == "num":
        u = M.mul_rne(t, s)
        if dt in FP8_FMT:
            want = M.narrow_f32_to_fp8(u, FP8_FMT[dt])
        else:
            want = u if dt == "f32" else (M.narrow_f32_to_f16(u) if dt == "f16" else M.narrow_f32_to_bf16(u))
        assert want == exp
    got = out_bits(oracle.combine_avg(col([a], dtype)[0], col([b], dtype)[0], scale, dtype))
    assert got == exp, "%s: got %x want %x" % (row[5], got, exp)


# ------------------------------------------------------------- closed forms

def _random_f32_patterns(rng, n, allow_special=True):
    """Bit patterns spread over all exponents (incl. subnormals, zeros, inf)."""
    u = rng.integers(0, 1 << 32, size=n, dtype=np.uint64).astype(np.uint32)
    if not allow_special:
        e = (u >> 23) & 0xFF
        u = np.where(e == 0xFF, u & np.uint32(0x7F7FFFFF), u)
    else:
        # keep inf, drop NaN (payloads are not compared)
        nan = (((u >> 23) & 0xFF) == 0xFF) & ((u & 0x7FFFFF) != 0)
        u = np.where(nan, u & np.uint32(0xFF800000), u)
    return u.astype(np.uint32)


def test_k1_identity_f32():
    rng = np.random.default_rng(11)
    u = _random_f32_patterns(rng, 100003)
    out = oracle.reduce_sum([u.view(np.float32)], oracle.F32)
    assert np.array_equal(out.view(np.uint32), u)


def test_k1_identity_bf16_all_patterns():
    h = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    out = oracle.reduce_sum([h], oracle.BF16)
    is_nan = ((h & 0x7F80) == 0x7F80) & ((h & 0x007F) != 0)
    assert np.array_equal(out[~is_nan], h[~is_nan])
    o_nan = ((out & 0x7F80) == 0x7F80) & ((out & 0x007F) != 0)
    assert np.array_equal(o_nan, is_nan)  # NaN stays NaN, never becomes inf


@pytest.mark.parametrize("c", [1.0, -3.0, 0.5, 2.0 ** -20, 255.0])
@pytest.mark.parametrize("K", [1, 2, 3, 8, 16])
def test_constant_inputs_f32(c, K):
    n = 37
    ins = [np.full(n, c, dtype=np.float32) for _ in range(K)]
    out = oracle.reduce_sum(ins, oracle.F32)
    assert np.array_equal(bits32(out), bits32(np.full(n, K * c, dtype=np.float32)))


@pytest.mark.parametrize("K", [1, 2, 4, 8, 16])
def test_constant_inputs_bf16(K):
    # c = 0.5: K*c <= 8 is exact in bf16 as is every partial sum
    n = 19
    half = np.full(n, 0x3F00, dtype=np.uint16)
    out = oracle.reduce_sum([half.copy() for _ in range(K)], oracle.BF16)
    want = torch.full((n,), 0.5 * K, dtype=torch.float32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(out, want)


@pytest.mark.parametrize("K", [2, 4, 8, 16])
def test_alternating_sign_cancels_to_plus_zero(K):
    rng = np.random.default_rng(5)
    u = _random_f32_patterns(rng, 4099, allow_special=False)
    x = u.view(np.float32)
    ins = [x if j % 2 == 0 else -x for j in range(K)]
    out = oracle.reduce_sum(ins, oracle.F32)
    assert np.all(out.view(np.uint32) == 0)  # +0, never -0
    xb = (u >> 16).astype(np.uint16)
    insb = [xb if j % 2 == 0 else (xb ^ np.uint16(0x8000)) for j in range(K)]
    outb = oracle.reduce_sum(insb, oracle.BF16)
    assert np.all(outb == 0)


def test_order_discriminator():
    vals = [2.0 ** 24, 1, 1, 1, 1, 1, 1, -(2.0 ** 24)]
    fwd = [np.array([v, w], dtype=np.float32) for v, w in zip(vals, reversed(vals))]
    out = oracle.reduce_sum(fwd, oracle.F32)
    assert out[0] == 0.0 and out[1] == 6.0
    # other plausible orders give other answers on column 0
    tree = np.float32(0)
    lvl = [np.float32(v) for v in vals]
    while len(lvl) > 1:
        lvl = [np.float32(lvl[i] + lvl[i + 1]) for i in range(0, len(lvl), 2)]
    assert lvl[0] != out[0]


# ------------------------------------------------- exact rational brute force

@pytest.mark.parametrize("seed", range(6))
def test_exact_grid_inputs_match_rational_sum(seed):
    """Integers * 2^-10 in [-4, 4]: every partial sum is exactly representable,
    so the result must be the exact rational sum whatever the rounding."""
    rng = np.random.default_rng(100 + seed)
    K = int(rng.integers(1, 17))
    n = int(rng.integers(1, 4097))
    ints = rng.integers(-4096, 4097, size=(K, n))
    ins = [(ints[j] / 1024.0).astype(np.float32) for j in range(K)]
    out = oracle.reduce_sum(ins, oracle.F32)
    exact = ints.sum(axis=0)
    for i in range(n):
        assert Fraction(float(out[i])) == Fraction(int(exact[i]), 1024)


@pytest.mark.parametrize("seed", range(4))
def test_exact_grid_inputs_bf16(seed):
    """Integers in [-8, 8] are exact in bf16 and so is every sum up to 128."""
    rng = np.random.default_rng(200 + seed)
    K = int(rng.integers(1, 17))
    n = int(rng.integers(1, 2049))
    ints = rng.integers(-8, 9, size=(K, n))
    ins = [torch.from_numpy(ints[j].astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy()
           for j in range(K)]
    out = oracle.reduce_sum(ins, oracle.BF16)
    exact = ints.sum(axis=0)
    back = oracle.widen_bf16(out)
    assert np.array_equal(back.astype(np.int64), exact)


@pytest.mark.parametrize("seed", range(4))
def test_general_inputs_match_integer_rounding_model(seed):
    """Each partial sum rounded to binary32 by exact integer arithmetic."""
    rng = np.random.default_rng(300 + seed)
    K = int(rng.integers(2, 17))
    n = 160
    u = _random_f32_patterns(rng, K * n, allow_special=False).reshape(K, n)
    # squeeze exponents into a band so that adds really round (not just absorb)
    e = (u >> 23) & 0xFF
    e = 100 + (e % 40)
    if seed == 3:
        e = e % 3  # subnormal / tiny band
    u = (u & np.uint32(0x807FFFFF)) | (e.astype(np.uint32) << 23)
    ins = [np.ascontiguousarray(u[j]).view(np.float32) for j in range(K)]
    out = oracle.reduce_sum(ins, oracle.F32).view(np.uint32)
    for i in range(n):
        acc = int(u[0, i])
        for j in range(1, K):
            acc = M.add_rne(acc, int(u[j, i]))
        assert int(out[i]) == acc, (i, hex(int(out[i])), hex(acc))


@pytest.mark.parametrize("seed", range(3))
def test_general_inputs_bf16_match_integer_rounding_model(seed):
    rng = np.random.default_rng(400 + seed)
    K = int(rng.integers(2, 17))
    n = 160
    h = rng.integers(0, 1 << 16, size=(K, n)).astype(np.uint16)
    e = ((h >> 7) & 0xFF).astype(np.uint16)
    e = (120 + (e % 12)) if seed < 2 else (e % 3)
    h = (h & np.uint16(0x807F)) | (e.astype(np.uint16) << 7)
    ins = [np.ascontiguousarray(h[j]) for j in range(K)]
    out = oracle.reduce_sum(ins, oracle.BF16)
    for i in range(n):
        acc = int(h[0, i]) << 16
        for j in range(1, K):
            acc = M.add_rne(acc, int(h[j, i]) << 16)
        assert int(out[i]) == M.narrow_f32_to_bf16(acc)


# ------------------------------------------ library routines on special cases

def test_each_add_equals_float64_add_rounded_once():
    """fl32(x + y) == (float32)((float64)x + (float64)y): the double sum of two
    binary32 values is exact or innocuously double-rounded (53 >= 2*24 + 2)."""
    rng = np.random.default_rng(7)
    n = 1 << 20
    x = _random_f32_patterns(rng, n, allow_special=False)
    y = _random_f32_patterns(rng, n, allow_special=False)
    # bring half of the pairs close in exponent so the adds round
    ey = ((x >> 23) & 0xFF).astype(np.int64) + rng.integers(-3, 4, size=n)
    ey = np.clip(ey, 0, 254).astype(np.uint32)
    y2 = (y & np.uint32(0x807FFFFF)) | (ey << 23)
    y = np.where(np.arange(n) % 2 == 0, y2, y).astype(np.uint32)
    xf, yf = x.view(np.float32), y.view(np.float32)
    out = oracle.reduce_sum([xf, yf], oracle.F32)
    with np.errstate(over="ignore"):
        want = (xf.astype(np.float64) + yf.astype(np.float64)).astype(np.float32)
    assert np.array_equal(bits32(out), bits32(want))


def test_config1_shape_against_sequential_numpy_adds():
    """K=8, n=2^20 uniform[-1,1): same in-order float32 adds done by numpy."""
    from paper_2408_14158_amd import synth
    ins = [synth.as_numpy_bits(t) for t in synth.peer_buffers_uniform_f32(8, 1 << 20, 1000)]
    out = oracle.reduce_sum(ins, oracle.F32)
    acc = ins[0].copy()
    for j in range(1, 8):
        acc = acc + ins[j]
    assert acc.dtype == np.float32
    assert np.array_equal(bits32(out), bits32(acc))


def _torch_narrow(u32: np.ndarray) -> np.ndarray:
    t = torch.from_numpy(u32.view(np.int32).copy()).view(torch.float32)
    return t.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def test_narrow_against_torch_cast_on_rounding_boundaries():
    """Every upper half with the discarded half at / next to the tie point."""
    hi = np.arange(65536, dtype=np.uint32) << 16
    for lo in (0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF):
        u = (hi | np.uint32(lo)).astype(np.uint32)
        nan = (((u >> 23) & 0xFF) == 0xFF) & ((u & 0x7FFFFF) != 0)
        got = oracle.narrow_bf16(u.view(np.float32))
        want = _torch_narrow(u)
        assert np.array_equal(got[~nan], want[~nan]), hex(lo)
        g = got[nan]
        assert np.all(((g & 0x7F80) == 0x7F80) & ((g & 0x7F) != 0))


def test_narrow_against_torch_cast_random_patterns():
    rng = np.random.default_rng(9)
    u = _random_f32_patterns(rng, 1 << 22)
    got = oracle.narrow_bf16(u.view(np.float32))
    assert np.array_equal(got, _torch_narrow(u))


def test_narrow_against_exact_model_and_invariants():
    rng = np.random.default_rng(10)
    u = _random_f32_patterns(rng, 3000, allow_special=False)
    got = oracle.narrow_bf16(u.view(np.float32))
    for a, g in zip(u.tolist(), got.tolist()):
        assert g == M.narrow_f32_to_bf16(a)
    # monotone non-decreasing on sorted finite inputs; |error| <= half an ulp
    x = np.sort(u.view(np.float32))
    y = oracle.widen_bf16(oracle.narrow_bf16(x))
    assert np.all(np.diff(y.astype(np.float64)) >= 0)
    fin = np.isfinite(y)
    xa, ya = x[fin].astype(np.float64), y[fin].astype(np.float64)
    ulp = np.maximum(np.abs(ya), 2.0 ** -126) * 2.0 ** -7
    assert np.all(np.abs(xa - ya) <= 0.5 * ulp + 1e-300)


def test_narrow_carry_and_widen_exact():
    assert oracle.narrow_bf16(f32([0x3F7FFFFF]))[0] == 0x3F80  # carry into the exponent
    assert oracle.narrow_bf16(f32([0x7F7FFFFF]))[0] == 0x7F80  # fp32 max -> +inf
    assert oracle.narrow_bf16(f32([0xFF7FFFFF]))[0] == 0xFF80
    assert oracle.narrow_bf16(f32([0x7F800000]))[0] == 0x7F80
    h = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    w = oracle.widen_bf16(h).view(np.uint32)
    assert np.array_equal(w, h.astype(np.uint32) << 16)


def test_config2_distribution_against_torch_float_pipeline():
    """bf16 N(0,1e-3) gradients, K=8: widen / add in fp32 / cast with torch ops
    in the same order reproduces the oracle (torch's cast is RNE)."""
    from paper_2408_14158_amd import synth
    ts = synth.peer_buffers_normal_bf16(8, 300001, 1e-3, 2000)
    out = oracle.reduce_sum([synth.as_numpy_bits(t) for t in ts], oracle.BF16)
    acc = ts[0].to(torch.float32)
    for t in ts[1:]:
        acc = acc + t.to(torch.float32)
    want = synth.as_numpy_bits(acc.to(torch.bfloat16))
    assert np.array_equal(out, want)


# --------------------------------------------------------------------- fp16

def _np_narrow_f16(u32: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        return u32.view(np.float32).astype(np.float16).view(np.uint16)


def test_f16_widen_every_pattern_against_numpy_and_model():
    h = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = oracle.widen_f16(h).view(np.uint32)
    want = h.view(np.float16).astype(np.float32).view(np.uint32)
    nan = ((h & 0x7C00) == 0x7C00) & ((h & 0x03FF) != 0)
    assert np.array_equal(got[~nan], want[~nan])
    g = got[nan]
    assert np.all(((g & 0x7F800000) == 0x7F800000) & ((g & 0x7FFFFF) != 0))
    for hb in list(range(0, 0x0420)) + [0x3C00, 0x7BFF, 0x8001, 0x83FF, 0xFBFF, 0x0400, 0x8400]:
        assert int(got[hb]) == M.widen_f16_to_f32(hb)


def test_f16_narrow_on_every_rounding_boundary():
    """For every pair of adjacent fp16 values: the exact midpoint (a tie in
    fp32) and its two fp32 neighbours, against numpy's cast and the model."""
    h = np.arange(0, 0x7C00, dtype=np.uint32).astype(np.uint16)          # all finite non-negative
    lo = oracle.widen_f16(h).astype(np.float64)
    hi = np.append(lo[1:], 65536.0)                                       # the value after max is 2^16
    mid = ((lo + hi) / 2).astype(np.float32)                              # exact: one more bit than fp16
    assert np.array_equal(mid.astype(np.float64), (lo + hi) / 2)
    mb = mid.view(np.uint32)
    for delta in (-1, 0, 1):
        u = (mb.astype(np.int64) + delta).astype(np.uint32)
        for sign in (0, 0x80000000):
            v = (u | np.uint32(sign)).astype(np.uint32)
            got = oracle.narrow_f16(v.view(np.float32))
            assert np.array_equal(got, _np_narrow_f16(v)), (delta, sign)
    # spot-check the model on the same boundaries
    for i in list(range(0, 1030)) + list(range(0x7BF0, 0x7C00)):
        for delta in (-1, 0, 1):
            ub = int(mb[i]) + delta
            assert int(oracle.narrow_f16(f32([ub]))[0]) == M.narrow_f32_to_f16(ub)


def test_f16_narrow_random_patterns_and_invariants():
    rng = np.random.default_rng(19)
    u = _random_f32_patterns(rng, 1 << 22)
    # concentrate half of them in the fp16 range (2^-26 .. 2^17)
    e = ((u >> 23) & 0xFF).astype(np.int64)
    e2 = (101 + (e % 44)).astype(np.uint32)
    u2 = (u & np.uint32(0x807FFFFF)) | (e2 << 23)
    u = np.where(np.arange(u.shape[0]) % 2 == 0, u2, u).astype(np.uint32)
    got = oracle.narrow_f16(u.view(np.float32))
    assert np.array_equal(got, _np_narrow_f16(u))
    x = np.sort(u2.view(np.float32)[:100000])
    y = oracle.widen_f16(oracle.narrow_f16(x))
    assert np.all(y[1:] >= y[:-1])                               # monotone (infinities included)
    assert oracle.narrow_f16(f32([0x477FF000]))[0] == 0x7C00   # 65520 -> +inf
    assert oracle.narrow_f16(f32([0x477FEFFF]))[0] == 0x7BFF   # just below -> 65504
    assert oracle.narrow_f16(f32([0x33000000]))[0] == 0x0000   # 2^-25: tie with zero -> 0
    assert oracle.narrow_f16(f32([0x33000001]))[0] == 0x0001


def test_f16_k1_identity_all_patterns_and_fp32_accumulation():
    h = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    out = oracle.reduce_sum([h], oracle.F16)
    nan = ((h & 0x7C00) == 0x7C00) & ((h & 0x03FF) != 0)
    assert np.array_equal(out[~nan], h[~nan])
    assert np.all(((out[nan] & 0x7C00) == 0x7C00) & ((out[nan] & 0x03FF) != 0))
    # K=8 against numpy: widen, add in float32 in order, cast once
    rng = np.random.default_rng(20)
    K, n = 8, 200001
    hs = [(rng.integers(0, 1 << 16, size=n).astype(np.uint16) & np.uint16(0xBFFF)) for _ in range(K)]  # |x| < 2
    acc = hs[0].view(np.float16).astype(np.float32)
    for j in range(1, K):
        acc = acc + hs[j].view(np.float16).astype(np.float32)
    want = acc.astype(np.float16).view(np.uint16)
    assert np.array_equal(oracle.reduce_sum(hs, oracle.F16), want)
    s = np.float32(0.1)
    wantc = ((hs[0].view(np.float16).astype(np.float32) + hs[1].view(np.float16).astype(np.float32)) * s)
    assert np.array_equal(oracle.combine_avg(hs[0], hs[1], 0.1, oracle.F16), wantc.astype(np.float16).view(np.uint16))
    wanta = (acc * s).astype(np.float16).view(np.uint16)
    assert np.array_equal(oracle.reduce_avg(hs, 0.1, oracle.F16), wanta)


def test_f16_general_inputs_match_integer_rounding_model():
    rng = random.Random(21)
    K, n = 6, 250
    cols = [[(rng.getrandbits(1) << 15) | (rng.randrange(0, 31) << 10) | rng.getrandbits(10) for _ in range(n)]
            for _ in range(K)]
    out = oracle.reduce_sum([np.array(c, dtype=np.uint16) for c in cols], oracle.F16)
    for i in range(n):
        acc = M.widen_f16_to_f32(cols[0][i])
        for j in range(1, K):
            acc = M.add_rne(acc, M.widen_f16_to_f32(cols[j][i]))
        if M.decode(acc, M.BINARY32)[0] == "num":
            assert int(out[i]) == M.narrow_f32_to_f16(acc)


# ---------------------------------------------------------------------- fp8

FP8_CASES = [("e4m3", oracle.FP8_E4M3, torch.float8_e4m3fn, M.E4M3), ("e5m2", oracle.FP8_E5M2, torch.float8_e5m2, M.E5M2)]


def _torch_narrow_fp8(u32: np.ndarray, tdt) -> np.ndarray:
    return torch.from_numpy(u32.view(np.int32).copy()).view(torch.float32).to(tdt).view(torch.uint8).numpy()


def _fp8_nan(b: np.ndarray, name: str) -> np.ndarray:
    return ((b & 0x7F) == 0x7F) if name == "e4m3" else (((b & 0x7C) == 0x7C) & ((b & 3) != 0))


@pytest.mark.parametrize("name,odt,tdt,fmt", FP8_CASES)
def test_fp8_widen_every_pattern(name, odt, tdt, fmt):
    b = np.arange(256, dtype=np.uint8)
    got = oracle.widen_fp8(b, odt).view(np.uint32)
    want = torch.from_numpy(b.copy()).view(tdt).to(torch.float32).view(torch.int32).numpy().view(np.uint32)
    nan = _fp8_nan(b, name)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.all(((got[nan] & 0x7F800000) == 0x7F800000) & ((got[nan] & 0x7FFFFF) != 0))
    for x in range(256):
        if not nan[x]:
            assert int(got[x]) == M.widen_fp8_to_f32(x, fmt)


@pytest.mark.parametrize("name,odt,tdt,fmt", FP8_CASES)
def test_fp8_narrow_on_every_rounding_boundary(name, odt, tdt, fmt):
    """Midpoint of every pair of adjacent values (a tie in fp32) and its two
    fp32 neighbours, both signs, and the overflow edge; against torch's cast
    and the rational model."""
    b = np.arange(0, 0x7F if name == "e4m3" else 0x7C, dtype=np.uint8)     # finite, non-negative
    lo = oracle.widen_fp8(b, odt).astype(np.float64)
    top = 2.0 * lo[-1] - lo[-2]                                             # one step beyond the largest number
    hi = np.append(lo[1:], top)
    mid = ((lo + hi) / 2).astype(np.float32)
    assert np.array_equal(mid.astype(np.float64), (lo + hi) / 2)
    mb = mid.view(np.uint32)
    pats = []
    for delta in (-1, 0, 1):
        for sign in (0, 0x80000000):
            pats.append(((mb.astype(np.int64) + delta).astype(np.uint32) | np.uint32(sign)).astype(np.uint32))
    extra = np.array([0x7F800000, 0xFF800000, 0x7F7FFFFF, 0x00000001, 0x80000001, 0, 0x80000000,
                      np.float32(top).view(np.uint32), np.float32(top * 4).view(np.uint32)], dtype=np.uint32)
    u = np.concatenate(pats + [extra])
    got = oracle.narrow_fp8(u.view(np.float32), odt)
    want = _torch_narrow_fp8(u, tdt)
    both_nan = _fp8_nan(got, name) & _fp8_nan(want, name)
    assert np.all((got == want) | both_nan)
    for ub, g in zip(u.tolist(), got.tolist()):
        w = M.narrow_f32_to_fp8(ub, fmt)
        assert g == w or (_fp8_nan(np.array([g], dtype=np.uint8), name)[0] and _fp8_nan(np.array([w], dtype=np.uint8), name)[0])


@pytest.mark.parametrize("name,odt,tdt,fmt", FP8_CASES)
def test_fp8_narrow_random_and_k8_pipeline(name, odt, tdt, fmt):
    rng = np.random.default_rng(33)
    u = _random_f32_patterns(rng, 1 << 21)
    e2 = (100 + (((u >> 23) & 0xFF) % 48)).astype(np.uint32)
    u = np.where(np.arange(u.shape[0]) % 4 != 0, (u & np.uint32(0x807FFFFF)) | (e2 << 23), u).astype(np.uint32)
    got = oracle.narrow_fp8(u.view(np.float32), odt)
    want = _torch_narrow_fp8(u, tdt)
    assert np.all((got == want) | (_fp8_nan(got, name) & _fp8_nan(want, name)))
    # K=8: widen / add in fp32 in order / cast once, with torch ops
    K, n = 8, 100003
    bs = [rng.integers(0, 256, size=n).astype(np.uint8) for _ in range(K)]
    ts = [torch.from_numpy(b.copy()).view(tdt).to(torch.float32) for b in bs]
    acc = ts[0]
    for t in ts[1:]:
        acc = acc + t
    want = acc.to(tdt).view(torch.uint8).numpy()
    got = oracle.reduce_sum(bs, odt)
    assert np.all((got == want) | (_fp8_nan(got, name) & _fp8_nan(want, name)))
    wantc = ((ts[0] + ts[1]) * np.float32(0.3)).to(tdt).view(torch.uint8).numpy()
    gotc = oracle.combine_avg(bs[0], bs[1], 0.3, odt)
    assert np.all((gotc == wantc) | (_fp8_nan(gotc, name) & _fp8_nan(wantc, name)))
    wanta = (acc * np.float32(0.125)).to(tdt).view(torch.uint8).numpy()
    gota = oracle.reduce_avg(bs, 0.125, odt)
    assert np.all((gota == wanta) | (_fp8_nan(gota, name) & _fp8_nan(wanta, name)))
    # K = 1 is the identity on every non-NaN pattern
    b = np.arange(256, dtype=np.uint8)
    out = oracle.reduce_sum([b], odt)
    nan = _fp8_nan(b, name)
    assert np.array_equal(out[~nan], b[~nan]) and np.all(_fp8_nan(out[nan], name))


# ------------------------------------------------------------------ combine

def test_combine_scale_one_is_two_way_sum():
    rng = np.random.default_rng(21)
    a = _random_f32_patterns(rng, 50001, allow_special=False).view(np.float32)
    b = _random_f32_patterns(rng, 50001, allow_special=False).view(np.float32)
    s = oracle.reduce_sum([a, b], oracle.F32)
    c = oracle.combine_avg(a, b, 1.0, oracle.F32)
    assert np.array_equal(bits32(s), bits32(c))
    ab, bb = (bits32(a) >> 16).astype(np.uint16), (bits32(b) >> 16).astype(np.uint16)
    assert np.array_equal(oracle.reduce_sum([ab, bb], oracle.BF16),
                          oracle.combine_avg(ab, bb, 1.0, oracle.BF16))


def test_combine_power_of_two_scale_is_exact():
    """scale = 2^-7 with no underflow: out * 128 == fl(a + b) bit for bit."""
    a = torch.randn(1 << 18, generator=torch.Generator().manual_seed(5000)).numpy()
    b = torch.randn(1 << 18, generator=torch.Generator().manual_seed(5001)).numpy()
    out = oracle.combine_avg(a, b, 2.0 ** -7, oracle.F32)
    with np.errstate(over="ignore"):
        s = (a.astype(np.float64) + b.astype(np.float64)).astype(np.float32)
    assert np.array_equal(bits32(out * np.float32(128.0)), bits32(s))
    z = oracle.combine_avg(a, -a, 2.0 ** -7, oracle.F32)
    assert np.all(bits32(z) == 0)


def test_combine_two_roundings_model_and_discrimination():
    """Random triples against the exact model; some of them must tell the
    two-rounding result apart from a fused and from a distributed evaluation."""
    rng = random.Random(31)
    n = 1500
    a_bits, b_bits = [], []
    for _ in range(n):
        ea = rng.randrange(110, 140)
        a_bits.append((rng.getrandbits(1) << 31) | (ea << 23) | rng.getrandbits(23))
        eb = ea + rng.randrange(-2, 3)
        b_bits.append((rng.getrandbits(1) << 31) | (eb << 23) | rng.getrandbits(23))
    s_bits = 0x3DCCCCCD  # fl(0.1): not a power of two
    a = np.array(a_bits, dtype=np.uint32).view(np.float32)
    b = np.array(b_bits, dtype=np.uint32).view(np.float32)
    out = bits32(oracle.combine_avg(a, b, f32([s_bits])[0], oracle.F32))
    sv = M.value(s_bits, M.BINARY32)
    differs_fused = differs_dist = 0
    for i in range(n):
        t = M.add_rne(a_bits[i], b_bits[i])
        want = M.mul_rne(t, s_bits)
        assert int(out[i]) == want
        exact = (M.value(a_bits[i], M.BINARY32) + M.value(b_bits[i], M.BINARY32)) * sv
        fused = M.encode_rne(exact, M.BINARY32)
        dist = M.add_rne(M.mul_rne(a_bits[i], s_bits), M.mul_rne(b_bits[i], s_bits))
        differs_fused += fused != want
        differs_dist += dist != want
    assert differs_fused > 0 and differs_dist > 0


def test_combine_bf16_three_roundings_model():
    rng = random.Random(32)
    n = 1500
    a = [(rng.getrandbits(1) << 15) | (rng.randrange(118, 130) << 7) | rng.getrandbits(7) for _ in range(n)]
    b = [(rng.getrandbits(1) << 15) | (rng.randrange(118, 130) << 7) | rng.getrandbits(7) for _ in range(n)]
    s_bits = 0x3DCCCCCD
    out = oracle.combine_avg(np.array(a, dtype=np.uint16), np.array(b, dtype=np.uint16),
                             f32([s_bits])[0], oracle.BF16)
    for i in range(n):
        t = M.add_rne(a[i] << 16, b[i] << 16)
        assert int(out[i]) == M.narrow_f32_to_bf16(M.mul_rne(t, s_bits))


# ------------------------------------------------------ buckets and aliasing

def test_bucket_cuts_do_not_change_the_result():
    from paper_2408_14158_amd import synth
    K, n = 5, 10007
    ts = synth.peer_buffers_normal_bf16(K, n, 1e-3, 77)
    ins = [synth.as_numpy_bits(t) for t in ts]
    flat = oracle.reduce_sum(ins, oracle.BF16)
    for cap in (1, 7, 1000, 4096, n, n + 5):
        outs = np.zeros(n, dtype=np.uint16)
        buckets = []
        for off, ln in synth.bucket_cuts(n, cap):
            buckets.append(([np.ascontiguousarray(a[off:off + ln]) for a in ins], outs[off:off + ln]))
        oracle.reduce_buckets(buckets, oracle.BF16)
        assert np.array_equal(outs, flat)


def test_whole_tensor_packing_covers_the_flat_buffer_without_straddling():
    """Host logic of the secondary packing of the bucketed workload: cuts are
    contiguous, cover every element once, fall on tensor edges only, every
    bucket but the last holds at least the cap, and the counts for the
    full-size tensor list are the expected ones (41 buckets, 2^25 to 131,076,096)."""
    from paper_2408_14158_amd import synth
    ts = synth.transformer_grad_tensors()
    cuts = synth.bucket_cuts_whole_tensors(ts)
    total = sum(t.numel for t in ts)
    assert total == 1_750_142_976 and len(ts) == 74
    assert cuts[0][0] == 0 and sum(l for _, l in cuts) == total
    edges = {0}
    acc = 0
    for t in reversed(ts):
        acc += t.numel
        edges.add(acc)
    for (o, l), (o2, _) in zip(cuts, cuts[1:]):
        assert o + l == o2
    assert all(o in edges and o + l in edges for o, l in cuts)
    assert all(l >= synth.BUCKET_CAP_ELEMS for _, l in cuts[:-1])
    assert len(cuts) == 41
    assert min(l for _, l in cuts) == 1 << 25 and max(l for _, l in cuts) == 131_076_096
    # same bits as the flat sum on a small instance
    small = synth.transformer_grad_tensors(n_layers=2, d_model=32, ffn=88, vocab=100)
    K = 3
    flats = [synth.as_numpy_bits(synth.flat_gradient_bf16(small, 50 + j)) for j in range(K)]
    flat = oracle.reduce_sum(flats, oracle.BF16)
    outs = np.zeros_like(flat)
    buckets = [([np.ascontiguousarray(a[o:o + l]) for a in flats], outs[o:o + l])
               for o, l in synth.bucket_cuts_whole_tensors(small, 3000)]
    assert len(buckets) > 3
    oracle.reduce_buckets(buckets, oracle.BF16)
    assert np.array_equal(outs, flat)


def test_in_place_forms():
    rng = np.random.default_rng(41)
    ins = [rng.standard_normal(1001).astype(np.float32) for _ in range(4)]
    want = oracle.reduce_sum(ins, oracle.F32)
    for j in range(4):
        work = [a.copy() for a in ins]
        oracle.reduce_sum(work, oracle.F32, out=work[j])
        assert np.array_equal(bits32(work[j]), bits32(want))
    a, b = ins[0].copy(), ins[1].copy()
    want = oracle.combine_avg(a, b, 0.25, oracle.F32)
    oracle.combine_avg(a, b, 0.25, oracle.F32, out=a)
    assert np.array_equal(bits32(a), bits32(want))


def test_empty_and_bad_arguments():
    e = np.empty(0, dtype=np.float32)
    assert oracle.reduce_sum([e, e], oracle.F32).shape == (0,)
    assert oracle.combine_avg(e, e, 1.0, oracle.F32).shape == (0,)
    with pytest.raises(ValueError):
        oracle.reduce_sum([np.zeros(3, dtype=np.float64)], oracle.F32)


# ------------------------------------------- fused average and slice variants

def test_reduce_avg_scale_one_is_the_plain_sum():
    rng = np.random.default_rng(61)
    ins = [_random_f32_patterns(rng, 30011, allow_special=False).view(np.float32) for _ in range(5)]
    assert np.array_equal(bits32(oracle.reduce_avg(ins, 1.0, oracle.F32)),
                          bits32(oracle.reduce_sum(ins, oracle.F32)))
    insb = [(bits32(a) >> 16).astype(np.uint16) for a in ins]
    assert np.array_equal(oracle.reduce_avg(insb, 1.0, oracle.BF16), oracle.reduce_sum(insb, oracle.BF16))


def test_reduce_avg_matches_rational_model():
    """fp32 sum in order, ONE multiply, ONE narrowing (bf16): exact model."""
    rng = random.Random(62)
    K, n = 8, 400
    s_bits = 0x3E000000  # 0.125 exactly; and a non power of two below
    for s_bits in (0x3E000000, 0x3DCCCCCD):
        cols = [[(rng.getrandbits(1) << 15) | (rng.randrange(120, 130) << 7) | rng.getrandbits(7)
                 for _ in range(n)] for _ in range(K)]
        out = oracle.reduce_avg([np.array(c, dtype=np.uint16) for c in cols], f32([s_bits])[0], oracle.BF16)
        differs = 0
        for i in range(n):
            acc = cols[0][i] << 16
            for j in range(1, K):
                acc = M.add_rne(acc, cols[j][i] << 16)
            want = M.narrow_f32_to_bf16(M.mul_rne(acc, s_bits))
            assert int(out[i]) == want
            # narrowing BEFORE the multiply (the two-call sequence) is a different function
            early = M.narrow_f32_to_bf16(M.mul_rne(M.narrow_f32_to_bf16(acc) << 16, s_bits))
            differs += early != want
        if s_bits == 0x3DCCCCCD:
            assert differs > 0
    # fp32
    cols = [[(rng.getrandbits(1) << 31) | (rng.randrange(120, 130) << 23) | rng.getrandbits(23)
             for _ in range(n)] for _ in range(K)]
    out = bits32(oracle.reduce_avg([np.array(c, dtype=np.uint32).view(np.float32) for c in cols],
                                   f32([0x3DCCCCCD])[0], oracle.F32))
    for i in range(n):
        acc = cols[0][i]
        for j in range(1, K):
            acc = M.add_rne(acc, cols[j][i])
        assert int(out[i]) == M.mul_rne(acc, 0x3DCCCCCD)


def test_reduce_avg_constants():
    # eight copies of 3.0 averaged with 1/8 is 3.0 exactly; 1/128 of 256 + 7 ones: 263/128 exactly in fp32
    ins = [np.full(9, 3.0, dtype=np.float32) for _ in range(8)]
    assert np.all(oracle.reduce_avg(ins, 0.125, oracle.F32) == 3.0)
    col = [np.array([0x4380], dtype=np.uint16)] + [np.array([0x3F80], dtype=np.uint16)] * 7
    got = oracle.reduce_avg(col, 1.0 / 128, oracle.BF16)
    # 263/128 = 2.0546875 = 2 * (1 + 7/256): tie between 2*(1+3/128) and 2*(1+4/128) -> even -> 0x4004
    assert int(got[0]) == 0x4004


@pytest.mark.parametrize("n,world", [(0, 3), (1, 4), (10, 3), (17, 8), (4096, 8), (100003, 7), (5, 16)])
def test_slice_bounds_partition(n, world):
    """Brute force: the slices are contiguous, disjoint, cover [0, n) and
    differ in length by at most one, longer ones first."""
    prev_end, lens = 0, []
    for r in range(world):
        b, e = oracle.slice_bounds(n, r, world)
        assert b == prev_end and e >= b
        prev_end = e
        lens.append(e - b)
    assert prev_end == n
    assert max(lens) - min(lens) <= 1 and lens == sorted(lens, reverse=True)


def test_reduce_scatter_slice_is_the_sum_restricted_to_the_slice():
    rng = np.random.default_rng(63)
    K, n, world = 4, 10007, 6
    ins = [rng.standard_normal(n).astype(np.float32) for _ in range(K)]
    full = oracle.reduce_sum(ins, oracle.F32)
    gathered = np.full(n, np.float32(-7.0))
    for r in range(world):
        out = np.full(n, np.float32(-7.0))
        oracle.reduce_scatter_slice(ins, r, world, oracle.F32, out)
        b, e = oracle.slice_bounds(n, r, world)
        assert np.array_equal(bits32(out[b:e]), bits32(full[b:e]))
        assert np.all(out[:b] == -7.0) and np.all(out[e:] == -7.0)   # untouched outside
        gathered[b:e] = out[b:e]
    assert np.array_equal(bits32(gathered), bits32(full))
    with pytest.raises(ValueError):
        oracle.reduce_scatter_slice(ins, 6, 6, oracle.F32, np.zeros(n, dtype=np.float32))


def test_broadcast_is_k_exact_copies():
    """Closed form: every destination equals the source bit for bit (NaN
    payloads included: it is a copy, no arithmetic) and is its own buffer."""
    rng = np.random.default_rng(71)
    u = rng.integers(0, 1 << 32, size=10007, dtype=np.uint64).astype(np.uint32)
    outs = oracle.broadcast(u.view(np.float32), 5, oracle.F32)
    assert len(outs) == 5 and all(np.array_equal(o.view(np.uint32), u) for o in outs)
    assert len({o.ctypes.data for o in outs}) == 5
    h = rng.integers(0, 1 << 16, size=999).astype(np.uint16)
    for dt in (oracle.BF16, oracle.F16):
        assert all(np.array_equal(o, h) for o in oracle.broadcast(h, 3, dt))
    assert oracle.broadcast(np.empty(0, dtype=np.float32), 2, oracle.F32)[0].shape == (0,)


# ------------------------------------------------------------------ mutants

def _py_sum(vals, order="ltr"):
    v = [np.float32(x) for x in vals]
    if order == "ltr":
        acc = v[0]
        for x in v[1:]:
            acc = np.float32(acc + x)
        return acc
    if order == "rtl":
        return _py_sum(list(reversed(vals)))
    if order == "tree":
        while len(v) > 1:
            v = [np.float32(v[i] + v[i + 1]) if i + 1 < len(v) else v[i] for i in range(0, len(v), 2)]
        return v[0]
    if order == "zero_start":
        acc = np.float32(0)
        for x in v:
            acc = np.float32(acc + x)
        return acc
    raise ValueError(order)


def test_pins_reject_plausible_mistakes():
    """The pinned inputs separate the paper's in-order sum from nearby wrong
    implementations (each 'mutant' is evaluated here, on the CPU)."""
    disc = [2.0 ** 24, 1, 1, 1, 1, 1, 1, -(2.0 ** 24)]
    assert _py_sum(disc, "ltr") == 0.0
    assert _py_sum(disc, "tree") != 0.0
    assert _py_sum(disc, "rtl") != 0.0
    # zero-start accumulator turns an all(-0) column into +0
    z = _py_sum([-0.0] * 8, "zero_start")
    assert np.signbit(_py_sum([-0.0] * 8, "ltr")) and not np.signbit(z)
    # accumulating in bf16 loses 256 + 7*1
    acc = torch.tensor(256.0, dtype=torch.bfloat16)
    for _ in range(7):
        acc = acc + torch.tensor(1.0, dtype=torch.bfloat16)
    assert float(acc) == 256.0  # the mutant's answer; the fixture demands 264
    # truncating instead of rounding fails the carry case 0x3F7FFFFF -> 0x3F80
    assert (0x3F7FFFFF >> 16) == 0x3F7F
    # round-half-up fails the tie-to-even case 1 + 2^-8 -> 1.0
    assert ((0x3F808000 + 0x8000) >> 16) == 0x3F81
