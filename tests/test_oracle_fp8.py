"""Pins of the FP8 oracle to the published E4M3 format: the full code table from the definition, brute-force
nearest-value rounding with ties to even, saturation, and the library's conversions where one is installed
(torch.float8_e4m3fn as a second opinion)."""
import numpy as np
import pytest

from oracle import fp8


def _finite_codes():
    c = np.arange(256, dtype=np.uint8)
    return c[(c & 0x7F) != 0x7F]                      # 0x7F / 0xFF are the NaN codes


def test_code_table_landmarks():
    d = fp8.e4m3_decode
    assert d(np.array([0x00, 0x80]))[0] == 0.0 and np.signbit(d(np.array([0x80]))[0])
    assert d(np.array([0x01]))[0] == 2.0 ** -9                      # smallest subnormal
    assert d(np.array([0x07]))[0] == 7 * 2.0 ** -9 and d(np.array([0x08]))[0] == 2.0 ** -6      # largest subnormal, smallest normal
    assert d(np.array([0x38]))[0] == 1.0 and d(np.array([0x3C]))[0] == 1.5 and d(np.array([0xB8]))[0] == -1.0
    assert d(np.array([0x7E]))[0] == 448.0 and d(np.array([0x78]))[0] == 256.0
    vals = d(_finite_codes())
    assert len(np.unique(vals)) == 253                              # 254 finite codes, +0 and -0 coincide
    pos = np.sort(vals[vals > 0])
    assert np.all(np.diff(pos) > 0) and pos[0] == 2.0 ** -9 and pos[-1] == 448.0


def test_rounding_is_nearest_with_ties_to_even_by_brute_force():
    codes = _finite_codes()
    table = fp8.e4m3_decode(codes)
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.normal(size=4000) * 3, rng.uniform(-448, 448, 2000), rng.normal(size=2000) * 0.01, table,
                        0.5 * (np.sort(table)[1:] + np.sort(table)[:-1])])         # every value and every midpoint
    q, c = fp8.e4m3_round(x)
    for xi, qi, ci in zip(x, q, c):
        d = np.abs(table - xi)
        near = table[d == d.min()]
        if len(np.unique(near)) == 1:
            assert qi == near[0], (xi, qi, near)
        else:                                          # a tie between two neighbours: the one with the even mantissa
            even = [t for t, cc in zip(table, codes) if t in near and (cc & 1) == 0 and np.signbit(t) == np.signbit(xi)]
            assert qi in even, (xi, qi, near)
        assert fp8.e4m3_decode(np.array([ci]))[0] == qi and (np.signbit(qi) == bool(ci & 0x80) or qi == 0)


def test_quantize_saturates_and_takes_the_product_in_fp32():
    v, c = fp8.quantize(np.array([1e6, -1e6, 448.0, 449.0, 464.0]), 1.0)
    assert list(v) == [448.0, -448.0, 448.0, 448.0, 448.0] and list(c) == [0x7E, 0xFE, 0x7E, 0x7E, 0x7E]
    # a scale whose reciprocal is inexact in fp32: the code follows the fp32 product
    x, scale = np.array([0.3984375]), 0.3
    want = np.float32(0.3984375) * (np.float32(1.0) / np.float32(0.3))
    assert fp8.quantize(x, scale)[0][0] == fp8.e4m3_round(np.array([float(want)]))[0][0]
    # round trip of every representable value at scale 1
    t = fp8.e4m3_decode(_finite_codes())
    assert np.array_equal(fp8.quantize(t, 1.0)[0], t)


def test_against_torch_float8_when_available():
    torch = pytest.importorskip("torch")
    if not hasattr(torch, "float8_e4m3fn"):
        pytest.skip("no float8 dtype in this torch")
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.normal(size=5000) * 5, rng.uniform(-448, 448, 3000), rng.normal(size=2000) * 0.02]).astype(np.float32)
    t = torch.from_numpy(x).to(torch.float8_e4m3fn)
    q, c = fp8.e4m3_round(x.astype(np.float64))
    assert np.array_equal(t.to(torch.float32).numpy().astype(np.float64), q)
    assert np.array_equal(t.view(torch.uint8).numpy(), c)


def test_gemm_is_the_product_of_the_decoded_values():
    rng = np.random.default_rng(2)
    a, _ = fp8.quantize(rng.normal(size=(5, 16)), 0.05)
    b, _ = fp8.quantize(rng.normal(size=(3, 16)), 0.02)
    bias = rng.normal(size=3)
    want = np.array([[0.05 * 0.02 * sum(a[i, k] * b[j, k] for k in range(16)) + bias[j] for j in range(3)] for i in range(5)])
    assert np.allclose(fp8.gemm(a, b, np.float32(0.05) * np.float32(0.02), bias), want, rtol=1e-6)
