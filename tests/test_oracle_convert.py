"""Pins for the oracle's downcasts (nearest representable, ties to even).

The converters are found by search over the target format's value list; here
they are held against (a) torch's CPU casts, a library routine, over all
65,536 bf16 inputs, (b) closed-form values of the formats, (c) a brute-force
linear scan written differently from the oracle's bisection.
"""
import math

import numpy as np
import torch


def _all_bf16():
    bits = np.arange(65536, dtype=np.uint16)
    return bits, torch.from_numpy(bits.astype(np.int16)).view(torch.bfloat16)


def test_fp16_matches_torch_cpu_cast_exhaustively(oracle):
    bits, x = _all_bf16()
    ref = x.to(torch.float16).view(torch.int16).numpy().astype(np.uint16)
    got = np.array([oracle.bf16_to_fp16(int(b)) for b in bits], dtype=np.uint16)
    xf = x.float().numpy()
    nan = np.isnan(xf)
    assert (got[~nan] == ref[~nan]).all()
    # NaN: quiet NaN, sign kept
    assert (got[nan] == ((bits[nan] & 0x8000) | 0x7E00)).all()
    assert np.isnan(torch.from_numpy(ref[nan].astype(np.int16)).view(torch.float16).float().numpy()).all()


def test_fp8_matches_torch_cpu_cast_in_range(oracle):
    bits, x = _all_bf16()
    xf = x.float().numpy()
    in_range = np.isfinite(xf) & (np.abs(xf) <= 464.0)
    ref = x.to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([oracle.bf16_to_fp8(int(b)) for b in bits], dtype=np.uint8)
    assert (got[in_range] == ref[in_range]).all()
    # beyond the range: saturate to +-448, NaN stays NaN with its sign
    big = ~np.isnan(xf) & (np.abs(xf) > 464.0)
    assert (got[big] == np.where(bits[big] & 0x8000, 0xFE, 0x7E)).all()
    nan = np.isnan(xf)
    assert (got[nan] == np.where(bits[nan] & 0x8000, 0xFF, 0x7F)).all()


def _bf16_bits(v: float) -> int:
    return int(torch.tensor([v], dtype=torch.float32).to(torch.bfloat16).view(torch.int16).item()) & 0xFFFF


def test_fp8_closed_form_values(oracle):
    cases = {448.0: 0x7E, 464.0: 0x7E, 480.0: 0x7E, 1.0: 0x38, 2.0 ** -9: 0x01, 2.0 ** -10: 0x00,
             1.5 * 2.0 ** -9: 0x02,      # tie between 0x01 and 0x02 -> even
             0.0: 0x00, -1.0: 0xB8, 0.875 * 2 ** -6: 0x07, 2.0 ** -6: 0x08,
             432.0: 0x7E,                # tie 416 (0x7D) / 448 (0x7E) -> even code 0x7E
             float("inf"): 0x7E, float("-inf"): 0xFE}
    for v, code in cases.items():
        b = _bf16_bits(v)
        assert oracle.bf16_to_fp8(b) == code, (v, hex(oracle.bf16_to_fp8(b)), hex(code))
    assert oracle.bf16_to_fp8(0x8000) == 0x80                     # -0 keeps its sign
    assert oracle.bf16_to_fp8(_bf16_bits(-(2.0 ** -11))) == 0x80  # tiny negative -> -0
    # decode table closed form: (-1)^s 2^(e-7) (1 + m/8), subnormal 2^-6 m/8
    for c in range(256):
        s, e, m = c >> 7, (c >> 3) & 15, c & 7
        v = oracle.fp8_value(c)
        if e == 15 and m == 7:
            assert math.isnan(v)
        elif e == 0:
            assert v == (-1) ** s * 2.0 ** -6 * m / 8
        else:
            assert v == (-1) ** s * 2.0 ** (e - 7) * (1 + m / 8)
    assert oracle.fp8_value(0x7E) == 448.0


def test_fp8_brute_force_linear_scan(oracle):
    """Second route, exhaustive: for every one of the 65,536 bf16 inputs the nearest of the 127
    finite magnitudes (a 65,536 x 127 distance matrix), ties to the even code, magnitudes
    beyond 448 and infinities saturating to 448, NaN to sign | 0x7F."""
    mags = np.array([oracle.fp8_value(c) for c in range(0x7F)], dtype=np.float64)
    assert np.all(np.diff(mags) > 0)
    bits, x = _all_bf16()
    xf = x.float().numpy().astype(np.float64)
    nan = np.isnan(xf)
    a = np.minimum(np.abs(np.where(nan, 0.0, xf)), 1000.0)            # beyond the largest magnitude: saturates
    d = np.abs(a[:, None] - mags[None, :])                             # exact: both are short binary fractions
    dmin = d.min(axis=1, keepdims=True)
    is_best = d == dmin
    assert is_best.sum(axis=1).max() <= 2                              # a tie is between two neighbours
    first = is_best.argmax(axis=1)
    last = 126 - is_best[:, ::-1].argmax(axis=1)
    code = np.where(first == last, first, np.where(first % 2 == 0, first, last))   # of two neighbours one is even
    sign = np.where((np.arange(65536) & 0x8000) != 0, 0x80, 0)
    want = np.where(nan, sign | 0x7F, sign | code)
    got = np.array([oracle.bf16_to_fp8(b) for b in range(65536)])
    bad = np.flatnonzero(got != want)
    assert bad.size == 0, [(hex(int(b)), hex(int(got[b])), hex(int(want[b]))) for b in bad[:8]]


def test_fp16_closed_form_values(oracle):
    cases = {1.0: 0x3C00, 65280.0: 0x7BF8, 65536.0: 0x7C00, 2.0 ** -24: 0x0001,
             2.0 ** -25: 0x0000,         # tie between 0 and the smallest subnormal -> even (0)
             3 * 2.0 ** -25: 0x0002,     # tie between 0x0001 and 0x0002 -> even
             2.0 ** -26: 0x0000, -2.0: 0xC000, float("inf"): 0x7C00, float("-inf"): 0xFC00,
             1e38: 0x7C00}
    for v, code in cases.items():
        assert oracle.bf16_to_fp16(_bf16_bits(v)) == code, v
    assert oracle.bf16_to_fp16(0x8000) == 0x8000
    # 65520 is not a bf16 value; the largest bf16 below 65536 is 65280 -> exact in fp16?
    b = _bf16_bits(65280.0)
    assert oracle.fp16_value(oracle.bf16_to_fp16(b)) == 65280.0
