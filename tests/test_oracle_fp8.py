"""Pins of the oracle's fp8 KV-row format (oracle.fp8_rows): against PyTorch's own float8_e4m3fn cast on the CPU, the
format's value table written out from its definition, ties, and the minimality of the row exponent."""
import numpy as np
import torch

import oracle
from paper_2407_00023_amd import workloads as W


def table():
    """The 127 non-negative values of the format from its definition: 4 exponent bits (bias 7), 3 mantissa bits,
    subnormals at exponent field 0, no infinities, 448 the largest."""
    vals = []
    for code in range(127):
        e, m = code >> 3, code & 7
        vals.append(m * 2.0 ** -9 if e == 0 else (1 + m / 8) * 2.0 ** (e - 7))
    return np.array(vals)


def bf16(x):
    return W.f32_to_bf16_bits(np.asarray(x, np.float32))


def test_codes_equal_pytorch_cast():
    """code = round-to-nearest-even of x * 2^-k into float8_e4m3fn: the library's cast does the same rounding."""
    rng = np.random.default_rng(0)
    x = rng.standard_normal((64, 128)).astype(np.float32) * np.exp2(rng.integers(-20, 20, (64, 1))).astype(np.float32)
    x[3] *= 0.0
    x[5, :64] = 0.0
    rows = bf16(x)
    codes, exps, stored = oracle.fp8_rows(rows)
    xf = W.bf16_bits_to_f32(rows).astype(np.float64)
    y = (xf * np.exp2(-exps.astype(np.float64))[:, None]).astype(np.float32)   # exact: a power of two
    assert np.abs(y).max() <= 448.0
    want = torch.from_numpy(y).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    # (the cast gives -0 the sign bit, as the oracle does)
    np.testing.assert_array_equal(codes, want)
    back = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)
    np.testing.assert_array_equal(W.bf16_bits_to_f32(stored).astype(np.float64), back * np.exp2(exps.astype(np.float64))[:, None])


def test_every_value_of_the_format_survives():
    t = table()
    assert t[-1] == 448.0 and t[1] == 2.0 ** -9 and t[8] == 2.0 ** -6 and (np.diff(t) > 0).all()
    for k in (-9, 0, 4):
        row = np.zeros(128, np.float64)
        row[:127] = t * 2.0 ** k
        row[127] = -448.0 * 2.0 ** k
        rows = bf16(row[None])
        assert (W.bf16_bits_to_f32(rows)[0] == row).all()          # every value of the format is a bfloat16
        codes, exps, stored = oracle.fp8_rows(rows)
        assert exps[0] == k
        np.testing.assert_array_equal(codes[0, :127], np.arange(127))
        assert codes[0, 127] == 126 | 0x80
        np.testing.assert_array_equal(W.bf16_bits_to_f32(stored)[0], row.astype(np.float32))


def test_ties_go_to_the_even_mantissa_and_errors_stay_within_half_a_step():
    t = table()
    mid = (t[:-1] + t[1:]) / 2                       # representable in bfloat16: at most 5 significant bits
    row = np.zeros(128, np.float64)
    row[:126] = mid
    row[126] = 448.0                                 # fixes k = 0
    rows = bf16(row[None])
    assert (W.bf16_bits_to_f32(rows)[0] == row).all()
    codes, exps, _ = oracle.fp8_rows(rows)
    assert exps[0] == 0
    lo = np.arange(126)
    np.testing.assert_array_equal(codes[0, :126], np.where(lo % 2 == 0, lo, lo + 1))
    rng = np.random.default_rng(1)
    x = bf16(rng.standard_normal((200, 64)) * 3)
    codes, exps, stored = oracle.fp8_rows(x)
    xf, sf = W.bf16_bits_to_f32(x).astype(np.float64), W.bf16_bits_to_f32(stored).astype(np.float64)
    y = np.abs(xf) * np.exp2(-exps.astype(np.float64))[:, None]
    idx = np.searchsorted(t, y, side="right") - 1
    step = np.where(idx < 126, t[np.minimum(idx + 1, 126)] - t[idx], 0.0)
    assert (np.abs(xf - sf) <= step / 2 * np.exp2(exps.astype(np.float64))[:, None] + 0).all()


def test_row_exponent_is_the_smallest_that_fits():
    rng = np.random.default_rng(2)
    amax = np.concatenate([448.0 * np.exp2(np.arange(-30, 30)), 449.0 * np.exp2(np.arange(-10, 10)),
                           np.exp(rng.uniform(-40, 40, 300))])
    rows = np.zeros((len(amax), 64), np.float32)
    rows[:, 7] = amax
    rows[:, 9] = -amax / 3
    b = bf16(rows)
    a = np.abs(W.bf16_bits_to_f32(b)).max(axis=1).astype(np.float64)
    _, exps, _ = oracle.fp8_rows(b)
    k = exps.astype(np.float64)
    assert (a * np.exp2(-k) <= 448.0).all() and (a * np.exp2(-(k - 1)) > 448.0).all()
    zero = np.zeros((2, 64), np.uint16)
    codes, exps, stored = oracle.fp8_rows(zero)
    assert not codes.any() and not exps.any() and not stored.any()


def test_the_largest_bfloat16_values_stay_finite():
    """k stops at 119, so that 448 * 2^k is still a bfloat16; what exceeds 448 after scaling is stored as 448."""
    big = np.array([[0x7F7F, 0xFF7F, 0x7F60, 0x7F00] + [0] * 60], np.uint16)   # +-max, 1.75 * 2^127, 2^127
    codes, exps, stored = oracle.fp8_rows(big)
    assert exps[0] == 119
    assert list(codes[0, :4]) == [126, 126 | 0x80, 126, 120]
    got = W.bf16_bits_to_f32(stored)[0, :4].astype(np.float64)
    assert list(got) == [448 * 2.0 ** 119, -448 * 2.0 ** 119, 448 * 2.0 ** 119, 2.0 ** 127]
