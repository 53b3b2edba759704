"""Pins of the oracle's software rounding (storage rounding of FP16 / FP8 tiles).

FP16 is pinned to numpy's binary16 conversion (an independent library routine that
rounds once from FP64); FP8 e4m3fn to a brute-force nearest-value search over the
table of all codes written from the format's definition, and to torch's e4m3fn cast.
"""
from fractions import Fraction

import numpy as np
import pytest

from oracle import gemm_mp_oracle as orc
from tests.exact import e4m3_table


def _all_half():
    codes = np.arange(65536, dtype=np.uint16)
    return codes, codes.view(np.float16).astype(np.float64)


def test_fp16_every_value_is_a_fixed_point_and_codes_round_trip():
    codes, vals = _all_half()
    finite = np.isfinite(vals)
    y, bits = orc.round_fp16(vals[finite])
    assert np.array_equal(y, vals[finite])
    assert np.array_equal(bits, codes[finite])
    for c in (0x0001, 0x03FF, 0x0400, 0x3C00, 0x7BFF, 0x8001, 0xFBFF, 0x7C00, 0xFC00):
        assert orc.fp16_value(c) == float(np.array(c, dtype=np.uint16).view(np.float16))


def test_fp16_midpoints_and_their_neighbours_match_numpy():
    codes = np.arange(0x0000, 0x7C00, dtype=np.uint16)          # positive finite, ascending
    v = codes.view(np.float16).astype(np.float64)
    mid = 0.5 * (v[:-1] + v[1:])                                 # exact in FP64
    probes = np.concatenate([mid, np.nextafter(mid, np.inf), np.nextafter(mid, -np.inf),
                             [65504.0 + 16.0, np.nextafter(65520.0, 0), np.nextafter(65520.0, np.inf), 1e300, 5e-324]])
    probes = np.concatenate([probes, -probes])
    with np.errstate(over="ignore"):
        want = probes.astype(np.float16)
    y, bits = orc.round_fp16(probes)
    assert np.array_equal(bits, want.view(np.uint16))
    assert np.array_equal(y, want.astype(np.float64))


def test_fp16_random_doubles_match_numpy_and_avoid_double_rounding():
    rng = np.random.default_rng(1)
    x = np.exp(rng.uniform(np.log(1e-9), np.log(1e5), 200000)) * rng.choice([-1.0, 1.0], 200000)
    with np.errstate(over="ignore"):
        want = x.astype(np.float16)
    y, bits = orc.round_fp16(x)
    assert np.array_equal(bits, want.view(np.uint16))
    # a value just above an FP16 midpoint that FP32 would first pull onto the midpoint
    trap = 1.0 + 2.0 ** -11 + 2.0 ** -40
    assert orc.round_fp16([trap])[0][0] == 1.0 + 2.0 ** -10
    assert float(np.float16(np.float32(trap))) == 1.0          # what double rounding would give


def test_fp16_specials():
    y, bits = orc.round_fp16(np.array([np.inf, -np.inf, 0.0, -0.0]))
    assert list(bits) == [0x7C00, 0xFC00, 0x0000, 0x8000]
    y, bits = orc.round_fp16(np.array([np.nan]))
    assert np.isnan(y[0]) and (bits[0] & 0x7C00) == 0x7C00 and (bits[0] & 0x3FF) != 0


def _brute_force_e4m3(x, table):
    """Nearest finite e4m3 value (ties to the even code); beyond the largest -> +-448."""
    fx = Fraction(x)
    sign = 1 if np.signbit(x) else 0
    best = None
    for code, v in table:
        if (code >> 7) != sign:
            continue
        d = abs(v - fx)
        if best is None or d < best[0] or (d == best[0] and code % 2 == 0):
            best = (d, code, v)
    return best[1], best[2]


def test_fp8_matches_brute_force_search_over_all_codes():
    table = e4m3_table()
    pos = sorted(v for c, v in table if c < 0x80)
    probes = []
    for a, b in zip(pos[:-1], pos[1:]):
        m = float((a + b) / 2)
        probes += [float(a), m, np.nextafter(m, np.inf), np.nextafter(m, -np.inf)]
    probes += [448.0, 449.0, 463.9, 464.0, 465.0, 480.0, 1e6, 1e300, 2.0 ** -10, 2.0 ** -10 * 1.001, 2.0 ** -11, 1e-300]
    rng = np.random.default_rng(2)
    probes += list(np.exp(rng.uniform(np.log(1e-4), np.log(600.0), 3000)))
    probes = np.array(probes + [-p for p in probes] + [0.0, -0.0])
    y, bits = orc.round_fp8(probes)
    for x, yy, bb in zip(probes, y, bits):
        code, val = _brute_force_e4m3(float(x), table)
        assert bb == code, (x, hex(bb), hex(code))
        assert Fraction(float(yy)) == val


def test_fp8_specials_saturate_and_nan():
    y, bits = orc.round_fp8(np.array([np.inf, -np.inf, np.nan, 1e10, -1e10]))
    assert list(bits[:2]) == [0x7E, 0xFE] and list(bits[3:]) == [0x7E, 0xFE]
    assert np.isnan(y[2]) and (bits[2] & 0x7F) == 0x7F
    assert y[0] == 448.0 and y[1] == -448.0


def test_fp8_decode_and_round_agree_with_torch_e4m3fn():
    torch = pytest.importorskip("torch")
    codes = torch.arange(256, dtype=torch.uint8)
    want = codes.view(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)
    got = np.array([orc.fp8_value(c) for c in range(256)])
    assert np.array_equal(np.isnan(want), np.isnan(got))
    ok = ~np.isnan(want)
    assert np.array_equal(want[ok], got[ok])
    rng = np.random.default_rng(3)
    x32 = (np.exp(rng.uniform(np.log(1e-4), np.log(440.0), 100000)) * rng.choice([-1, 1], 100000)).astype(np.float32)
    tb = torch.from_numpy(x32).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    _, bits = orc.round_fp8(x32.astype(np.float64))
    assert np.array_equal(bits, tb)


def test_bf16_matches_nearest_search_over_all_codes_and_torch():
    """BF16 (8 exponent bits, 7 fraction bits): the rounded value must be the nearest of all
    finite BF16 numbers (decoded here from the bit fields, ties to the even code), for doubles
    that FP32 cannot hold too (no detour through FP32); on FP32 inputs it must equal torch's
    cast; every code decodes to what torch decodes it to."""
    torch = pytest.importorskip("torch")
    codes = np.arange(0x7F80, dtype=np.int64)                      # non-negative finite codes, ascending in value
    e, m = codes >> 7, codes & 127
    table = np.where(e == 0, np.ldexp(m.astype(np.float64), -133), np.ldexp(1.0 + m / 128.0, (e - 127).astype(np.int64)))
    assert np.all(np.diff(table) > 0)
    got = np.array([orc.bf16_value(int(c)) for c in range(0, 0x7F80, 37)])
    assert np.array_equal(got, table[::37])
    want_t = torch.arange(0, 0x7F80, 37, dtype=torch.int32).to(torch.int16).view(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(got, want_t)
    rng = np.random.default_rng(5)
    x = np.concatenate([
        np.exp(rng.uniform(np.log(1e-42), np.log(3e38), 20000)),
        (table[1000:3000] + table[1001:3001]) / 2,                      # midpoints: ties
        np.nextafter((table[1000:3000] + table[1001:3001]) / 2, np.inf),
        np.nextafter((table[1000:3000] + table[1001:3001]) / 2, -np.inf),
        (table[:300] + table[1:301]) / 2,                               # the subnormal range
        1.0 + 2.0 ** -8 + np.array([0.0, 2.0 ** -40, -2.0 ** -40]),     # a tie FP32 would break the other way
        [0.0, 2.0 ** -134, 2.0 ** -134 * 1.0001, 2.0 ** -140]])
    y, bits = orc.round_bf16(x)
    idx = np.searchsorted(table, x)
    lo = np.clip(idx - 1, 0, len(table) - 1)
    hi = np.clip(idx, 0, len(table) - 1)
    dlo, dhi = x - table[lo], table[hi] - x                             # exact: neighbours within a factor of two
    pick_hi = (dhi < dlo) | ((dhi == dlo) & (hi % 2 == 0))
    want = np.where(pick_hi, hi, lo)
    assert np.array_equal(bits.astype(np.int64), want)
    assert np.array_equal(y, table[want])
    y, bits = orc.round_bf16(-x)
    assert np.array_equal(bits.astype(np.int64), want | 0x8000)
    x32 = (np.exp(rng.uniform(np.log(1e-30), np.log(1e30), 100000)) * rng.choice([-1, 1], 100000)).astype(np.float32)
    tb = torch.from_numpy(x32).to(torch.bfloat16).view(torch.int16).numpy().astype(np.uint16)
    assert np.array_equal(orc.round_bf16(x32.astype(np.float64))[1], tb)
    y, bits = orc.round_bf16(np.array([np.inf, -np.inf, np.nan, 3.4e38, -3.4e38, 3.39e38]))
    assert list(bits[:2]) == [0x7F80, 0xFF80] and np.isnan(y[2])
    assert y[3] == np.inf and y[4] == -np.inf and np.isfinite(y[5])


def test_mxfp8_blocks_scale_window_nearest_elements_and_exactness():
    """MXFP8 (block of 32, one power-of-two scale): the scale is floor(log2 max) - 8, so the largest
    scaled magnitude lies in [2^8, 2^9) (and saturates at 448 above it); every element is the
    e4m3 number nearest to x * 2^-s (brute force over the code table); blocks of integers up to
    15 in magnitude come back exactly; zero blocks have scale code 127."""
    table = e4m3_table()
    rng = np.random.default_rng(9)
    x = rng.standard_normal((200, 32)) * np.exp(rng.uniform(-60, 60, (200, 1))) * np.exp(rng.uniform(-6, 0, (200, 32)))
    y, codes, scales = orc.mx_blocks(x)
    for b in range(200):
        s = int(scales[b]) - 127
        m = np.abs(x[b]).max()
        assert s == int(np.floor(np.log2(m))) - 8
        assert 2.0 ** 8 <= m * 2.0 ** -s < 2.0 ** 9
        for k in range(0, 32, 5):
            code, val = _brute_force_e4m3(float(np.ldexp(x[b, k], -s)), table)
            assert codes[b, k] == code and Fraction(float(y[b, k])) == val
    ints = rng.integers(-14, 15, (50, 32)).astype(np.float64)
    ints[0] = 0.0
    y, codes, scales = orc.mx_blocks(ints)
    assert scales[0] == 127 and not y[0].any()
    assert np.array_equal(np.ldexp(y, (scales.astype(np.int64) - 127)[:, None]), ints)
    y, codes, scales = orc.mx_blocks(np.array([15.0] + [1.0] * 31))
    assert y[0] * 2.0 ** (int(scales[0]) - 127) == 14.0 and y[1] * 2.0 ** (int(scales[0]) - 127) == 1.0
    # the E8M0 range is kept
    y, codes, scales = orc.mx_blocks(np.full(32, 1e-60))
    assert scales[0] == 0


def test_mxfp4_blocks_scale_window_and_nearest_e2m1_elements():
    """MXFP4: e2m1 elements (magnitudes 0, 0.5, 1, 1.5, 2, 3, 4, 6; code = sign, two exponent bits,
    one fraction bit), scale 2^(floor(log2 max) - 2); every element is the grid value nearest to
    x * 2^-s with ties to the even code and saturation at 6 (the grid is written out here)."""
    grid = [Fraction(0), Fraction(1, 2), Fraction(1), Fraction(3, 2), Fraction(2), Fraction(3), Fraction(4), Fraction(6)]
    rng = np.random.default_rng(10)
    x = rng.standard_normal((300, 32)) * np.exp(rng.uniform(-40, 40, (300, 1))) * np.exp(rng.uniform(-3, 0, (300, 32)))
    x[0, :8] = [0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 4.0]       # ties of the grid at scale 1 (largest entry 5 -> s = 0)
    x[0, 8:] = 0.0
    y, codes, scales = orc.mx4_blocks(x)
    for b in range(300):
        s = int(scales[b]) - 127
        m = np.abs(x[b]).max()
        assert s == int(np.floor(np.log2(m))) - 2 and 4.0 <= m * 2.0 ** -s < 8.0
        for k in range(32):
            v = abs(Fraction(float(np.ldexp(x[b, k], -s))))
            best = min(range(8), key=lambda c: (abs(grid[c] - v), c & 1))          # nearest, ties to the even code
            if v > 6:
                best = 7
            assert int(codes[b, k]) & 7 == best and Fraction(float(abs(y[b, k]))) == grid[best], (b, k, float(v))
            assert (int(codes[b, k]) >> 3) == (1 if x[b, k] < 0 and best else int(codes[b, k]) >> 3)
    assert list(y[0, :8]) == [0.0, 1.0, 1.0, 2.0, 2.0, 4.0, 4.0, 4.0]
    ints = rng.integers(-3, 4, (40, 32)).astype(np.float64)
    y, codes, scales = orc.mx4_blocks(ints)
    assert np.array_equal(np.ldexp(y, (scales.astype(np.int64) - 127)[:, None]), ints)


def test_mxfp6_blocks_scale_window_and_nearest_e2m3_elements():
    """MXFP6: e2m3 elements (code = sign, two exponent bits with bias 1, three fraction bits: the
    32 magnitudes are the multiples of 1/8 below 2, of 1/4 from 2 to 4 and of 1/2 from 4 to 7.5,
    written out here from the bit fields), scale 2^(floor(log2 max) - 2); every element is the grid
    value nearest to x * 2^-s with ties to the even code and saturation at 7.5; the 6-bit code is
    the index into the ascending grid plus 32 for a negative number; blocks of integers up
    to 7 in magnitude come back exactly."""
    grid = []
    for code in range(32):
        e, m = code >> 3, code & 7
        grid.append(Fraction(m, 8) if e == 0 else (1 + Fraction(m, 8)) * 2 ** (e - 1))
    assert grid == sorted(grid) and grid[8] == 1 and grid[-1] == Fraction(15, 2) and grid[1] == Fraction(1, 8)
    rng = np.random.default_rng(12)
    x = rng.standard_normal((300, 32)) * np.exp(rng.uniform(-40, 40, (300, 1))) * np.exp(rng.uniform(-4, 0, (300, 32)))
    # ties of the grid at scale 1 (largest entry 5 -> s = 0): subnormal step, the three normal steps, and beyond the top
    x[0, :12] = [1 / 16, 3 / 16, 1.0625, 1.1875, 2.125, 2.375, 4.25, 4.75, 5.0, 7.75, -7.25, 7.6]
    x[0, 12:] = 0.0
    x[0, 8] = 5.0
    x[1, :4] = [4.0, 7.75, -7.9, 7.5]                               # largest entry 7.9 -> s = 0: saturation at 7.5
    x[1, 4:] = 0.0
    y, codes, scales = orc.mx6_blocks(x)
    for b in range(300):
        s = int(scales[b]) - 127
        m = np.abs(x[b]).max()
        assert s == int(np.floor(np.log2(m))) - 2 and 4.0 <= m * 2.0 ** -s < 8.0
        for k in range(32):
            v = abs(Fraction(float(np.ldexp(x[b, k], -s))))
            best = min(range(32), key=lambda c: (abs(grid[c] - v), c & 1))         # nearest, ties to the even code
            if v > grid[31]:
                best = 31
            assert int(codes[b, k]) & 31 == best and Fraction(float(abs(y[b, k]))) == grid[best], (b, k, float(v))
            if best:
                assert (int(codes[b, k]) >> 5) == (1 if x[b, k] < 0 else 0)
            assert int(codes[b, k]) < 64
    assert list(y[0, :8]) == [0.0, 0.25, 1.0, 1.25, 2.0, 2.5, 4.0, 5.0]
    assert list(y[1, :4]) == [4.0, 7.5, -7.5, 7.5]
    ints = rng.integers(-7, 8, (40, 32)).astype(np.float64)
    ints[0] = 0.0
    y, codes, scales = orc.mx6_blocks(ints)
    assert scales[0] == 127 and not y[0].any()
    assert np.array_equal(np.ldexp(y, (scales.astype(np.int64) - 127)[:, None]), ints)
    # NaN has no code: stored as zero, and it does not enter the block maximum; infinities saturate
    y, codes, scales = orc.mx6_blocks(np.array([np.nan, 3.0, -np.inf] + [0.5] * 29))
    assert y[0] == 0.0 and scales[0] == 127 and y[1] == 3.0 and y[2] == -7.5
