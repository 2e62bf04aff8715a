"""Pins of the RTN quantizer oracle (CPU): worked examples, exact recoveries, the error bound,
nearest-level brute force, and the packer against the independent C unpacker."""
import itertools

import numpy as np
import pytest

import oracle
from oracle import rtn


def f16(bits):
    return np.asarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)


def test_worked_example_two_bits():
    """Group {-1, 0, 0.75, 2} (repeated to fill 32), 2 bits: range 3 over 3 steps -> scale 1,
    zero point 1, codes rne(w) + 1 = 0, 1, 2, 3."""
    W = np.tile(np.array([-1.0, 0.0, 0.75, 2.0], dtype=np.float32), 8)[None, :]
    codes, scales, zeros = rtn.quantize(W, 2, 32)
    assert f16(scales)[0, 0] == 1.0 and zeros[0, 0] == 1
    assert codes[0, :4].tolist() == [0, 1, 2, 3]
    # ties go to the even integer before the zero point is added: 0.5 -> 0 -> code 1, 1.5 -> 2 -> code 3
    W2 = np.tile(np.array([-1.0, 0.5, 1.5, 2.0], dtype=np.float32), 8)[None, :]
    assert rtn.quantize(W2, 2, 32)[0][0, :4].tolist() == [0, 1, 3, 3]
    # packed: 16 codes per word, LSB first: pattern 0,1,2,3 = 0b11100100 per byte
    q, _, _ = rtn.quantize_packed(W, 2, 32)
    assert q.shape == (2, 1) and q[0, 0] == 0xE4E4E4E4 and q[1, 0] == 0xE4E4E4E4


def test_three_bit_word_straddle_by_hand():
    """32 codes of 3 bits fill 3 words; code 10 occupies stream bits 30..32 and code 21 bits 63..65."""
    codes = np.zeros((1, 32), dtype=np.uint8)
    codes[0, 10] = 0b101
    codes[0, 21] = 0b110
    w = rtn.pack(codes, 3)[:, 0]
    assert w[0] == (0b01 << 30) and w[1] == (0b1 | (0b0 << 31)) and w[2] == 0b11
    assert np.array_equal(oracle.unpack(rtn.pack(codes, 3), 32, 1, 3), codes)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_pack_round_trips_through_the_c_unpacker(bits):
    rng = np.random.default_rng(bits)
    codes = rng.integers(0, 1 << bits, size=(24, 160), dtype=np.uint8)
    assert np.array_equal(oracle.unpack(rtn.pack(codes, bits), 160, 24, bits), codes)


@pytest.mark.parametrize("bits,group", [(2, 32), (3, 64), (4, 128)])
def test_weights_on_a_grid_are_recovered_exactly(bits, group):
    """W built as (q - z) * s with power-of-two s and both end codes present in every group:
    the quantizer must return exactly q, z and s."""
    rng = np.random.default_rng(10 + bits)
    N, K = 16, 4 * group
    maxq = (1 << bits) - 1
    q = rng.integers(0, maxq + 1, size=(N, K))
    qg = q.reshape(N, K // group, group)
    qg[:, :, 0], qg[:, :, 1] = 0, maxq
    z = rng.integers(1, maxq, size=(N, K // group))           # strictly inside: the range contains zero
    s = 2.0 ** rng.integers(-8, -2, size=(N, K // group))
    W = ((qg - z[:, :, None]) * s[:, :, None]).reshape(N, K).astype(np.float32)
    codes, scales, zeros = rtn.quantize(W, bits, group)
    assert np.array_equal(codes, q.astype(np.uint8))
    assert np.array_equal(f16(scales), s.T) and np.array_equal(zeros, z.T.astype(np.uint8))


@pytest.mark.parametrize("bits,group", [(2, 64), (3, 32), (4, 128), (4, 256)])
def test_round_trip_error_bound_and_range(bits, group):
    rng = np.random.default_rng(20 + bits)
    N, K = 40, 2 * group
    W = (rng.normal(size=(N, K)) * rng.lognormal(sigma=2.0, size=(N, 1)) * 0.02).astype(np.float32)
    W[3] = np.abs(W[3])                                   # an all-positive row: the range is widened to zero
    W[4] = 0.0                                            # a degenerate group
    W[5, :group] = -np.abs(W[5, :group])
    qw, scales, zeros = rtn.quantize_packed(W, bits, group)
    back = oracle.dequant_f32(qw, scales, zeros, K, N, bits, group).astype(np.float64)   # the C dequantizer
    s = np.repeat(f16(scales).T, group, axis=1)           # [N][K]
    assert np.all(np.abs(W.astype(np.float64) - back) <= s * (0.5 + 2.0 ** -20))
    assert np.all(back[4] == 0.0)
    # the scale is tight: no smaller binary16 would cover the range (or it is the floor 2^-14)
    Wg = W.reshape(N, K // group, group).astype(np.float64)
    span = np.maximum(Wg.max(axis=2), 0) - np.minimum(Wg.min(axis=2), 0)
    need = span / ((1 << bits) - 1)
    sc = f16(scales).T
    below = (scales.T - 1).view(np.float16).astype(np.float64)
    assert np.all(sc >= need * (1 - 2.0 ** -23))
    assert np.all((below < need * (1 + 2.0 ** -23)) | (sc == 2.0 ** -14))


def test_codes_are_the_nearest_levels_brute_force():
    """For every weight, no other code of the group's grid is closer (ties aside)."""
    rng = np.random.default_rng(5)
    bits, group, N = 3, 32, 6
    W = rng.normal(size=(N, group)).astype(np.float32)
    codes, scales, zeros = rtn.quantize(W, bits, group)
    s, z = f16(scales)[0], zeros[0].astype(np.float64)
    for n, k in itertools.product(range(N), range(group)):
        errs = [abs(float(W[n, k]) - (c - z[n]) * s[n]) for c in range(1 << bits)]
        assert errs[codes[n, k]] <= min(errs) + 1e-6 * s[n]


def test_f16_round_up():
    x = np.array([1.0, 1.0 + 2.0 ** -12, 1.0 + 2.0 ** -10, 6.1e-5, 0.3333333], dtype=np.float32)
    up = rtn.f16_round_up(x).view(np.float16).astype(np.float32)
    assert np.all(up >= x)
    down = (rtn.f16_round_up(x) - 1).view(np.float16).astype(np.float32)
    assert np.all((down < x))
    assert up[0] == 1.0 and up[1] == np.float32(1.0 + 2.0 ** -10) and up[2] == np.float32(1.0 + 2.0 ** -10)


def test_planted_mistakes_are_caught():
    """One plausible mistake each (in a copy of the rule, on the CPU): the pins above would fail."""
    rng = np.random.default_rng(6)
    bits, group = 4, 32
    W = rng.normal(size=(8, 64)).astype(np.float32)
    codes, scales, zeros = rtn.quantize(W, bits, group)
    s = np.repeat(f16(scales).T, group, axis=1)
    z = np.repeat(zeros.T.astype(np.float64), group, axis=1)
    good = (codes - z) * s
    assert np.all(np.abs(W - good) <= s * (0.5 + 2.0 ** -20))
    truncated = np.clip(np.floor(W / s) + z, 0, 15)                # floor instead of round
    assert np.any(np.abs(W - (truncated - z) * s) > s * 0.51)
    # a scale rounded to the nearest binary16 instead of up: some groups no longer span their range,
    # which is what the tightness pin (scale >= range / levels) checks
    Wbig = rng.normal(size=(64, 64)).astype(np.float32)
    Wg = Wbig.reshape(64, 2, 32).astype(np.float64)
    need = (np.maximum(Wg.max(axis=2), 0) - np.minimum(Wg.min(axis=2), 0)) / 15
    nearest = need.astype(np.float32).astype(np.float16).astype(np.float64)
    assert np.any(nearest < need)
    assert np.all(f16(rtn.quantize(Wbig, bits, group)[1]).T >= need * (1 - 2.0 ** -23))
