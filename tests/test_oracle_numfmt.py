"""Pins for the oracle's number-format code and the generators' encoders (CPU only)."""
import math
import os

import numpy as np
import torch

from oracle import numfmt
from paper_2105_14450_amd import synth


def test_golden_bit_patterns(golden_dir):
    n = 0
    for line in open(os.path.join(golden_dir, "number_formats.txt")):
        if line.startswith("#") or not line.strip():
            continue
        fmt, pat, val = line.split()
        code = int(pat, 16)
        got = (numfmt.decode_bf16(np.array([code], dtype=np.uint16))[0] if fmt == "bf16"
               else numfmt.decode_e4m3(np.array([code], dtype=np.uint8))[0])
        if val == "nan":
            assert math.isnan(got)
        else:
            assert got == float(val), (fmt, pat)
        n += 1
    assert n == 19


def test_bf16_decode_all_patterns_against_torch():
    bits = np.arange(65536, dtype=np.uint16)
    ours = numfmt.decode_bf16(bits)
    t = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(ours, t)      # NaNs compare equal position-wise here


def test_e4m3_decode_all_patterns_against_torch():
    codes = np.arange(256, dtype=np.uint8)
    ours = numfmt.decode_e4m3(codes)
    t = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    np.testing.assert_array_equal(ours, t)
    assert np.nanmax(np.abs(ours)) == 448.0
    np.testing.assert_array_equal(numfmt.decode_e4m3(codes, 0.5)[:0x7F], ours[:0x7F] * 0.5)


def test_round_to_bf16_ties_and_torch():
    # ties go to the even neighbour
    assert numfmt.round_to_bf16(1.0 + 2.0 ** -8) == 1.0
    assert numfmt.round_to_bf16(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6
    assert numfmt.round_to_bf16(-(1.0 + 2.0 ** -8)) == -1.0
    # just above a tie goes up even though the fp32 rounding of it would hit the tie
    assert numfmt.round_to_bf16(1.0 + 2.0 ** -8 + 2.0 ** -40) == 1.0 + 2.0 ** -7
    assert numfmt.round_to_bf16(0.0) == 0.0
    assert numfmt.round_to_bf16(2.0 ** -134) == 0.0            # half the smallest subnormal: tie to even
    assert numfmt.round_to_bf16(3 * 2.0 ** -134) == 2.0 ** -132
    assert numfmt.round_to_bf16(3.4e38) == np.inf
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-30, 30, 20000),
                        rng.integers(-70000, 70000, 5000)]).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(numfmt.round_to_bf16(x.astype(np.float64)), ref)
    np.testing.assert_array_equal(
        numfmt.bf16_bits(ref),
        torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))


def test_generator_encoders_against_oracle_decoders():
    rng = np.random.default_rng(2)
    x = (rng.standard_normal(50000) * 3).astype(np.float32)
    # bf16: the encoder (generators) followed by the decoder (oracle) is the oracle's own rounding
    bits = synth.f32_to_bf16_bits(x)
    np.testing.assert_array_equal(numfmt.decode_bf16(bits), numfmt.round_to_bf16(x.astype(np.float64)))
    # e4m3: decode(encode(x)) is the nearest representable value, saturating at 448
    scale = 0.01
    codes = synth.f32_to_e4m3(x, scale)
    back = numfmt.decode_e4m3(codes, scale)
    grid = np.sort(numfmt.decode_e4m3(np.arange(256, dtype=np.uint8))[~np.isnan(
        numfmt.decode_e4m3(np.arange(256, dtype=np.uint8)))]) * scale
    clipped = np.clip(x.astype(np.float64), -448 * scale, 448 * scale)
    nearest = np.min(np.abs(clipped[:, None] - grid[None, :]), axis=1)
    np.testing.assert_allclose(np.abs(back - clipped), nearest, rtol=0, atol=1e-15)
    t = (torch.from_numpy(x.astype(np.float64) / scale).to(torch.float32).clamp(-448, 448)
         .to(torch.float8_e4m3fn).view(torch.uint8).numpy())
    exact = (x.astype(np.float64) / scale).astype(np.float32).astype(np.float64) == x.astype(np.float64) / scale
    zero = (codes & 0x7F) == 0                    # sign of zero may differ; value is the same
    ok = exact & ~zero
    np.testing.assert_array_equal(codes[ok], t[ok])
    # small integers are stored exactly in every format
    ints = np.arange(-4, 5).astype(np.float32)
    np.testing.assert_array_equal(numfmt.decode_bf16(synth.f32_to_bf16_bits(ints)), ints)
    np.testing.assert_array_equal(numfmt.decode_e4m3(synth.f32_to_e4m3(ints, 1.0)), ints)


def test_streams_are_seeded_and_independent():
    a = synth.draw((4, 5), "normal", 3, synth.TID_X)
    b = synth.draw((4, 5), "normal", 3, synth.TID_X)
    c = synth.draw((4, 5), "normal", 3, synth.TID_W)
    np.testing.assert_array_equal(a, b)
    assert not np.array_equal(a, c)
    ints = synth.draw((1000,), "int", 1, 1)
    assert ints.min() == -4 and ints.max() == 4
    u = synth.draw((1000,), "uniform", 1, 1)
    assert -1 <= u.min() and u.max() < 1
