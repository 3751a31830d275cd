"""Pins for the oracle's bf16 conversion: field-by-field decoding, round trip
over every bit pattern, hand-computed ties, and agreement with the input
generator's independent fp32->bf16 rounding."""
import numpy as np

from oracle import bf16
from paper_2604_26837_amd import synth


def test_decode_matches_field_formula_for_every_pattern():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    a, b = bf16.decode(bits), bf16.decode_fields(bits)
    nan = np.isnan(a)
    assert np.array_equal(nan, np.isnan(b))
    assert np.array_equal(a[~nan], b[~nan])


def test_known_values():
    assert bf16.decode(np.uint16(0x3F80)) == 1.0
    assert bf16.decode(np.uint16(0xC000)) == -2.0
    assert bf16.decode(np.uint16(0x3F81)) == 1.0 + 2.0 ** -7
    assert bf16.decode(np.uint16(0x0001)) == 2.0 ** -133
    assert bf16.decode(np.uint16(0x7F7F)) == (2.0 - 2.0 ** -7) * 2.0 ** 127


def test_encode_round_trip_every_finite_pattern():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = bf16.decode(bits)
    keep = ~np.isnan(vals)
    assert np.array_equal(bf16.encode_rne(vals[keep]), bits[keep])


def test_encode_ties_to_even_and_neighbours():
    one = 0x3F80
    ulp = 2.0 ** -7
    assert bf16.encode_rne(1.0 + ulp / 2) == one            # tie -> even (mantissa 0)
    assert bf16.encode_rne(1.0 + 3 * ulp / 2) == one + 2    # tie -> even (mantissa 2)
    assert bf16.encode_rne(1.0 + ulp / 2 + 1e-9) == one + 1
    assert bf16.encode_rne(1.0 + ulp / 2 - 1e-9) == one
    assert bf16.encode_rne(-(1.0 + 3 * ulp / 2)) == 0x8000 | (one + 2)
    assert bf16.encode_rne(2.0 - ulp / 2) == 0x4000          # rounds up across the binade
    assert bf16.encode_rne(1e40) == 0x7F80
    assert bf16.encode_rne(2.0 ** -134) == 0                 # tie -> even (0)
    assert bf16.encode_rne(3 * 2.0 ** -134) == 2             # tie -> even (2)


def test_generator_rounding_agrees_with_oracle_encoding():
    rng = np.random.default_rng(7)
    x = np.concatenate([rng.standard_normal(4000), rng.standard_normal(1000) * 1e-3,
                        rng.standard_normal(1000) * 1e4]).astype(np.float32)
    # add exact ties
    ties = (1.0 + (2 * np.arange(64) + 1) * 2.0 ** -8).astype(np.float32)
    x = np.concatenate([x, ties, -ties])
    assert np.array_equal(synth.f32_to_bf16_bits(x), bf16.encode_rne(x.astype(np.float64)))
    assert np.array_equal(synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(x)).astype(np.float64),
                          bf16.decode(synth.f32_to_bf16_bits(x)))
