"""Pins for the oracle's bf16 / fp32 rounding helpers (CPU only)."""
import numpy as np
import torch

from oracle import flux_oracle as fo


def test_bf16_exhaustive_round_trip():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    x = fo.bf16_bits_to_f64(bits)
    back = fo.f64_to_bf16_bits(x)
    nan = np.isnan(x)
    assert np.array_equal(back[~nan], bits[~nan])
    assert np.all(np.isnan(fo.bf16_bits_to_f64(back[nan])))


def test_bf16_decode_matches_closed_form():
    # value = (-1)^s * 2^(e-127) * (1 + m/128) for normal numbers
    for s, e, m in [(0, 127, 0), (1, 127, 0), (0, 128, 64), (0, 120, 1), (1, 134, 127), (0, 1, 0)]:
        bits = np.array([(s << 15) | (e << 7) | m], dtype=np.uint16)
        want = (-1.0) ** s * 2.0 ** (e - 127) * (1 + m / 128.0)
        assert fo.bf16_bits_to_f64(bits)[0] == want
    # subnormal: 2^-126 * m/128
    assert fo.bf16_bits_to_f64(np.array([3], dtype=np.uint16))[0] == 2.0 ** -126 * 3 / 128


def test_rne_ties_to_even_on_hand_built_midpoints():
    # bf16 neighbours around 1.0 are 1 and 1 + 2^-7; the midpoint 1 + 2^-8 ties to even (1.0)
    one = 0x3F80
    assert fo.f64_to_bf16_bits(np.array([1.0 + 2.0 ** -8]))[0] == one
    # next midpoint (between 1+2^-7 [odd] and 1+2^-6 [even]) ties up to the even one
    assert fo.f64_to_bf16_bits(np.array([1.0 + 3 * 2.0 ** -8]))[0] == one + 2
    # just below / above a midpoint
    assert fo.f64_to_bf16_bits(np.array([1.0 + 2.0 ** -8 - 2.0 ** -30]))[0] == one
    assert fo.f64_to_bf16_bits(np.array([1.0 + 2.0 ** -8 + 2.0 ** -30]))[0] == one + 1
    # negative values mirror
    assert fo.f64_to_bf16_bits(np.array([-(1.0 + 2.0 ** -8)]))[0] == (0x8000 | one)
    assert fo.f64_to_bf16_bits(np.array([-(1.0 + 2.0 ** -8 + 2.0 ** -30)]))[0] == (0x8000 | (one + 1))


def test_no_double_rounding_from_fp64():
    # 1 + 2^-8 + 2^-40 lies above the midpoint, but a nearest rounding to fp32 first lands
    # exactly on the midpoint and a second nearest-even rounding would then go down.
    x = np.array([1.0 + 2.0 ** -8 + 2.0 ** -40, -(1.0 + 2.0 ** -8 + 2.0 ** -40),
                  1.0 + 3 * 2.0 ** -8 - 2.0 ** -40])
    got = fo.f64_to_bf16_bits(x)
    assert got[0] == 0x3F81
    assert got[1] == 0xBF81
    assert got[2] == 0x3F81


def test_special_values():
    x = np.array([0.0, -0.0, np.inf, -np.inf, 1e300, -1e300, 3.3895313892515355e38])
    got = fo.f64_to_bf16_bits(x)
    assert list(got[:4]) == [0x0000, 0x8000, 0x7F80, 0xFF80]
    assert got[4] == 0x7F80 and got[5] == 0xFF80
    assert got[6] == 0x7F7F            # largest finite bf16 stays finite
    assert np.isnan(fo.bf16_bits_to_f64(fo.f64_to_bf16_bits(np.array([np.nan]))))[0]


def test_fp32_to_bf16_agrees_with_torch_library_conversion():
    # an independent implementation of the same published format conversion
    g = torch.Generator().manual_seed(7)
    x = torch.randn(200_000, generator=g) * torch.exp(torch.randn(200_000, generator=g) * 8)
    x[:8] = torch.tensor([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 65504.0, 1e-40, -1e-40])
    want = x.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got_from_bits = fo.f32_bits_to_bf16_bits(x.numpy().view(np.uint32))
    got_from_f64 = fo.f64_to_bf16_bits(x.numpy().astype(np.float64))
    assert np.array_equal(got_from_bits, want)
    assert np.array_equal(got_from_f64, want)


def test_round_to_f32_is_nearest_even():
    # fp32 neighbours of 1.0 are 1 and 1 + 2^-23; midpoint ties to 1.0
    assert fo.f64_to_f32(np.array([1.0 + 2.0 ** -24]))[0] == np.float32(1.0)
    assert fo.f64_to_f32(np.array([1.0 + 2.0 ** -24 + 2.0 ** -50]))[0] == np.float32(1.0 + 2.0 ** -23)
    assert fo.f64_to_f32(np.array([1.0 + 3 * 2.0 ** -24]))[0] == np.float32(1.0 + 2.0 ** -22)
