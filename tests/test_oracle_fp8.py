"""Pins of the fp8 (E4M3) storage oracle: the format's landmark values, a library's conversion,
round-to-nearest-even by brute force against the list of representable values."""
import numpy as np
import torch

from oracle.fp8 import decode_e4m3, encode_e4m3, round_e4m3


def test_landmark_codes_of_the_format():
    assert decode_e4m3([0x00, 0x80]).tolist() == [0.0, -0.0]
    assert decode_e4m3([0x38])[0] == 1.0                       # exponent field 7 = bias
    assert decode_e4m3([0x01])[0] == 2.0 ** -9                 # smallest subnormal
    assert decode_e4m3([0x07])[0] == 7 * 2.0 ** -9             # largest subnormal
    assert decode_e4m3([0x08])[0] == 2.0 ** -6                 # smallest normal
    assert decode_e4m3([0x7E, 0xFE]).tolist() == [448.0, -448.0]
    assert np.isnan(decode_e4m3([0x7F, 0xFF])).all()
    assert decode_e4m3([0x78])[0] == 256.0                     # no infinities: exponent 15 is finite


def test_decode_matches_the_library_type_for_all_codes():
    codes = np.arange(256, dtype=np.uint8)
    lib = torch.from_numpy(codes).view(torch.float8_e4m3fn).double().numpy()
    ours = decode_e4m3(codes)
    assert np.array_equal(np.isnan(lib), np.isnan(ours))
    ok = ~np.isnan(lib)
    assert np.array_equal(lib[ok], ours[ok]) and np.array_equal(np.signbit(lib[ok]), np.signbit(ours[ok]))


def test_every_code_round_trips():
    codes = np.arange(256, dtype=np.uint8)
    vals = decode_e4m3(codes)
    back = encode_e4m3(vals)
    keep = ~np.isnan(vals)
    assert np.array_equal(back[keep], codes[keep])
    assert np.all(back[~keep] & 0x7F == 0x7F)


def test_rounding_is_nearest_even_by_brute_force():
    reps = np.sort(decode_e4m3(np.arange(0x7F, dtype=np.uint8)))          # non-negative finite values, ascending
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.uniform(0, 460, 4000), rng.uniform(0, 0.05, 2000), (reps[1:] + reps[:-1]) / 2, reps])
    got = round_e4m3(x)
    for xi, gi in zip(x, got):
        d = np.abs(reps - xi)
        best = d.min()
        cands = reps[d == best]
        if len(cands) == 1:
            assert gi == cands[0], xi
        else:                                                             # a tie: the even mantissa wins
            even = [c for c in cands if (int(encode_e4m3([c])[0]) & 1) == 0]
            assert gi == even[0], xi
    assert np.array_equal(round_e4m3(-x), -got)


def test_agrees_with_the_library_conversion_inside_the_range_and_saturates_outside():
    # every bf16 value of magnitude <= 448 (all that a bf16 cache row can hold there)
    bits = np.arange(1 << 16, dtype=np.uint32).astype(np.uint32) << 16
    vals = bits.view(np.float32)
    inside = np.isfinite(vals) & (np.abs(vals) <= 448.0)
    lib = torch.from_numpy(vals[inside].copy()).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    ours = encode_e4m3(vals[inside])
    assert np.array_equal(lib, ours)
    assert encode_e4m3([449.0, 1e9, np.inf, -470.0, -np.inf]).tolist() == [0x7E, 0x7E, 0x7E, 0xFE, 0xFE]
    assert encode_e4m3([np.nan])[0] & 0x7F == 0x7F
