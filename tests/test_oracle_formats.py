"""Pins for the oracle's number-format widening (CPU only)."""
import math
import struct

import numpy as np
import torch

from oracle import formats as F


def test_bf16_widening_matches_struct_packing():
    rng = np.random.default_rng(5)
    bits = rng.integers(0, 1 << 16, size=4096).astype(np.uint16)
    got = F.bf16_bits_to_f64(bits)
    for b, g in zip(bits[:512], got[:512]):
        want = struct.unpack("<f", struct.pack("<I", int(b) << 16))[0]
        assert (math.isnan(want) and math.isnan(g)) or want == g
    # hand values: 0x3F80 = 1.0, 0xC000 = -2.0, 0x3DCD ~ 0.1001 (bf16 of 0.1), 0x0080 = 2^-126
    assert F.bf16_bits_to_f64(np.array([0x3F80, 0xC000, 0x0080], np.uint16)).tolist() == [1.0, -2.0, 2.0 ** -126]


def test_e4m3_hand_values():
    """Values fixed by the OCP E4M3 definition: bias 7, 3 mantissa bits,
    subnormals at exponent field 0, max finite 448, 0x7F/0xFF NaN, no infinity."""
    t = F.E4M3_TABLE
    assert t[0x00] == 0.0 and t[0x80] == 0.0 and math.copysign(1, t[0x80]) == -1
    assert t[0x01] == 2.0 ** -9            # smallest subnormal
    assert t[0x07] == 7 * 2.0 ** -9        # largest subnormal
    assert t[0x08] == 2.0 ** -6            # smallest normal
    assert t[0x38] == 1.0 and t[0x40] == 2.0 and t[0xC0] == -2.0
    assert t[0x3C] == 1.5 and t[0x39] == 1.125
    assert t[0x7E] == 448.0 and t[0xFE] == -448.0
    assert t[0x78] == 256.0                # exponent field 15 is still finite
    assert math.isnan(t[0x7F]) and math.isnan(t[0xFF])
    assert np.isfinite(np.delete(t, [0x7F, 0xFF])).all()
    # monotone on the positive half
    pos = t[:0x7F]
    assert (np.diff(pos) > 0).all()


def test_e4m3_all_codes_match_torch_cast():
    codes = torch.arange(256, dtype=torch.int32).to(torch.uint8)
    ref = codes.view(torch.float8_e4m3fn).to(torch.float64).numpy()
    got = F.e4m3_codes_to_f64(codes.numpy())
    assert np.array_equal(np.isnan(ref), np.isnan(got))
    ok = ~np.isnan(ref)
    assert np.array_equal(ref[ok], got[ok])


def test_e4m3_roundtrip_error_bound():
    """Nearest-value quantisation of normals has relative error <= 2^-4."""
    rng = np.random.default_rng(0)
    x = np.exp(rng.uniform(np.log(2.0 ** -6), np.log(448.0), size=4000)) * rng.choice([-1, 1], size=4000)
    q = torch.from_numpy(x.astype(np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    back = F.e4m3_codes_to_f64(q)
    assert (np.abs(back - x) <= 2.0 ** -4 * np.abs(x) + 1e-12).all()
