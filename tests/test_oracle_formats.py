"""Pins for the oracle's storage-format decoders and for the input packers, against an
independent library conversion (torch) and the format definitions."""
import os
import numpy as np
import torch

from oracle import formats
import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_bf16_decode_all_patterns_vs_torch():
    bits = np.arange(65536, dtype=np.uint16)
    ref = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float64).numpy()
    got = formats.decode_bf16(bits)
    fin = np.isfinite(ref)
    assert np.array_equal(got[fin], ref[fin])
    assert np.array_equal(np.isnan(got), np.isnan(ref))


def test_bf16_encode_rne_vs_torch():
    rng = np.random.default_rng(1)
    x = rng.standard_normal(200000).astype(np.float32) * np.float32(37.0)
    # add exact ties: value halfway between two bf16 neighbours
    base = (rng.integers(0x3F00, 0x4200, size=2000).astype(np.uint32) << 16) | np.uint32(0x8000)
    x = np.concatenate([x, base.view(np.float32)])
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(formats.encode_bf16_rne(x), ref)
    assert np.array_equal(synth.f32_to_bf16_bits(x), ref)


def test_e4m3_decode_all_codes_vs_torch():
    codes = np.arange(256, dtype=np.uint8)
    ref = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    got = formats.decode_e4m3(codes)
    fin = np.isfinite(ref)
    assert np.array_equal(got[fin], ref[fin])
    assert np.isnan(got[0x7F]) and np.isnan(got[0xFF]) and int(np.isnan(got).sum()) == 2


def test_e4m3_format_points():
    for line in open(os.path.join(GOLD, "e4m3_format_points.txt")):
        if line.startswith("#") or not line.strip():
            continue
        code, val = line.split()
        assert formats.decode_e4m3(np.array([int(code, 16)], dtype=np.uint8))[0] == float(val)
    assert np.nanmax(np.abs(formats.E4M3_TABLE)) == 448.0


def test_e4m3_quantizer_is_nearest_and_saturating():
    rng = np.random.default_rng(2)
    x = np.concatenate([rng.standard_normal(50000) * 100, rng.standard_normal(50000) * 0.01,
                        [0.0, 448.0, 1e9, -1e9, 2.0 ** -10, 3 * 2.0 ** -10]])
    codes = synth.quantize_e4m3(x, 1.0)
    val = formats.decode_e4m3(codes)
    assert np.all(np.isfinite(val))
    grid = np.sort(formats.E4M3_TABLE[np.isfinite(formats.E4M3_TABLE)])
    xc = np.clip(x, -448, 448)
    best = np.abs(xc[:, None] - grid[None, :]).min(axis=1)
    assert np.allclose(np.abs(val - xc), best, rtol=0, atol=1e-12)
    # ties go to the even mantissa: 2^-10 is halfway between 0 and 2^-9 -> 0 ; 3*2^-10 -> 2^-8
    assert val[-2] == 0.0 and val[-1] == 2.0 ** -8
    # per-column scales broadcast
    c2 = synth.quantize_e4m3(np.array([[1.0, 2.0]]), np.array([[0.5, 2.0]]))
    assert list(formats.decode_e4m3(c2)[0]) == [2.0, 1.0]
