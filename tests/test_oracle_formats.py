"""Pins for the oracle's storage-format decoders."""
import numpy as np
import torch

from oracle import bf16_bits_to_f64, e4m3_bytes_to_f64, E4M3_TABLE


def test_bf16_decode_matches_library_cast_for_every_pattern():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ours = bf16_bits_to_f64(bits)
    lib = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(np.isnan(ours), np.isnan(lib))
    ok = ~np.isnan(lib)
    assert np.array_equal(ours[ok], lib[ok])


def test_bf16_spot_values():
    # 0x3F80 = 1.0, 0xC000 = -2.0, 0x3DCD ~ 0.1 rounded to bf16 = 0.10009765625
    got = bf16_bits_to_f64(np.array([0x3F80, 0xC000, 0x3DCD, 0x0000], dtype=np.uint16))
    assert got.tolist() == [1.0, -2.0, 0.10009765625, 0.0]


def test_e4m3_table_matches_library_cast_for_every_byte():
    b = np.arange(256, dtype=np.uint8)
    lib = torch.from_numpy(b).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(np.isnan(E4M3_TABLE), np.isnan(lib))
    ok = ~np.isnan(lib)
    assert np.array_equal(E4M3_TABLE[ok], lib[ok])
    assert np.isnan(E4M3_TABLE[[0x7F, 0xFF]]).all() and np.isnan(E4M3_TABLE).sum() == 2


def test_e4m3_format_landmarks():
    # largest finite, one, smallest subnormal, smallest normal, negative zero
    assert E4M3_TABLE[0x7E] == 448.0
    assert E4M3_TABLE[0x38] == 1.0
    assert E4M3_TABLE[0x01] == 2.0 ** -9
    assert E4M3_TABLE[0x08] == 2.0 ** -6
    assert E4M3_TABLE[0x80] == 0.0 and np.signbit(E4M3_TABLE[0x80])
    assert E4M3_TABLE[0xFE] == -448.0
    assert e4m3_bytes_to_f64(np.array([[0x38, 0x40]], dtype=np.uint8)).tolist() == [[1.0, 2.0]]
