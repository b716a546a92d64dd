"""Pins for the oracle's number formats and bit packing: numpy float16 and torch
bfloat16 (independent library conversions) and a hand-written byte layout."""
import numpy as np
import torch

from oracle import qvg_oracle as O
from conftest import bf16_bits


def test_f16_to_f32_all_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float32)
    got = O.f16_to_f32(bits)
    ok = (got == want) | (np.isnan(got) & np.isnan(want))
    assert ok.all()


def test_f32_to_f16_rne_matches_numpy(rng):
    # normal range, subnormal range, ties, overflow edge
    x = np.concatenate([
        rng.standard_normal(20000).astype(np.float32) * 10.0,
        rng.standard_normal(5000).astype(np.float32) * 1e-5,
        rng.standard_normal(5000).astype(np.float32) * 1e-7,
        np.array([0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e9, 2.0**-24, 2.0**-25,
                  1.5 * 2.0**-24, 2.5 * 2.0**-24, 1.0 + 2.0**-11, 1.0 + 3 * 2.0**-11,
                  6.103515625e-05, 6.0975552e-05], dtype=np.float32),
    ])
    # every midpoint between consecutive positive finite f16 values (exact ties)
    h = np.arange(0, 0x7bff, dtype=np.uint16)
    lo = h.view(np.float16).astype(np.float64)
    hi = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    mid = ((lo + hi) / 2).astype(np.float32)          # exactly representable in fp32
    x = np.concatenate([x, mid[::7], -mid[::11]])
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    got = O.f32_to_f16(x)
    assert np.array_equal(got, want)


def test_bf16_conversions_match_torch(rng):
    x = np.concatenate([
        rng.standard_normal(20000).astype(np.float32) * 100.0,
        np.array([1.0 + 2.0**-8, 1.0 + 3 * 2.0**-8, 1.0 + 2.0**-9, -1.0 - 2.0**-8, 3.3895314e38,
                  0.0, -0.0, 1e-40], dtype=np.float32)])
    want = bf16_bits(torch.from_numpy(x).to(torch.bfloat16))
    assert np.array_equal(O.f32_to_bf16(x), want)
    back = torch.from_numpy(want.view(np.int16)).view(torch.bfloat16).float().numpy()
    assert np.array_equal(O.bf16_to_f32(want), back)


def test_pack_layout_by_hand():
    # element i of a token: byte i//4, bits 2*(i%4).. ; code = two's complement of q (-1 -> 0b11)
    q = np.array([[-1, 0, 1, 0, 1, 1, -1, -1]], dtype=np.int8)
    # codes 3,0,1,0 -> 0b00_01_00_11 = 0x13 ; codes 1,1,3,3 -> 0b11_11_01_01 = 0xf5
    assert O.pack(q, 2).tolist() == [[0x13, 0xF5]]
    # 4 bit: two's complement nibble, low nibble first
    q4 = np.array([[-7, 7, 0, 1]], dtype=np.int8)
    assert O.pack(q4, 4).tolist() == [[0x9 | (7 << 4), 0 | (1 << 4)]]


def test_pack_unpack_roundtrip(rng):
    q = rng.integers(-1, 2, size=(33, 128)).astype(np.int8)
    assert np.array_equal(O.unpack(O.pack(q, 2), 2), q)
    q4 = rng.integers(-7, 8, size=(5, 128)).astype(np.int8)
    assert np.array_equal(O.unpack(O.pack(q4, 4), 4), q4)
