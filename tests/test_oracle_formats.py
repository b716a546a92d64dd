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


# ---- FP8 E4M3 (the scale format of Sec. 5 "Implementation"), pinned to torch.float8_e4m3fn ----
def test_e4m3_decode_all_codes_matches_torch():
    codes = np.arange(256, dtype=np.uint8)
    want = torch.from_numpy(codes).view(torch.float8_e4m3fn).float().numpy()
    got = O.e4m3_to_f32(codes)
    assert ((got == want) | (np.isnan(got) & np.isnan(want))).all()
    # the layout's landmarks, by hand: smallest subnormal, smallest normal, one, largest finite
    assert got[0x01] == 2.0 ** -9 and got[0x08] == 2.0 ** -6 and got[0x38] == 1.0 and got[0x7E] == 448.0
    assert np.isnan(got[0x7F]) and got[0x80 | 0x38] == -1.0


def test_e4m3_encode_rne_matches_torch_in_range(rng):
    # random values over the whole range, every exact midpoint between neighbouring codes (ties)
    # and points just off the midpoints
    codes = np.arange(0, 0x7E, dtype=np.uint8)
    lo = O.e4m3_to_f32(codes).astype(np.float64)
    hi = O.e4m3_to_f32(codes + 1).astype(np.float64)
    mid = ((lo + hi) / 2).astype(np.float32)                       # exact in fp32
    x = np.concatenate([
        np.exp(rng.uniform(np.log(2.0 ** -11), np.log(448.0), 20000)).astype(np.float32),
        mid, np.nextafter(mid, np.float32(0)), np.nextafter(mid, np.float32(1e9)),
        lo.astype(np.float32), np.array([0.0, 448.0, 2.0 ** -10, 2.0 ** -11], np.float32)])
    x = x[x <= 448.0]
    want = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(O.f32_to_e4m3(x), want)
    assert np.array_equal(O.f32_to_e4m3(-x[x > 2.0 ** -10]), want[x > 2.0 ** -10] | 0x80)
    # ties go to the even code: 1.0625 lies between 1.0 (0x38) and 1.125 (0x39)
    assert O.f32_to_e4m3(np.array([1.0625, 1.1875], np.float32)).tolist() == [0x38, 0x3A]
    # half of the smallest subnormal is a tie with zero and goes to zero
    assert O.f32_to_e4m3(np.array([2.0 ** -10, np.nextafter(np.float32(2.0 ** -10), np.float32(1))],
                                  np.float32)).tolist() == [0, 1]


def test_e4m3_encode_saturates_beyond_448():
    x = np.array([448.0, 449.0, 464.0, 480.0, 1e6, 3e38], np.float32)
    assert (O.f32_to_e4m3(x) == 0x7E).all()
    assert (O.f32_to_e4m3(-x) == 0xFE).all()
