"""Pins for the oracle functions the GPU parity tests lean on most: the batched drivers (per-unit
offsets), the two shortened encoders the tie rule uses, and the distance the tie rule reads.

Each is checked against numpy written out here from the paper's formulas (Sec. 4.1 assignment,
Eq. 5 residual, Eq. 2 rounds with b = 2, Eq. 7 replay) on data that differs per unit, per stage
and per round, so that a wrong offset, a swapped argument or a skipped step changes the result.
"""
import numpy as np
import pytest

from oracle import qvg_oracle as O
from conftest import bits_to_f32, f32_to_bf16_bits_torch


@pytest.fixture
def rng(request):
    # a stream of this file's own, one per test, so that the other files' draws do not move
    import zlib
    return np.random.default_rng(zlib.crc32(request.node.name.encode()))


def _units(rng, H, N, d, spread=1.0):
    """H different bf16 tensors [N, d]: unit h is centred at 3 h so that no two units look alike."""
    x = rng.standard_normal((H, N, d)) * spread + 3.0 * np.arange(H)[:, None, None]
    return f32_to_bf16_bits_torch(x.astype(np.float32)).reshape(H, N, d)


def _np_argmin(xf, cf):
    d2 = ((xf[:, None, :].astype(np.float64) - cf[None].astype(np.float64)) ** 2).sum(-1)
    return d2.argmin(1), d2


def _np_rounds(r, B, T):
    """Eq. 2 with b = 2 on an fp32 residual [N, d], T times on what is left: levels [T, N, d] in
    {-1, 0, 1} and binary16 scale bits [T, N, d/B], in numpy float32 arithmetic."""
    N, d = r.shape
    r = r.astype(np.float32).copy()
    qs, ss = [], []
    for _ in range(T):
        g = r.reshape(N, d // B, B)
        m = np.abs(g).max(-1)
        s16 = np.minimum(m, np.float32(65504.0)).astype(np.float16)
        s = s16.astype(np.float32)
        with np.errstate(divide="ignore"):
            inv = np.where(s == 0, np.float32(0), np.float32(1.0) / s).astype(np.float32)
        u = (g * inv[..., None]).astype(np.float32)
        q = np.clip(np.rint(u), -1, 1).astype(np.float32)
        # r - s q with one rounding: s q is exact, and so is the fp64 difference of these operands
        g2 = (g.astype(np.float64) - s[..., None].astype(np.float64) * q).astype(np.float32)
        r = g2.reshape(N, d)
        qs.append(q.reshape(N, d).astype(np.int8)); ss.append(s16.view(np.uint16))
    return np.stack(qs), np.stack(ss)


def _np_pack2(q):
    """levels [..., d] in {-1, 0, 1} -> bytes [..., d/4]: element 4i+j in bits 2j..2j+1 of byte i,
    two's complement (Sec. 4.3 leaves the packing open; this is the documented format)."""
    f = (q.astype(np.int16) & 3).astype(np.uint8).reshape(q.shape[:-1] + (q.shape[-1] // 4, 4))
    return f[..., 0] | (f[..., 1] << 2) | (f[..., 2] << 4) | (f[..., 3] << 6)


def _np_encode_with_ids(x_bits, cent_bits, ids, B, T):
    xf, cf = bits_to_f32(x_bits), bits_to_f32(cent_bits)
    r = (xf - cf[ids]).astype(np.float32)                         # Eq. 5, one fp32 subtraction
    q, s = _np_rounds(r, B, T)
    codes = np.stack([_np_pack2(q[t]) for t in range(T)], axis=1)  # [N, T, d/4]
    return codes, np.stack([s[t] for t in range(T)], axis=1)       # [N, T, d/B]


# ------------------------------------------------------------------ dist_to
def test_dist_to_is_the_squared_distance_to_the_named_row(rng):
    N, K, d = 40, 11, 128
    xf = rng.standard_normal((N, d)).astype(np.float32)
    cb = f32_to_bf16_bits_torch(rng.standard_normal((K, d)) + np.arange(K)[:, None])
    ids = rng.permutation(np.arange(N) % K).astype(np.uint16)      # every row named, in shuffled order
    want = ((xf.astype(np.float64) - bits_to_f32(cb)[ids].astype(np.float64)) ** 2).sum(1)
    got = O.dist_to(xf, cb, ids)
    assert np.allclose(got, want, rtol=1e-13, atol=0)
    # a row off by one would be visible: the rows are a unit apart in every channel
    assert not np.allclose(got, O.dist_to(xf, cb, (ids + 1) % K), rtol=1e-3)


# ------------------------------------------------------------------ encode_given_ids
@pytest.mark.parametrize("B,T", [(64, 2), (32, 3), (16, 1), (128, 2)])
def test_encode_given_ids_follows_the_given_ids_not_the_nearest(rng, B, T):
    N, K, d = 48, 6, 128
    x = _units(rng, 1, N, d)[0]
    cb = f32_to_bf16_bits_torch(rng.standard_normal((K, d)))
    near, _ = _np_argmin(bits_to_f32(x), bits_to_f32(cb))
    ids = ((near + 1 + rng.integers(0, K - 1, N)) % K).astype(np.uint16)      # never the nearest row
    assert (ids != near).all()
    got = O.encode_given_ids(x, cb, ids, B, T)
    codes, scales = _np_encode_with_ids(x, cb, ids, B, T)
    assert np.array_equal(got["codes"], codes)
    assert np.array_equal(got["scales"], scales)
    # and it is not what the nearest rows would give
    assert not np.array_equal(got["codes"], _np_encode_with_ids(x, cb, near, B, T)[0])


# ------------------------------------------------------------------ encode_given_centroids
@pytest.mark.parametrize("B,T,K", [(64, 2, 16), (32, 3, 5)])
def test_encode_given_centroids_is_argmin_then_rounds(rng, B, T, K):
    N, d = 60, 128
    x = _units(rng, 1, N, d)[0]
    cb = f32_to_bf16_bits_torch(rng.standard_normal((K, d)))
    got = O.encode_given_centroids(x, cb, B, T)
    near, d2 = _np_argmin(bits_to_f32(x), bits_to_f32(cb))
    part = np.partition(d2, 1, axis=1)
    assert ((part[:, 1] - part[:, 0]) > 1e-9).all()               # no near ties in this draw
    assert np.array_equal(got["ids"], near.astype(np.uint8))
    codes, scales = _np_encode_with_ids(x, cb, near, B, T)
    assert np.array_equal(got["codes"], codes)
    assert np.array_equal(got["scales"], scales)
    # the centroids are kept: an encode_unit with no Lloyd iteration stores the same
    full = O.encode_unit(x, K, B, 1, T, 0, init=cb[None])
    assert np.array_equal(full["cent"][0], cb)
    assert np.array_equal(full["codes"], got["codes"]) and np.array_equal(full["ids"][0], got["ids"])


# ------------------------------------------------------------------ encode_batch / decode_batch
@pytest.mark.parametrize("S,T,B,I", [(1, 2, 64, 0), (1, 3, 32, 2), (2, 1, 16, 1), (2, 2, 64, 0)])
def test_encode_batch_is_encode_unit_per_unit(rng, S, T, B, I):
    H, N, K, d = 3, 37, 4, 128
    x = _units(rng, H, N, d)
    init = np.stack([np.stack([x[h, rng.permutation(N)[:K]] for _ in range(S)]) for h in range(H)])
    if S > 1:                                     # later stages cluster residuals: start them small
        init[:, 1:] = f32_to_bf16_bits_torch(0.3 * rng.standard_normal((H, S - 1, K, d))).reshape(H, S - 1, K, d)
    got = O.encode_batch(x, init, K, B, T, I, S=S)
    for h in range(H):
        one = O.encode_unit(x[h], K, B, S, T, I, init=init[h])
        for key in ("cent", "ids", "codes", "scales"):
            assert np.array_equal(got[key][h], one[key]), (h, key)
    # units differ, so an offset that lands in another unit cannot go unnoticed
    assert not np.array_equal(got["codes"][0], got["codes"][1])
    assert not np.array_equal(got["cent"][1], got["cent"][2])


def test_encode_batch_single_pass_against_numpy(rng):
    # no Lloyd iteration, one smoothing stage: every stored array of every unit from numpy alone
    H, N, K, d, B, T = 4, 29, 7, 128, 32, 2
    x = _units(rng, H, N, d)
    init = np.stack([x[h, rng.permutation(N)[:K]] for h in range(H)])
    got = O.encode_batch(x, init, K, B, T, 0)
    for h in range(H):
        near, d2 = _np_argmin(bits_to_f32(x[h]), bits_to_f32(init[h]))
        part = np.partition(d2, 1, axis=1)
        sure = (part[:, 1] - part[:, 0]) > 1e-9
        assert np.array_equal(got["ids"][h, 0][sure], near[sure].astype(np.uint8))
        codes, scales = _np_encode_with_ids(x[h], init[h], got["ids"][h, 0].astype(np.int64), B, T)
        assert np.array_equal(got["codes"][h], codes), h
        assert np.array_equal(got["scales"][h], scales), h
        assert np.array_equal(got["cent"][h, 0], init[h])


def _np_decode(cent_bits, ids, codes, scale_bits, B):
    """Eq. 7 in numpy: centroid rows in stage order (fp32 adds), then scale * level per round with
    one rounding each, then bf16.  cent [S,K,d], ids [S,N], codes [N,T,d/4], scales [N,T,d/B]."""
    S = cent_bits.shape[0]
    N, T = codes.shape[:2]
    acc = bits_to_f32(cent_bits[0])[ids[0]].astype(np.float32)
    for s in range(1, S):
        acc = (acc + bits_to_f32(cent_bits[s])[ids[s]]).astype(np.float32)
    for t in range(T):
        f = np.stack([(codes[:, t] >> (2 * j)) & 3 for j in range(4)], axis=-1).reshape(N, -1).astype(np.int16)
        q = np.where(f >= 2, f - 4, f).astype(np.float64)
        s = np.repeat(scale_bits[:, t].view(np.float16).astype(np.float64), B, axis=1)
        acc = (acc.astype(np.float64) + s * q).astype(np.float32)       # s q exact, one rounding
    return f32_to_bf16_bits_torch(acc)


@pytest.mark.parametrize("S,T,B", [(1, 2, 64), (2, 3, 32), (3, 1, 16)])
def test_decode_batch_is_eq7_per_unit(rng, S, T, B):
    H, N, K, d = 3, 23, 5, 128
    # storage that no encoder made, different in every unit, stage and round
    cent = f32_to_bf16_bits_torch(rng.standard_normal((H, S, K, d)) + np.arange(H)[:, None, None, None]).reshape(H, S, K, d)
    ids = rng.integers(0, K, (H, S, N)).astype(np.uint8)
    f = rng.integers(0, 3, (H, N, T, d)).astype(np.uint8)
    f = np.where(f == 2, 3, f).astype(np.uint8).reshape(H, N, T, d // 4, 4)           # fields 00, 01, 11
    codes = (f[..., 0] | (f[..., 1] << 2) | (f[..., 2] << 4) | (f[..., 3] << 6)).astype(np.uint8)
    scales = np.abs(rng.standard_normal((H, N, T, d // B)) * (1 + np.arange(T))[None, None, :, None]
                    ).astype(np.float16).view(np.uint16)
    got = O.decode_batch(cent, ids, codes, scales, B)
    for h in range(H):
        assert np.array_equal(got[h], O.decode_unit(cent[h], ids[h], codes[h], scales[h], B)), h
        assert np.array_equal(got[h], _np_decode(cent[h], ids[h].astype(np.int64), codes[h], scales[h], B)), h
    assert not np.array_equal(got[0], got[1])
