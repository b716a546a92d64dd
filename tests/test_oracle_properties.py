"""Property tests of the CPU oracle on drawn inputs (hypothesis): what must hold for ANY input,
beside the fixed pins of the other test_oracle_* files.  CPU only; nothing here touches the
product package."""
import os
import sys

import numpy as np
import pytest

hypothesis = pytest.importorskip("hypothesis")
from hypothesis import given, settings, strategies as st  # noqa: E402
from hypothesis.extra import numpy as hnp  # noqa: E402

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
from oracle import qvg_oracle as O  # noqa: E402

# the same drawn examples on every run (a failure must be reproducible, and a pass must stay one), nothing written to disk
SETTINGS = dict(max_examples=200, deadline=None, derandomize=True, database=None)


@settings(**SETTINGS)
@given(st.sampled_from([2, 4]), st.integers(1, 5), st.integers(1, 6), st.data())
def test_pack_then_unpack_returns_every_level(bits, n, groups, data):
    """The stored field is the level's two's complement: every level of the b-bit range comes
    back, whatever its neighbours in the byte are."""
    lo, hi = -(1 << (bits - 1)), (1 << (bits - 1)) - 1
    q = data.draw(hnp.arrays(np.int8, (n, 8 * groups), elements=st.integers(lo, hi)))
    packed = O.pack(q, bits)
    assert packed.shape == (n, 8 * groups * bits // 8)
    assert np.array_equal(O.unpack(packed, bits), q)
    # an element only touches its own field: flipping one level changes exactly one byte
    q2 = q.copy()
    q2[0, 3] = lo if q[0, 3] != lo else hi
    diff = np.flatnonzero(O.pack(q2, bits).ravel() != packed.ravel())
    assert diff.tolist() == [3 * bits // 8]


def _finite_f32(max_abs):
    m = float(np.float32(max_abs))
    return st.floats(-m, m, width=32, allow_nan=False, allow_infinity=False)


@settings(**SETTINGS)
@given(st.sampled_from([(2, 0), (4, 0), (2, 1), (4, 1)]), st.sampled_from([16, 32, 64, 128]), st.data())
def test_quant_round_bound_for_any_group(fmt, B, data):
    """Eq. 1-2 on arbitrary finite groups (zeros, denormal-scale magnitudes, mixed signs): levels
    stay in [-qmax, qmax]; the part removed is scale * level; what remains is at most half a
    step, plus what the rounding of the stored scale takes from the largest element (Eq. 3)."""
    bits, scale_fmt = fmt
    qmax = (1 << (bits - 1)) - 1
    top = 400.0 * qmax if scale_fmt == 1 else 6.0e4 * qmax            # below the scale format's saturation
    mag = data.draw(st.sampled_from([top, 1.0, 1e-3, 1e-6, 3e-8]))
    r = data.draw(hnp.arrays(np.float32, (3, 128), elements=_finite_f32(mag)))
    q, sc, after = O.quant_round(r, B, bits, scale_fmt)
    assert q.min() >= -qmax and q.max() <= qmax
    s = (O.e4m3_to_f32(sc.astype(np.uint8)) if scale_fmt == 1 else O.f16_to_f32(sc)).astype(np.float64)
    G = 128 // B
    rg = r.astype(np.float64).reshape(3, G, B)
    qg = q.astype(np.float64).reshape(3, G, B)
    ag = after.astype(np.float64).reshape(3, G, B)
    m = np.abs(rg).max(axis=2)
    for n in range(3):
        for g in range(G):
            if s[n, g] == 0.0:                                         # scale rounded to zero: nothing removed
                assert not q.reshape(3, G, B)[n, g].any()
                assert np.array_equal(ag[n, g], rg[n, g])
                continue
            # the removed part, up to the one rounding of the fma
            assert np.allclose(rg[n, g] - ag[n, g], s[n, g] * qg[n, g], rtol=0, atol=2.0 ** -22 * max(m[n, g], s[n, g]))
            bound = s[n, g] / 2 + qmax * abs(m[n, g] / qmax - s[n, g])
            assert np.abs(ag[n, g]).max() <= bound * (1 + 1e-6) + 1e-45


@settings(max_examples=60, deadline=None, derandomize=True, database=None)
@given(st.sampled_from([(1, 2, 2, 0, 64), (1, 3, 2, 0, 32), (2, 1, 4, 1, 16), (1, 1, 2, 1, 64)]),
       st.integers(1, 40), st.integers(1, 9), st.integers(0, 2), st.integers(0, 2 ** 31 - 1))
def test_decode_plus_what_remained_is_the_input(form, N, K, iters, seed):
    """Sec. 4.2 / Eq. 7: whatever the chunk, the stage and round counts and the start centroids,
    the decoder's fp32 sum plus the residual the encoder was left with is the input, up to the
    fp32 roundings of the two chains (and the bf16 rounding of a residual handed to a further
    smoothing stage); ids are valid rows and codes unpack to levels in range."""
    S, T, bits, scale_fmt, B = form
    rng = np.random.default_rng(seed)
    x32 = (rng.standard_normal((N, 128)) * rng.choice([0.01, 1.0, 30.0])).astype(np.float32)
    x = O.f32_to_bf16(x32)
    init_idx = rng.integers(0, N, K).astype(np.int32)
    e = O.encode_unit(x, K, B, S, T, iters, init_idx=init_idx, bits=bits, want_resid=True, scale_fmt=scale_fmt)
    ids = e["ids"].astype(np.int64)
    assert ids.min() >= 0 and ids.max() < K
    qmax = (1 << (bits - 1)) - 1
    lv = O.unpack(e["codes"], bits)
    assert lv.min() >= -qmax and lv.max() <= qmax
    out, f32 = O.decode_unit(e["cent"], e["ids"], e["codes"], e["scales"], B, bits, want_f32=True, scale_fmt=scale_fmt)
    xin = O.bf16_to_f32(x).astype(np.float64)
    # magnitude that passes through the fp32 additions of either chain
    size = np.abs(xin).max() + np.abs(O.bf16_to_f32(e["cent"]).astype(np.float64)).max() * S
    # a residual that feeds another smoothing stage travels as bf16: half a unit of its last place per such stage
    tol = 2.0 ** -19 * size * (S + T) + (S - 1) * 2.0 ** -8 * size + 1e-30       # bf16: 8 significant bits
    assert np.abs(f32.astype(np.float64) + e["resid"].astype(np.float64) - xin).max() <= tol
    # the stored output is the fp32 sum rounded once to bf16
    assert np.array_equal(out, O.f32_to_bf16(f32))
