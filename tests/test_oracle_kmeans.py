"""Pins for the oracle's k-means (Sec. 4.1): brute force, the member mean, library
Lloyd implementations, and the special cases K = 1 and K >= N."""
import numpy as np
import pytest

from oracle import qvg_oracle as O
from conftest import bits_to_f32, f32_to_bf16_bits_torch


def _brute_assign(r, c):
    # all pairwise squared distances at once, fp64, numpy argmin = first minimum
    d2 = ((r[:, None, :].astype(np.float64) - c[None, :, :].astype(np.float64)) ** 2).sum(-1)
    return d2.argmin(1).astype(np.uint8), d2


@pytest.mark.parametrize("N,K,d", [(64, 8, 16), (50, 3, 128), (7, 5, 4), (1, 1, 8)])
def test_assign_matches_brute_force(rng, N, K, d):
    r = rng.standard_normal((N, d)).astype(np.float32)
    cb = f32_to_bf16_bits_torch(rng.standard_normal((K, d)))
    ids, bd = O.assign(r, cb, want_dist=True)
    want, d2 = _brute_assign(r, bits_to_f32(cb))
    assert np.array_equal(ids, want)
    assert np.allclose(bd, d2.min(1), rtol=1e-13, atol=0)


def test_assign_ties_go_to_lowest_index():
    # token at the origin, centroids at +-1 on different axes: all equidistant
    r = np.zeros((3, 4), np.float32)
    r[1, 0] = 0.5          # nearer to centroid 2 (the only one with +1 on axis 0)
    c = np.array([[0, 1, 0, 0], [0, -1, 0, 0], [1, 0, 0, 0], [0, 0, 0, 1]], np.float32)
    cb = f32_to_bf16_bits_torch(c)
    assert O.assign(r, cb).tolist() == [0, 2, 0]
    # duplicate centroids: lowest copy wins
    cb2 = f32_to_bf16_bits_torch(np.array([[5, 5, 5, 5], [1, 0, 0, 0], [1, 0, 0, 0]], np.float32))
    assert O.assign(r, cb2).tolist() == [1, 1, 1]


def test_assign_detects_transposed_or_shifted_centroid_index(rng):
    # guards against an off-by-one in the centroid row: the token IS centroid j
    K, d = 9, 32
    c = rng.standard_normal((K, d)).astype(np.float32)
    cb = f32_to_bf16_bits_torch(c)
    r = bits_to_f32(cb)[::-1].copy()               # token n equals centroid K-1-n
    assert O.assign(r, cb).tolist() == list(range(K - 1, -1, -1))


def test_update_is_member_mean_and_empty_keeps_previous(rng):
    N, K, d = 200, 6, 16
    r = rng.standard_normal((N, d)).astype(np.float32)
    ids = rng.integers(0, K - 1, N).astype(np.uint8)          # cluster K-1 stays empty
    prev = f32_to_bf16_bits_torch(rng.standard_normal((K, d)))
    cent, cnt = O.update(r, ids, prev)
    for j in range(K - 1):
        mean = r[ids == j].astype(np.float64).mean(0)
        assert np.array_equal(cent[j], f32_to_bf16_bits_torch(mean.astype(np.float32)))
        assert cnt[j] == (ids == j).sum()
    assert cnt[K - 1] == 0 and np.array_equal(cent[K - 1], prev[K - 1])


def test_update_exact_rational_mean_small():
    # integers: the mean is an exact rational, compare with Python fractions
    from fractions import Fraction
    r = np.array([[1, 2], [2, 2], [4, -3], [9, 9]], np.float32)
    ids = np.array([0, 0, 0, 1], np.uint8)
    prev = np.zeros((2, 2), np.uint16)
    cent, cnt = O.update(r, ids, prev)
    want0 = [float(Fraction(1 + 2 + 4, 3)), float(Fraction(2 + 2 - 3, 3))]
    assert np.array_equal(cent[0], f32_to_bf16_bits_torch(np.array(want0, np.float32)))
    assert bits_to_f32(cent[1]).tolist() == [9.0, 9.0]
    assert cnt.tolist() == [3, 1]


def test_k1_centroid_is_chunk_mean(rng):
    r = rng.standard_normal((100, 8)).astype(np.float32)
    init = f32_to_bf16_bits_torch(np.zeros((1, 8)))
    cent, ids, inertia = O.lloyd(r, init, 1)
    assert (ids == 0).all()
    assert np.array_equal(cent[0], f32_to_bf16_bits_torch(r.astype(np.float64).mean(0).astype(np.float32)))


def test_k_ge_n_tokens_as_centroids_gives_zero_residual(rng):
    N, d = 12, 16
    xb = f32_to_bf16_bits_torch(rng.standard_normal((N, d)))
    r = bits_to_f32(xb)
    init = np.concatenate([xb, xb[:4]])            # K = 16 >= N, duplicates at the end
    cent, ids, inertia = O.lloyd(r, init, 2)
    assert ids.tolist() == list(range(N))
    assert inertia[-1] == 0.0
    assert (O.residual(r, cent, ids) == 0).all()


def _separated(rng, N, K, d, spread=8.0, sigma=0.3):
    centres = rng.standard_normal((K, d)) * spread
    lab = rng.integers(0, K, N)
    return (centres[lab] + sigma * rng.standard_normal((N, d))).astype(np.float32), lab


def test_lloyd_inertia_non_increasing(rng):
    r, _ = _separated(rng, 600, 12, 32, spread=1.0, sigma=0.7)    # overlapping: many moves
    init = f32_to_bf16_bits_torch(r[rng.permutation(600)[:12]])
    _, _, inertia = O.lloyd(r, init, 8)
    # centroids are rounded to bf16 after every update: allow 1e-4 relative slack
    assert (inertia[1:] <= inertia[:-1] * (1 + 1e-4)).all()
    assert inertia[-1] < inertia[0]


def test_lloyd_matches_scipy_kmeans2(rng):
    from scipy.cluster.vq import kmeans2
    N, K, d, I = 500, 6, 16, 4
    r, lab = _separated(rng, N, K, d, spread=2.0, sigma=1.0)   # overlapping: ids keep moving
    r = bits_to_f32(f32_to_bf16_bits_torch(r))           # data exactly representable
    first = [int(np.flatnonzero(lab == j)[0]) for j in range(K)]   # one start token per mode
    init_b = f32_to_bf16_bits_torch(r[first])
    cent, ids, _ = O.lloyd(r, init_b, I)
    # scipy: I x (assign, update); its labels are those of the last assign BEFORE the last
    # update, i.e. ours after I-1 iterations.
    c_sp, lab_sp = kmeans2(r.astype(np.float64), bits_to_f32(init_b).astype(np.float64),
                           iter=I, minit="matrix", missing="raise")
    _, ids_prev, _ = O.lloyd(r, init_b, I - 1)
    assert np.array_equal(ids_prev, lab_sp.astype(np.uint8))
    # centroids agree up to the bf16 rounding the oracle applies each iteration
    assert np.allclose(bits_to_f32(cent), c_sp, rtol=2.0**-7, atol=1e-3)


def test_lloyd_matches_sklearn(rng):
    from sklearn.cluster import KMeans
    N, K, d, I = 400, 5, 8, 3
    r, lab = _separated(rng, N, K, d, spread=2.0, sigma=1.0)
    r = bits_to_f32(f32_to_bf16_bits_torch(r))
    first = [int(np.flatnonzero(lab == j)[0]) for j in range(K)]
    init_b = f32_to_bf16_bits_torch(r[first])
    cent, ids, _ = O.lloyd(r, init_b, I)
    km = KMeans(n_clusters=K, init=bits_to_f32(init_b).astype(np.float64), n_init=1,
                algorithm="lloyd", max_iter=I, tol=0.0).fit(r.astype(np.float64))
    assert np.array_equal(ids, km.predict(r.astype(np.float64)).astype(np.uint8)) or \
        np.array_equal(ids, km.labels_.astype(np.uint8))
    assert np.allclose(bits_to_f32(cent), km.cluster_centers_, rtol=2.0**-7, atol=1e-3)


def test_residual_is_token_minus_assigned_centroid(rng):
    r = rng.standard_normal((40, 8)).astype(np.float32)
    cb = f32_to_bf16_bits_torch(rng.standard_normal((5, 8)))
    ids = rng.integers(0, 5, 40).astype(np.uint8)
    want = r - bits_to_f32(cb)[ids]
    assert np.array_equal(O.residual(r, cb, ids), want)
