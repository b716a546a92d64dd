"""Helpers for the GPU parity tests: move seeded inputs to the device, run the oracle on the
same bytes, and compare with the rules the tolerances are stated in.

Cluster ids and 2-bit codes: bit-exact, except that at a documented distance tie - the two
candidates' fp64 squared distances differ by at most 1e-6 * (||x||^2 + ||c||^2) - either id
is accepted, and that token's codes are then checked against the oracle run with the GPU's id.
"""
import numpy as np
import torch

from oracle import qvg_oracle as O
from conftest import bf16_bits, bits_to_f32

TIE_REL = 1e-6


def to_np_u16(t):
    """cuda bf16 / f16 tensor -> numpy uint16 bit patterns."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def to_np_u8(t):
    return t.detach().cpu().contiguous().numpy()


def compare_ids(x_bits, cent_bits, ids_gpu, ids_ref):
    """Per unit arrays [N,d], [K,d], [N], [N].  Returns the indices of accepted ties; raises on
    any other mismatch."""
    bad = np.flatnonzero(ids_gpu != ids_ref)
    if bad.size == 0:
        return bad
    xf = bits_to_f32(x_bits[bad])
    dg = O.dist_to(xf, cent_bits, ids_gpu[bad])
    dr = O.dist_to(xf, cent_bits, ids_ref[bad])
    cf = bits_to_f32(cent_bits).astype(np.float64)
    mag = (xf.astype(np.float64) ** 2).sum(1) + np.maximum((cf[ids_gpu[bad]] ** 2).sum(1),
                                                          (cf[ids_ref[bad]] ** 2).sum(1))
    ok = np.abs(dg - dr) <= TIE_REL * mag
    assert ok.all(), (f"{(~ok).sum()} ids differ beyond a tie; first: token {bad[~ok][0]} "
                      f"gpu {ids_gpu[bad[~ok][0]]} ref {ids_ref[bad[~ok][0]]} "
                      f"d_gpu {dg[~ok][0]} d_ref {dr[~ok][0]}")
    return bad


def check_encoded_unit(x_bits, cent_bits, gpu, B, T, ref=None):
    """gpu: dict(ids [N], codes [N,T,32], scales [N,T,G]) of one unit.  Compares with the oracle's
    encode against the SAME centroids.  Returns the number of accepted ties."""
    if ref is None:
        ref = O.encode_given_centroids(x_bits, cent_bits, B, T)
    ties = compare_ids(x_bits, cent_bits, gpu["ids"], ref["ids"])
    same = np.ones(len(gpu["ids"]), bool)
    same[ties] = False
    assert np.array_equal(gpu["codes"][same], ref["codes"][same]), "codes differ"
    assert np.array_equal(gpu["scales"][same], ref["scales"][same]), "scales differ"
    if ties.size:
        alt = O.encode_given_ids(x_bits[ties], cent_bits, gpu["ids"][ties], B, T)
        assert np.array_equal(gpu["codes"][ties], alt["codes"])
        assert np.array_equal(gpu["scales"][ties], alt["scales"])
    c = gpu["codes"]
    assert (((c & 0xAA) >> 1) & (~c & 0x55)).max() == 0, "a 2-bit field holds the unused code 0b10"
    return int(ties.size)


def gpu_unit(enc, h, lo=0, hi=None):
    """Slice unit h (tokens lo:hi) of a binding.Encoded into numpy arrays."""
    hi = enc.ids.shape[1] if hi is None else hi
    return dict(ids=to_np_u8(enc.ids[h, lo:hi]), codes=to_np_u8(enc.codes[h, lo:hi]),
                scales=to_np_u16(enc.scales[h, lo:hi]))


def attn_tolerance_ok(out_gpu_bits, ref_f64):
    """|o_gpu - o_ref| <= 2e-3 + 2^-8 |o_ref|: 2e-3 absolute as stated for the path, plus the bf16
    output rounding (half an ulp = 2^-9 relative) and the bf16 rounding of the probabilities."""
    got = bits_to_f32(out_gpu_bits).astype(np.float64)
    err = np.abs(got - ref_f64)
    tol = 2e-3 + 2.0 ** -8 * np.abs(ref_f64)
    return bool((err <= tol).all()), float(err.max()), float((err / tol).max())


def attn_tolerance_wide_range_ok(out_gpu_bits, ref_f64, q_bits, k_bits, v_bits, scale=None):
    """For values far from unit scale (outlier channels): the probabilities enter the PV contraction
    as f16 rounded toward zero, i.e. each weight is off by up to 2^-10 of itself, which moves an
    output by at most 2^-10 * sum_j p_j |v_j| however much the terms cancel.  Tolerance:
    2e-3 + 2^-8 |o| + 2^-10 * E_p|v| (the last term computed here in fp64)."""
    q = bits_to_f32(q_bits).astype(np.float64); k = bits_to_f32(k_bits).astype(np.float64)
    v = bits_to_f32(v_bits).astype(np.float64)
    s = (q @ k.T) * (1.0 / np.sqrt(q.shape[1]) if scale is None else scale)
    p = np.exp(s - s.max(1, keepdims=True)); p /= p.sum(1, keepdims=True)
    spread = p @ np.abs(v)
    got = bits_to_f32(out_gpu_bits).astype(np.float64)
    err = np.abs(got - ref_f64)
    tol = 2e-3 + 2.0 ** -8 * np.abs(ref_f64) + 2.0 ** -10 * spread
    return bool((err <= tol).all()), float(err.max()), float((err / tol).max())
