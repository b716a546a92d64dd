"""ctypes access to the CPU oracle (oracle/qvg_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
the cpu_baseline leg of bench.py.  Nothing in the product package imports it,
and it imports nothing from the product package.

Arrays are numpy: bf16 and binary16 values travel as uint16 bit patterns.
Each function names the paper passage its C counterpart follows.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qvg_oracle.c")
_LIB = os.path.join(_HERE, "libqvg_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fused multiply-add, no fast-math)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC",
               "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.qvgo_bf16_to_f32.restype = C.c_float
        _lib.qvgo_bf16_to_f32.argtypes = [C.c_uint16]
        _lib.qvgo_f32_to_bf16.restype = C.c_uint16
        _lib.qvgo_f32_to_bf16.argtypes = [C.c_float]
        _lib.qvgo_f16_to_f32.restype = C.c_float
        _lib.qvgo_f16_to_f32.argtypes = [C.c_uint16]
        _lib.qvgo_f32_to_f16.restype = C.c_uint16
        _lib.qvgo_f32_to_f16.argtypes = [C.c_float]
        _lib.qvgo_e4m3_to_f32.restype = C.c_float
        _lib.qvgo_e4m3_to_f32.argtypes = [C.c_uint8]
        _lib.qvgo_f32_to_e4m3.restype = C.c_uint8
        _lib.qvgo_f32_to_e4m3.argtypes = [C.c_float]
        _lib.qvgo_chunk_bytes.restype = C.c_double
        _lib.qvgo_chunk_bytes.argtypes = [C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                          C.c_int, C.c_double, C.c_double]
        _lib.qvgo_max_threads.restype = C.c_int
    return _lib


def _p(a, dtype):
    """Pointer to a C-contiguous numpy array of the given dtype (None -> NULL)."""
    if a is None:
        return None
    assert a.dtype == dtype and a.flags["C_CONTIGUOUS"], (a.dtype, dtype)
    return a.ctypes.data_as(C.c_void_p)


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def _stored_ids(ids, K):
    """ids as the stored format keeps them: one byte per id up to 256 centroids, two beyond."""
    return ids.astype(np.uint8) if K <= 256 else ids


# ---------------------------------------------------------------- formats
def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float32 (exact)."""
    return (bits.astype(np.uint32) << 16).view(np.float32)


def f32_to_bf16(x) -> np.ndarray:
    L = lib()
    x = _c(x, np.float32)
    out = np.empty(x.shape, np.uint16)
    xf, of = x.ravel(), out.ravel()
    for i in range(xf.size):
        of[i] = L.qvgo_f32_to_bf16(float(xf[i]))
    return out


def f16_to_f32(bits) -> np.ndarray:
    L = lib()
    bits = _c(bits, np.uint16)
    out = np.empty(bits.shape, np.float32)
    bf, of = bits.ravel(), out.ravel()
    for i in range(bf.size):
        of[i] = L.qvgo_f16_to_f32(int(bf[i]))
    return out


def f32_to_f16(x) -> np.ndarray:
    L = lib()
    x = _c(x, np.float32)
    out = np.empty(x.shape, np.uint16)
    xf, of = x.ravel(), out.ravel()
    for i in range(xf.size):
        of[i] = L.qvgo_f32_to_f16(float(xf[i]))
    return out


def e4m3_to_f32(codes) -> np.ndarray:
    """FP8 E4M3 codes (uint8) -> float32 (exact)."""
    L = lib()
    codes = _c(codes, np.uint8)
    out = np.empty(codes.shape, np.float32)
    cf, of = codes.ravel(), out.ravel()
    for i in range(cf.size):
        of[i] = L.qvgo_e4m3_to_f32(int(cf[i]))
    return out


def f32_to_e4m3(x) -> np.ndarray:
    """float32 -> FP8 E4M3 code, nearest even, saturating at 448."""
    L = lib()
    x = _c(x, np.float32)
    out = np.empty(x.shape, np.uint8)
    xf, of = x.ravel(), out.ravel()
    for i in range(xf.size):
        of[i] = L.qvgo_f32_to_e4m3(float(xf[i]))
    return out


SCALE_F16, SCALE_E4M3 = 0, 1


# ---------------------------------------------------------------- k-means (Sec. 4.1)
def assign(r, cent, want_dist=False):
    """Nearest-centroid assignment; r [N,d] float32, cent [K,d] bf16 bits."""
    r = _c(r, np.float32); cent = _c(cent, np.uint16)
    N, d = r.shape; K = cent.shape[0]
    ids = np.empty(N, np.uint16)
    bd = np.empty(N, np.float64) if want_dist else None
    lib().qvgo_assign(C.c_int64(N), d, K, _p(r, np.float32), _p(cent, np.uint16),
                      _p(ids, np.uint16), _p(bd, np.float64))
    ids = _stored_ids(ids, K)
    return (ids, bd) if want_dist else ids


def dist_to(r, cent, ids):
    """fp64 squared distance of every token to the centroid ids[n]."""
    r = _c(r, np.float32); cent = _c(cent, np.uint16); ids = _c(ids, np.uint16)
    N, d = r.shape
    out = np.empty(N, np.float64)
    lib().qvgo_dist_to(C.c_int64(N), d, _p(r, np.float32), _p(cent, np.uint16),
                       _p(ids, np.uint16), _p(out, np.float64))
    return out


def update(r, ids, cent_prev):
    """Centroid = mean of its members; empty groups keep cent_prev. -> (cent, counts)."""
    r = _c(r, np.float32); ids = _c(ids, np.uint16); cent_prev = _c(cent_prev, np.uint16)
    N, d = r.shape; K = cent_prev.shape[0]
    out = np.empty((K, d), np.uint16); cnt = np.empty(K, np.int32)
    lib().qvgo_update(C.c_int64(N), d, K, _p(r, np.float32), _p(ids, np.uint16),
                      _p(cent_prev, np.uint16), _p(out, np.uint16), _p(cnt, np.int32))
    return out, cnt


def lloyd(r, init, iters):
    """iters x (assign, update) + final assign. -> (cent, ids, inertia[iters+1])."""
    r = _c(r, np.float32); init = _c(init, np.uint16)
    N, d = r.shape; K = init.shape[0]
    cent = np.empty((K, d), np.uint16); ids = np.empty(N, np.uint16)
    inertia = np.empty(iters + 1, np.float64)
    lib().qvgo_lloyd(C.c_int64(N), d, K, iters, _p(r, np.float32), _p(init, np.uint16),
                     _p(cent, np.uint16), _p(ids, np.uint16), _p(inertia, np.float64))
    return cent, _stored_ids(ids, K), inertia


def residual(r, cent, ids):
    """Eq. 5."""
    r = _c(r, np.float32); cent = _c(cent, np.uint16); ids = _c(ids, np.uint16)
    N, d = r.shape
    out = np.empty((N, d), np.float32)
    lib().qvgo_residual(C.c_int64(N), d, _p(r, np.float32), _p(cent, np.uint16),
                        _p(ids, np.uint16), _p(out, np.float32))
    return out


# ---------------------------------------------------------------- quantization (Eq. 1-2)
def quant_round(r, B, bits=2, scale_fmt=0):
    """One round of group quantization. -> (q int8 [N,d], scales [N,d/B] uint16: f16 bits, or the
    E4M3 code when scale_fmt == SCALE_E4M3; r_after)."""
    r = np.array(r, dtype=np.float32, order="C", copy=True)
    N, d = r.shape
    q = np.empty((N, d), np.int8); sc = np.empty((N, d // B), np.uint16)
    lib().qvgo_quant_round(C.c_int64(N), d, B, bits, scale_fmt, _p(r, np.float32), _p(q, np.int8),
                           _p(sc, np.uint16))
    return q, sc, r


def pack(q, bits=2):
    q = _c(q, np.int8)
    out = np.empty(q.size * bits // 8, np.uint8)
    lib().qvgo_pack(C.c_int64(q.size), bits, _p(q, np.int8), _p(out, np.uint8))
    return out.reshape(q.shape[:-1] + (q.shape[-1] * bits // 8,))


def unpack(packed, bits=2):
    packed = _c(packed, np.uint8)
    n = packed.size * 8 // bits
    q = np.empty(n, np.int8)
    lib().qvgo_unpack(C.c_int64(n), bits, _p(packed, np.uint8), _p(q, np.int8))
    return q.reshape(packed.shape[:-1] + (packed.shape[-1] * 8 // bits,))


# ---------------------------------------------------------------- encode / decode (Sec. 4.2)
def encode_unit(x, K, B, S, T, iters, init=None, init_idx=None, bits=2, want_resid=False, scale_fmt=0):
    """Encode one chunk of one head.  x [N,d] bf16 bits.
    init [S,K,d] bf16 bits, or init_idx [K] token indices (see the C comment).
    -> dict(cent [S,K,d], ids [S,N], codes [N,T,d*bits/8], scales [N,T,d/B], resid?)"""
    x = _c(x, np.uint16)
    N, d = x.shape
    if init is not None:
        init = _c(init, np.uint16).reshape(S, K, d)
    else:
        init_idx = _c(init_idx, np.int32)
        assert init_idx.shape == (K,)
    cent = np.empty((S, K, d), np.uint16); ids = np.empty((S, N), np.uint16)
    codes = np.empty((N, T, d * bits // 8), np.uint8); sc = np.empty((N, T, d // B), np.uint16)
    resid = np.empty((N, d), np.float32) if want_resid else None
    lib().qvgo_encode_unit(C.c_int64(N), d, K, B, S, T, bits, scale_fmt, iters, _p(x, np.uint16),
                           _p(init, np.uint16), _p(init_idx, np.int32), _p(cent, np.uint16),
                           _p(ids, np.uint16), _p(codes, np.uint8), _p(sc, np.uint16),
                           _p(resid, np.float32))
    out = dict(cent=cent, ids=_stored_ids(ids, K), codes=codes, scales=sc)
    if want_resid:
        out["resid"] = resid
    return out


def encode_given_centroids(x, cent, B, T, bits=2, scale_fmt=0):
    x = _c(x, np.uint16); cent = _c(cent, np.uint16)
    N, d = x.shape; K = cent.shape[0]
    ids = np.empty(N, np.uint16)
    codes = np.empty((N, T, d * bits // 8), np.uint8); sc = np.empty((N, T, d // B), np.uint16)
    lib().qvgo_encode_given_centroids(C.c_int64(N), d, K, B, T, bits, scale_fmt, _p(x, np.uint16),
                                      _p(cent, np.uint16), _p(ids, np.uint16),
                                      _p(codes, np.uint8), _p(sc, np.uint16))
    return dict(ids=_stored_ids(ids, K), codes=codes, scales=sc)


def encode_given_ids(x, cent, ids, B, T, bits=2, scale_fmt=0):
    x = _c(x, np.uint16); cent = _c(cent, np.uint16); ids = _c(ids, np.uint16)
    N, d = x.shape
    codes = np.empty((N, T, d * bits // 8), np.uint8); sc = np.empty((N, T, d // B), np.uint16)
    lib().qvgo_encode_given_ids(C.c_int64(N), d, B, T, bits, scale_fmt, _p(x, np.uint16),
                                _p(cent, np.uint16), _p(ids, np.uint16),
                                _p(codes, np.uint8), _p(sc, np.uint16))
    return dict(codes=codes, scales=sc)


def decode_unit(cent, ids, codes, scales, B, bits=2, want_f32=False, scale_fmt=0):
    """Eq. 7 replay.  cent [S,K,d] (or [K,d]), ids [S,N] (or [N]). -> bf16 bits [N,d]."""
    cent = _c(cent, np.uint16); ids = _c(ids, np.uint16)
    codes = _c(codes, np.uint8); scales = _c(scales, np.uint16)
    if cent.ndim == 2:
        cent = cent[None]
    if ids.ndim == 1:
        ids = ids[None]
    S, K, d = cent.shape
    N, T = codes.shape[0], codes.shape[1]
    assert ids.shape == (S, N) and scales.shape[:2] == (N, T), (cent.shape, ids.shape, codes.shape, scales.shape)
    out = np.empty((N, d), np.uint16)
    f32 = np.empty((N, d), np.float32) if want_f32 else None
    lib().qvgo_decode_unit(C.c_int64(N), d, K, B, S, T, bits, scale_fmt, _p(cent, np.uint16),
                           _p(ids, np.uint16), _p(codes, np.uint8), _p(scales, np.uint16),
                           _p(out, np.uint16), _p(f32, np.float32))
    return (out, f32) if want_f32 else out


def attention(q, k, v, scale=None, want_lse=False):
    """softmax(scale q k^T) v in fp64, one head.  q,k,v bf16 bits [*,d]. -> float64 [Nq,d]."""
    q = _c(q, np.uint16); k = _c(k, np.uint16); v = _c(v, np.uint16)
    Nq, d = q.shape; Nk = k.shape[0]
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    out = np.empty((Nq, d), np.float64)
    lse = np.empty(Nq, np.float64) if want_lse else None
    lib().qvgo_attention_batch(1, C.c_int64(Nq), C.c_int64(Nk), d, _p(q, np.uint16),
                               _p(k, np.uint16), _p(v, np.uint16), C.c_double(scale),
                               _p(out, np.float64), _p(lse, np.float64))
    return (out, lse) if want_lse else out


def rope_keys(k, rope):
    """Rotary embedding of decoded keys (pre-RoPE key caching, Sec. 5 "Implementation").
    k [N,d] bf16 bits, rope [N,d/2,2] binary16 bits (cos, sin). -> bf16 bits [N,d]."""
    k = _c(k, np.uint16); rope = _c(rope, np.uint16)
    N, d = k.shape
    assert rope.shape == (N, d // 2, 2)
    out = np.empty((N, d), np.uint16)
    lib().qvgo_rope_keys(C.c_int64(N), d, _p(k, np.uint16), _p(rope, np.uint16), _p(out, np.uint16))
    return out


def attn_merge(oa, lsea, ob, lseb):
    """Attention over the union of two disjoint key sets from the two partial results.
    oa, ob float64 [R,d]; lsea, lseb float64 [R]. -> (o [R,d], lse [R])."""
    oa = _c(oa, np.float64); ob = _c(ob, np.float64)
    lsea = _c(lsea, np.float64); lseb = _c(lseb, np.float64)
    R, d = oa.shape
    out = np.empty((R, d), np.float64); lse = np.empty(R, np.float64)
    lib().qvgo_attn_merge(C.c_int64(R), d, _p(oa, np.float64), _p(lsea, np.float64), _p(ob, np.float64),
                          _p(lseb, np.float64), _p(out, np.float64), _p(lse, np.float64))
    return out, lse


# ---------------------------------------------------------------- batched (H independent units)
def encode_batch(x, init, K, B, T, iters, S=1, bits=2, scale_fmt=0):
    """x [H,N,d] bf16 bits, init [H,S,K,d] (or [H,K,d] when S == 1)."""
    x = _c(x, np.uint16); init = _c(init, np.uint16)
    H, N, d = x.shape
    init = init.reshape(H, S, K, d)
    cent = np.empty((H, S, K, d), np.uint16); ids = np.empty((H, S, N), np.uint16)
    codes = np.empty((H, N, T, d * bits // 8), np.uint8); sc = np.empty((H, N, T, d // B), np.uint16)
    lib().qvgo_encode_batch(H, C.c_int64(N), d, K, B, S, T, bits, scale_fmt, iters, _p(x, np.uint16),
                            _p(init, np.uint16), _p(cent, np.uint16), _p(ids, np.uint16),
                            _p(codes, np.uint8), _p(sc, np.uint16))
    return dict(cent=cent, ids=_stored_ids(ids, K), codes=codes, scales=sc)


def decode_batch(cent, ids, codes, scales, B, bits=2, scale_fmt=0):
    cent = _c(cent, np.uint16); ids = _c(ids, np.uint16)
    codes = _c(codes, np.uint8); scales = _c(scales, np.uint16)
    H, S, K, d = cent.shape
    N, T = codes.shape[1], codes.shape[2]
    assert ids.shape == (H, S, N) and codes.shape[0] == H and scales.shape[:3] == (H, N, T), \
        (cent.shape, ids.shape, codes.shape, scales.shape)
    out = np.empty((H, N, d), np.uint16)
    lib().qvgo_decode_batch(H, C.c_int64(N), d, K, B, S, T, bits, scale_fmt, _p(cent, np.uint16),
                            _p(ids, np.uint16), _p(codes, np.uint8), _p(scales, np.uint16),
                            _p(out, np.uint16))
    return out


def attention_batch(q, k, v, scale=None, want_lse=False):
    q = _c(q, np.uint16); k = _c(k, np.uint16); v = _c(v, np.uint16)
    H, Nq, d = q.shape; Nk = k.shape[1]
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    out = np.empty((H, Nq, d), np.float64)
    lse = np.empty((H, Nq), np.float64) if want_lse else None
    lib().qvgo_attention_batch(H, C.c_int64(Nq), C.c_int64(Nk), d, _p(q, np.uint16),
                               _p(k, np.uint16), _p(v, np.uint16), C.c_double(scale),
                               _p(out, np.float64), _p(lse, np.float64))
    return (out, lse) if want_lse else out


def chunk_bytes(N, d, K, B, S, T, bits, scale_bytes, id_bits):
    """Stored size of one chunk of one head (Sec. 5, compression ratio)."""
    return float(lib().qvgo_chunk_bytes(C.c_int64(N), d, K, B, S, T, bits,
                                        C.c_double(scale_bytes), C.c_double(id_bits)))


def max_threads() -> int:
    return int(lib().qvgo_max_threads())
