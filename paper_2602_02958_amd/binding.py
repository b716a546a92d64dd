"""Thin ctypes binding of libqvg.so (include/qvg.h): argument marshalling only.

Every step of the codec runs in the library's HIP kernels; this module converts torch
tensors to device pointers, allocates outputs and workspace with torch, passes torch's
current stream, and raises on a negative status.  It never falls back to a CPU path:
a missing library raises at the first call.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libqvg.so")
_lib = None

ENTRY_ENCODE, ENTRY_DECODE, ENTRY_ATTN, ENTRY_KMEANS_UPDATE, ENTRY_KMEANS_ASSIGN = 0, 1, 2, 3, 4
SCALE_F16, SCALE_E4M3 = 0, 1

EXPORTS = ["qvg_encode_chunk", "qvg_encode_chunk_static", "qvg_decode", "qvg_decode_ex", "qvg_attn_decode", "qvg_attn_decode_ex",
           "qvg_attn_decode_causal", "qvg_attn_decode_f32", "qvg_attn_merge",
           "qvg_kmeans_assign",
           "qvg_kmeans_update", "qvg_workspace_bytes", "qvg_compressed_bytes",
           "qvg_status_string", "qvg_version"]


class QvgParams(C.Structure):
    _fields_ = [("n_heads", C.c_int32), ("head_dim", C.c_int32), ("n_clusters", C.c_int32),
                ("group_size", C.c_int32), ("n_stages", C.c_int32), ("bits", C.c_int32),
                ("n_smooth_stages", C.c_int32), ("kmeans_iters", C.c_int32), ("scale_format", C.c_int32)]


class QvgError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def lib():
    """Load libqvg.so (built in-tree by paper_2602_02958_amd.build); raise if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2602_02958_amd.build` "
                "(there is no CPU fallback)")
        L = C.CDLL(_LIB_PATH)
        vp, i64, u8p = C.c_void_p, C.c_int64, C.c_void_p
        pp = C.POINTER(QvgParams)
        L.qvg_encode_chunk.restype = C.c_int
        L.qvg_encode_chunk.argtypes = [pp, i64, vp, i64, i64, vp, vp, i64, u8p, u8p, vp, i64, vp,
                                       C.c_size_t, vp]
        L.qvg_encode_chunk_static.restype = C.c_int
        L.qvg_encode_chunk_static.argtypes = [pp, i64, vp, i64, i64, vp, vp, i64, u8p, u8p, vp, i64, vp]
        L.qvg_decode.restype = C.c_int
        L.qvg_decode.argtypes = [pp, i64, i64, vp, u8p, u8p, vp, vp, i64, i64, vp]
        L.qvg_decode_ex.restype = C.c_int
        L.qvg_decode_ex.argtypes = [pp, i64, i64, i64, i64, vp, u8p, u8p, vp, vp, i64, i64, vp]
        L.qvg_attn_decode.restype = C.c_int
        L.qvg_attn_decode.argtypes = [pp, i64, vp, i64, i64, vp, u8p, u8p, vp, vp, u8p, u8p, vp,
                                      C.c_float, vp, vp, vp, C.c_size_t, vp]
        L.qvg_attn_decode_ex.restype = C.c_int
        L.qvg_attn_decode_ex.argtypes = [pp, i64, vp, i64, i64, i64, vp, u8p, u8p, vp, vp, u8p, u8p, vp, vp,
                                         C.c_float, vp, vp, vp, C.c_size_t, vp]
        L.qvg_attn_decode_causal.restype = C.c_int
        L.qvg_attn_decode_causal.argtypes = [pp, i64, vp, i64, i64, i64, vp, u8p, u8p, vp, vp, u8p, u8p, vp, vp, vp,
                                             C.c_float, vp, vp, vp, C.c_size_t, vp]
        L.qvg_attn_decode_f32.restype = C.c_int
        L.qvg_attn_decode_f32.argtypes = [pp, i64, vp, i64, i64, i64, vp, u8p, u8p, vp, vp, u8p, u8p, vp, vp, vp,
                                          C.c_float, vp, vp, vp]
        L.qvg_attn_merge.restype = C.c_int
        L.qvg_attn_merge.argtypes = [i64, C.c_int32, vp, vp, vp, vp, vp, vp, vp]
        L.qvg_kmeans_assign.restype = C.c_int
        L.qvg_kmeans_assign.argtypes = [pp, i64, vp, i64, i64, vp, u8p, vp, C.c_size_t, vp]
        L.qvg_kmeans_update.restype = C.c_int
        L.qvg_kmeans_update.argtypes = [pp, i64, vp, i64, i64, u8p, vp, vp, vp, vp, C.c_size_t, vp]
        L.qvg_workspace_bytes.restype = C.c_int
        L.qvg_workspace_bytes.argtypes = [pp, C.c_int, i64, i64, C.POINTER(C.c_size_t)]
        L.qvg_compressed_bytes.restype = C.c_int64
        L.qvg_compressed_bytes.argtypes = [pp, i64]
        L.qvg_status_string.restype = C.c_char_p
        L.qvg_status_string.argtypes = [C.c_int]
        L.qvg_version.restype = C.c_int
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().qvg_status_string(int(status)).decode()


def make_params(n_heads, n_clusters, group_size, n_stages, kmeans_iters=0, head_dim=128, bits=2,
                n_smooth_stages=1, scale_format=SCALE_F16) -> QvgParams:
    return QvgParams(n_heads, head_dim, n_clusters, group_size, n_stages, bits, n_smooth_stages,
                     kmeans_iters, scale_format)


def workspace_bytes(p: QvgParams, entry: int, n_tokens: int, n_q: int = 0) -> int:
    out = C.c_size_t(0)
    st = lib().qvg_workspace_bytes(C.byref(p), entry, n_tokens, n_q, C.byref(out))
    if st != 0:
        raise QvgError(st, "qvg_workspace_bytes")
    return int(out.value)


def compressed_bytes(p: QvgParams, n_tokens: int) -> int:
    v = int(lib().qvg_compressed_bytes(C.byref(p), n_tokens))
    if v < 0:
        raise QvgError(v, "qvg_compressed_bytes")
    return v


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else None


def _check(t, dtype, name):
    if t.dtype != dtype or not t.is_cuda:
        raise TypeError(f"{name}: expected a cuda tensor of {dtype}, got {t.dtype} on {t.device}")


def _view3(x, name):
    """[H, N, d] bf16 view with a contiguous last dim -> (stride_head, stride_token)."""
    _check(x, torch.bfloat16, name)
    if x.dim() != 3 or x.stride(2) != 1:
        raise ValueError(f"{name}: need [H, N, d] with unit stride along d")
    return x.stride(0), x.stride(1)


@dataclass
class Encoded:
    """Stored form of one chunk (or of a cache of chunks) for H units.  With n_smooth = S > 1
    smoothing stages the tables are [H, n_chunks, S, K, d] and a token has S ids: [H, N, S].
    The formats are read off the tensors: 4-bit levels have d/2 code bytes per round, FP8 E4M3
    scales are a uint8 tensor."""
    centroids: torch.Tensor   # [H, n_chunks, K, d] bf16
    ids: torch.Tensor         # [H, N] uint8 (int16 with more than 256 centroids)
    codes: torch.Tensor       # [H, N, T, d*bits/8] uint8
    scales: torch.Tensor      # [H, N, T, d/B] float16, or uint8 (E4M3)
    chunk_len: int
    n_smooth: int = 1

    @property
    def bits(self) -> int:
        return self.codes.shape[3] * 8 // self.centroids.shape[-1]

    @property
    def scale_format(self) -> int:
        return SCALE_E4M3 if self.scales.dtype == torch.uint8 else SCALE_F16


def id_dtype(n_clusters):
    """Cluster ids are bytes up to 256 centroids and 16-bit words beyond (int16 tensors here: the
    values stay below 512)."""
    return torch.uint8 if n_clusters <= 256 else torch.int16


def alloc_cache(n_heads, n_tokens, chunk_len, n_clusters, group_size, n_stages, head_dim=128,
                device="cuda", n_smooth=1, bits=2, scale_format=SCALE_F16) -> Encoded:
    """Uninitialised storage for a cache of n_tokens tokens per unit in chunks of chunk_len."""
    n_chunks = max(1, -(-n_tokens // chunk_len))
    S = n_smooth
    cshape = (n_heads, n_chunks, n_clusters, head_dim) if S == 1 else (n_heads, n_chunks, S, n_clusters, head_dim)
    ishape = (n_heads, n_tokens) if S == 1 else (n_heads, n_tokens, S)
    return Encoded(
        torch.empty(cshape, dtype=torch.bfloat16, device=device),
        torch.empty(ishape, dtype=id_dtype(n_clusters), device=device),
        torch.empty(n_heads, n_tokens, n_stages, head_dim * bits // 8, dtype=torch.uint8, device=device),
        torch.empty(n_heads, n_tokens, n_stages, head_dim // group_size,
                    dtype=torch.uint8 if scale_format == SCALE_E4M3 else torch.float16, device=device),
        chunk_len, S)


def encode_chunk(x, init_centroids, group_size, n_stages, kmeans_iters, cache: Encoded | None = None,
                 chunk_index: int = 0, workspace=None, bits=2, scale_format=SCALE_F16,
                 static_scratch: bool = False) -> Encoded:
    """qvg_encode_chunk.  x [H, N, d] bf16, init_centroids [H, K, d] bf16, or [H, S, K, d] for S
    smoothing stages.  Without `cache` a one-chunk cache is allocated and returned; with it, the
    chunk is written in place at chunk_index (tokens chunk_index*chunk_len ...), using the output
    strides; the cache's formats then apply (bits and scale_format describe a new cache).
    static_scratch: call qvg_encode_chunk_static instead (no workspace: the library's own static
    scratch array; with a `cache` given the call allocates nothing at all)."""
    sh, st_ = _view3(x, "x")
    H, N, d = x.shape
    _check(init_centroids, torch.bfloat16, "init_centroids")
    init_centroids = init_centroids.contiguous()
    K = init_centroids.shape[-2]
    S = init_centroids.shape[1] if init_centroids.dim() == 4 else 1
    if cache is None:
        cache = alloc_cache(H, N, max(N, 1), K, group_size, n_stages, d, x.device, n_smooth=S, bits=bits,
                            scale_format=scale_format)
    bits, scale_format = cache.bits, cache.scale_format
    n_total = cache.ids.shape[1]
    n_chunks = cache.centroids.shape[1]
    off = chunk_index * cache.chunk_len
    if not (0 <= chunk_index < n_chunks) or off + N > n_total or (N > cache.chunk_len):
        raise ValueError("chunk does not fit the cache")
    if cache.codes.shape[2] != n_stages or cache.scales.shape[3] != d // group_size or \
            cache.centroids.shape[-2] != K or cache.ids.shape[0] != H or cache.n_smooth != S or \
            cache.ids.dtype != id_dtype(K):
        raise ValueError("cache was allocated for other parameters")
    p = make_params(H, K, group_size, n_stages, kmeans_iters, head_dim=d, n_smooth_stages=S, bits=bits,
                    scale_format=scale_format)
    T, G = n_stages, d // group_size
    outs = (C.c_void_p(cache.centroids.data_ptr() + chunk_index * S * K * d * 2), n_chunks * S * K * d,
            C.c_void_p(cache.ids.data_ptr() + off * S * cache.ids.element_size()),
            C.c_void_p(cache.codes.data_ptr() + off * T * (d * bits // 8)),
            C.c_void_p(cache.scales.data_ptr() + off * T * G * cache.scales.element_size()), n_total)
    if static_scratch:
        st = lib().qvg_encode_chunk_static(C.byref(p), N, _ptr(x), sh, st_, _ptr(init_centroids), *outs, _stream())
        if st != 0:
            raise QvgError(st, "qvg_encode_chunk_static")
        return cache
    need = workspace_bytes(p, ENTRY_ENCODE, N)
    if need and (workspace is None or workspace.numel() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    st = lib().qvg_encode_chunk(C.byref(p), N, _ptr(x), sh, st_, _ptr(init_centroids), *outs,
                                _ptr(workspace) if need else None, need, _stream())
    if st != 0:
        raise QvgError(st, "qvg_encode_chunk")
    return cache


def decode(enc: Encoded, out=None, n_tokens=None, first_token=0) -> torch.Tensor:
    """qvg_decode_ex -> bf16 [H, n_tokens, d]: the whole cache, or n_tokens tokens starting at
    first_token (a multiple of the chunk length)."""
    H, cap = enc.ids.shape[:2]
    N = cap - first_token if n_tokens is None else int(n_tokens)
    if first_token < 0 or N < 0 or first_token + N > cap:
        raise ValueError("token range outside the cache")
    K, d = enc.centroids.shape[-2:]
    T, G = enc.codes.shape[2], enc.scales.shape[3]
    p = make_params(H, K, d // G, T, 0, head_dim=d, n_smooth_stages=enc.n_smooth, bits=enc.bits,
                    scale_format=enc.scale_format)
    if out is None:
        out = torch.empty(H, N, d, dtype=torch.bfloat16, device=enc.ids.device)
    sh, st_ = _view3(out, "out")
    for t, dt, nm in ((enc.centroids, torch.bfloat16, "centroids"), (enc.ids, id_dtype(K), "ids"),
                      (enc.codes, torch.uint8, "codes"), (enc.scales, enc.scales.dtype, "scales")):
        _check(t, dt, nm)
        if not t.is_contiguous():
            raise ValueError(f"{nm} must be contiguous")
    st = lib().qvg_decode_ex(C.byref(p), N, enc.chunk_len, cap, first_token, _ptr(enc.centroids), _ptr(enc.ids),
                             _ptr(enc.codes), _ptr(enc.scales), _ptr(out), sh, st_, _stream())
    if st != 0:
        raise QvgError(st, "qvg_decode_ex")
    return out


def attn_workspace(heads: int, n_q: int, chunk_len: int, n_chunks: int, device) -> torch.Tensor:
    """A workspace for attn_decode that holds the decoded tiles of n_chunks chunks (and the
    queries' running state, which is used when the cache has more chunks than that)."""
    p = make_params(heads, 2, 128, 1)
    padded = -(-chunk_len // 64) * 64 * n_chunks
    return torch.empty(workspace_bytes(p, ENTRY_ATTN, padded, n_q), dtype=torch.uint8, device=device)


def attn_decode(q, k: Encoded, v: Encoded, softmax_scale=None, want_lse=False, out=None, n_kv=None,
                k_rope=None, q_kv_len=None, f32_out=False, workspace=None):
    """qvg_attn_decode_ex.  q [H, Nq, d] bf16 contiguous -> out bf16 [H, Nq, d] (and lse fp32 [H, Nq]).
    n_kv: read only the first n_kv tokens of the caches (they are allocated for more);
    k_rope: [n_kv, d/2, 2] float16 (cos, sin), the rotary embedding of the decoded keys;
    q_kv_len: [Nq] int32, query i sees the first q_kv_len[i] tokens only (qvg_attn_decode_causal);
    f32_out: the result as float32, before the rounding to bf16 (qvg_attn_decode_f32);
    workspace: uint8 tensor (attn_workspace): every tile is then decoded once per unit into it and
    shared by all query blocks, a slab of chunks at a time, instead of once per 256 queries."""
    _check(q, torch.bfloat16, "q")
    q = q.contiguous()
    H, Nq, d = q.shape
    cap = k.ids.shape[1]
    Nk = cap if n_kv is None else int(n_kv)
    if not (1 <= Nk <= cap):
        raise ValueError("n_kv must lie in 1 .. the caches' token capacity")
    if k_rope is not None:
        _check(k_rope, torch.float16, "k_rope")
        if tuple(k_rope.shape) != (Nk, d // 2, 2) or not k_rope.is_contiguous():
            raise ValueError("k_rope: need a contiguous [n_kv, d/2, 2] float16 tensor")
    K = k.centroids.shape[-2]
    T, G = k.codes.shape[2], k.scales.shape[3]
    _check(k.ids, id_dtype(K), "k.ids")
    _check(v.ids, id_dtype(K), "v.ids")
    if (v.ids.shape, v.codes.shape, v.scales.shape, v.scales.dtype, v.centroids.shape, v.chunk_len, v.n_smooth) != \
            (k.ids.shape, k.codes.shape, k.scales.shape, k.scales.dtype, k.centroids.shape, k.chunk_len, k.n_smooth):
        raise ValueError("K and V caches must share shapes and parameters")
    p = make_params(H, K, d // G, T, 0, head_dim=d, n_smooth_stages=k.n_smooth, bits=k.bits,
                    scale_format=k.scale_format)
    if softmax_scale is None:
        softmax_scale = 1.0 / (d ** 0.5)
    if out is None:
        out = torch.empty(H, Nq, d, dtype=torch.float32 if f32_out else torch.bfloat16, device=q.device)
    lse = torch.empty(H, Nq, dtype=torch.float32, device=q.device) if want_lse else None
    if q_kv_len is not None:
        _check(q_kv_len, torch.int32, "q_kv_len")
        if tuple(q_kv_len.shape) != (Nq,) or not q_kv_len.is_contiguous():
            raise ValueError("q_kv_len: need a contiguous [n_q] int32 tensor")
    if f32_out:
        _check(out, torch.float32, "out")
        if not out.is_contiguous():
            raise ValueError("out must be contiguous")
        st = lib().qvg_attn_decode_f32(C.byref(p), Nq, _ptr(q), Nk, k.chunk_len, cap,
                                       _ptr(k.centroids), _ptr(k.ids), _ptr(k.codes), _ptr(k.scales),
                                       _ptr(v.centroids), _ptr(v.ids), _ptr(v.codes), _ptr(v.scales),
                                       _ptr(k_rope), _ptr(q_kv_len), C.c_float(softmax_scale), _ptr(out),
                                       _ptr(lse), _stream())
        if st != 0:
            raise QvgError(st, "qvg_attn_decode_f32")
        return (out, lse) if want_lse else out
    if q_kv_len is not None:
        st = lib().qvg_attn_decode_causal(C.byref(p), Nq, _ptr(q), Nk, k.chunk_len, cap,
                                          _ptr(k.centroids), _ptr(k.ids), _ptr(k.codes), _ptr(k.scales),
                                          _ptr(v.centroids), _ptr(v.ids), _ptr(v.codes), _ptr(v.scales),
                                          _ptr(k_rope), _ptr(q_kv_len), C.c_float(softmax_scale), _ptr(out),
                                          _ptr(lse), _ptr(workspace), 0 if workspace is None else workspace.numel(),
                                          _stream())
        if st != 0:
            raise QvgError(st, "qvg_attn_decode_causal")
        return (out, lse) if want_lse else out
    st = lib().qvg_attn_decode_ex(C.byref(p), Nq, _ptr(q), Nk, k.chunk_len, cap,
                                  _ptr(k.centroids), _ptr(k.ids), _ptr(k.codes), _ptr(k.scales),
                                  _ptr(v.centroids), _ptr(v.ids), _ptr(v.codes), _ptr(v.scales),
                                  _ptr(k_rope), C.c_float(softmax_scale), _ptr(out), _ptr(lse),
                                  _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream())
    if st != 0:
        raise QvgError(st, "qvg_attn_decode_ex")
    return (out, lse) if want_lse else out


def attn_merge(out_a, lse_a, out_b, lse_b, out=None, want_lse=False):
    """qvg_attn_merge.  out_* bf16 [..., d] contiguous, lse_* fp32 [...] -> merged bf16 (and lse)."""
    for t, dt, nm in ((out_a, torch.bfloat16, "out_a"), (out_b, torch.bfloat16, "out_b"),
                      (lse_a, torch.float32, "lse_a"), (lse_b, torch.float32, "lse_b")):
        _check(t, dt, nm)
        if not t.is_contiguous():
            raise ValueError(f"{nm} must be contiguous")
    d = out_a.shape[-1]
    rows = out_a.numel() // d
    if out_b.shape != out_a.shape or lse_a.numel() != rows or lse_b.numel() != rows:
        raise ValueError("shapes of the two partial results differ")
    if out is None:
        out = torch.empty_like(out_a)
    lse = torch.empty_like(lse_a) if want_lse else None
    st = lib().qvg_attn_merge(rows, d, _ptr(out_a), _ptr(lse_a), _ptr(out_b), _ptr(lse_b), _ptr(out), _ptr(lse),
                              _stream())
    if st != 0:
        raise QvgError(st, "qvg_attn_merge")
    return (out, lse) if want_lse else out


def kmeans_assign(x, centroids) -> torch.Tensor:
    """qvg_kmeans_assign -> ids [H, N], uint8 (int16 with more than 256 centroids)."""
    sh, st_ = _view3(x, "x")
    H, N, d = x.shape
    centroids = centroids.contiguous()
    p = make_params(H, centroids.shape[-2], 64, 1, 0, head_dim=d)
    ids = torch.empty(H, N, dtype=id_dtype(centroids.shape[-2]), device=x.device)
    need = workspace_bytes(p, ENTRY_KMEANS_ASSIGN, N)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=x.device)
    st = lib().qvg_kmeans_assign(C.byref(p), N, _ptr(x), sh, st_, _ptr(centroids), _ptr(ids), _ptr(ws), need,
                                 _stream())
    if st != 0:
        raise QvgError(st, "qvg_kmeans_assign")
    return ids


def kmeans_update(x, ids, centroids_prev):
    """qvg_kmeans_update -> (centroids bf16 [H, K, d], counts int32 [H, K])."""
    sh, st_ = _view3(x, "x")
    H, N, d = x.shape
    centroids_prev = centroids_prev.contiguous()
    K = centroids_prev.shape[-2]
    _check(ids, id_dtype(K), "ids")
    p = make_params(H, K, 64, 1, 0, head_dim=d)
    cent = torch.empty(H, K, d, dtype=torch.bfloat16, device=x.device)
    counts = torch.empty(H, K, dtype=torch.int32, device=x.device)
    need = workspace_bytes(p, ENTRY_KMEANS_UPDATE, N)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=x.device)
    st = lib().qvg_kmeans_update(C.byref(p), N, _ptr(x), sh, st_, _ptr(ids.contiguous()),
                                 _ptr(centroids_prev), _ptr(cent), _ptr(counts), _ptr(ws), need, _stream())
    if st != 0:
        raise QvgError(st, "qvg_kmeans_update")
    return cent, counts


class StreamingCache:
    """The compressed K and V cache of one layer during a chunk-by-chunk rollout (paper Sec. 3.1,
    4.3): allocated once for `capacity_tokens`, filled by `append`, read by `attend` / `decode`.
    K heads and V heads are stacked as 2 * heads independent units so that one library call
    encodes both.  Every chunk but the last appended one must be full (chunk_len tokens).
    Argument marshalling only: every step runs in the library's kernels.

    A chunk's k-means starts from the previous chunk's centroids (Sec. 4.3: centroid caching) and
    runs `warm_iters` Lloyd iterations; the first chunk starts from `init` ([2 * heads, K, d], or
    [2 * heads, S, K, d] with S smoothing stages) and runs `cold_iters`."""

    def __init__(self, heads, capacity_tokens, chunk_len, n_clusters, group_size, n_stages, head_dim=128,
                 device="cuda", n_smooth=1, bits=2, scale_format=SCALE_F16, warm_iters=3, cold_iters=10):
        self.heads, self.chunk_len = heads, chunk_len
        self.group_size, self.n_stages = group_size, n_stages
        self.warm_iters, self.cold_iters = warm_iters, cold_iters
        self.cache = alloc_cache(2 * heads, capacity_tokens, chunk_len, n_clusters, group_size, n_stages, head_dim,
                                 device, n_smooth=n_smooth, bits=bits, scale_format=scale_format)
        self.n_tokens = 0
        p = make_params(2 * heads, n_clusters, group_size, n_stages, max(warm_iters, cold_iters), head_dim=head_dim,
                        bits=bits, n_smooth_stages=n_smooth, scale_format=scale_format)
        need = workspace_bytes(p, ENTRY_ENCODE, chunk_len)
        self._ws = torch.empty(max(need, 16), dtype=torch.uint8, device=device)

    @property
    def capacity(self) -> int:
        return self.cache.ids.shape[1]

    def _side(self, lo, hi) -> Encoded:
        c = self.cache
        return Encoded(c.centroids[lo:hi], c.ids[lo:hi], c.codes[lo:hi], c.scales[lo:hi], c.chunk_len, c.n_smooth)

    @property
    def k(self) -> Encoded:
        return self._side(0, self.heads)

    @property
    def v(self) -> Encoded:
        return self._side(self.heads, 2 * self.heads)

    def append(self, kv_chunk, init=None, iters=None) -> int:
        """Encode one chunk, kv_chunk [2 * heads, n, d] bf16 (K heads first), n <= chunk_len, at the
        end of the cache.  Returns the chunk's index."""
        if self.n_tokens % self.chunk_len != 0:
            raise ValueError("the previous chunk was not full: nothing can be appended after it")
        n = kv_chunk.shape[1]
        if n < 1 or n > self.chunk_len or self.n_tokens + n > self.capacity:
            raise ValueError("chunk does not fit")
        c = self.n_tokens // self.chunk_len
        if c > 0 and init is None:
            init = self.cache.centroids[:, c - 1]
            iters = self.warm_iters if iters is None else iters
        elif init is None:
            raise ValueError("the first chunk needs start centroids")
        else:
            iters = (self.cold_iters if c == 0 else self.warm_iters) if iters is None else iters
        encode_chunk(kv_chunk, init, self.group_size, self.n_stages, iters, cache=self.cache, chunk_index=c,
                     workspace=self._ws)
        self.n_tokens += n
        return c

    def attend(self, q, k_rope=None, softmax_scale=None, want_lse=False, out=None, workspace=None):
        """Attention of q [heads, n_q, d] over the tokens appended so far (decode fused in)."""
        if self.n_tokens == 0:
            raise ValueError("the cache is empty")
        return attn_decode(q, self.k, self.v, softmax_scale=softmax_scale, want_lse=want_lse, out=out,
                           n_kv=self.n_tokens, k_rope=k_rope, workspace=workspace)

    def decode(self, out=None, first_chunk=0, n_tokens=None) -> torch.Tensor:
        """bf16 [2 * heads, n, d] of the tokens appended so far, from chunk `first_chunk` on."""
        first = first_chunk * self.chunk_len
        n = self.n_tokens - first if n_tokens is None else n_tokens
        if first + n > self.n_tokens:
            raise ValueError("range beyond the tokens appended so far")
        return decode(self.cache, out=out, n_tokens=n, first_token=first)

    def stored_bytes(self) -> int:
        """Bytes the appended tokens occupy (codes, scales, ids and the chunks' tables)."""
        c = self.cache
        per_tok = c.codes.shape[2] * c.codes.shape[3] + c.scales.shape[2] * c.scales.shape[3] * c.scales.element_size() \
            + c.n_smooth * c.ids.element_size()
        chunks = -(-self.n_tokens // self.chunk_len)
        table = c.n_smooth * c.centroids.shape[-2] * c.centroids.shape[-1] * 2
        return 2 * self.heads * (self.n_tokens * per_tok + chunks * table)
