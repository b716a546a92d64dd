"""The C-ABI library loads, exports every symbol include/qvg.h declares, and its host-side
argument validation answers without a GPU (no kernel is launched by any call here)."""
import ctypes as C
import os
import re

import pytest

from paper_2602_02958_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "qvg.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qvg_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    L = B.lib()
    names = _declared()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert hasattr(L, n), n


def test_version_and_status_strings():
    assert B.lib().qvg_version() >= 100
    for st in range(0, -8, -1):
        assert len(B.status_string(st)) > 0
    assert B.status_string(-99) == "unknown status"


def test_compressed_bytes_matches_format():
    p = B.make_params(24, 256, 64, 2)
    assert B.compressed_bytes(p, 4680) == 24 * (4680 * 73 + 256 * 128 * 2)
    p = B.make_params(1, 64, 32, 3)
    assert B.compressed_bytes(p, 10) == 10 * 121 + 64 * 256
    # the paper's own formats (Sec. 5): one round, FP8 scales; INT2 B=64 -> 32 + 2 + 1 bytes per
    # token, INT4 QVG-Pro (S = 4, B = 16) -> 64 + 8 + 4
    p = B.make_params(1, 256, 64, 1, scale_format=B.SCALE_E4M3)
    assert B.compressed_bytes(p, 1000) == 1000 * 35 + 256 * 256
    p = B.make_params(1, 256, 16, 1, bits=4, n_smooth_stages=4, scale_format=B.SCALE_E4M3)
    assert B.compressed_bytes(p, 1000) == 1000 * 76 + 4 * 256 * 256
    # more than 256 centroids: two id bytes per token
    p = B.make_params(1, 512, 64, 1, scale_format=B.SCALE_E4M3)
    assert B.compressed_bytes(p, 1000) == 1000 * 36 + 512 * 256


def test_params_struct_layout():
    # nine consecutive int32 fields, in the order of include/qvg.h
    text = open(os.path.join(ROOT, "include", "qvg.h")).read()
    body = text[text.index("typedef struct qvg_params {"):text.index("} qvg_params;")]
    names = re.findall(r"int32_t\s+([a-z_]+);", body)
    assert names == [f[0] for f in B.QvgParams._fields_]
    assert C.sizeof(B.QvgParams) == 4 * len(names)


@pytest.mark.parametrize("kw,status", [
    (dict(n_heads=0), -2), (dict(n_clusters=0), -2), (dict(n_clusters=257), 0), (dict(n_clusters=512), 0),
    (dict(n_clusters=513), -2), (dict(n_clusters=512, n_smooth_stages=2), 0),
    (dict(n_stages=0), -2), (dict(n_stages=9), -2), (dict(group_size=48), -2),
    (dict(head_dim=64), -3), (dict(bits=4), 0), (dict(bits=3), -2), (dict(bits=8), -2),
    (dict(scale_format=1), 0), (dict(scale_format=2), -2), (dict(scale_format=-1), -2),
    (dict(n_smooth_stages=5), -3), (dict(n_smooth_stages=0), -2), (dict(group_size=8), -3), (dict(kmeans_iters=-1), -2),
])
def test_parameter_validation(kw, status):
    base = dict(n_heads=2, n_clusters=16, group_size=64, n_stages=2, kmeans_iters=0,
                head_dim=128, bits=2, n_smooth_stages=1, scale_format=0)
    base.update(kw)
    p = B.make_params(**base)
    out = C.c_size_t(0)
    assert B.lib().qvg_workspace_bytes(C.byref(p), 0, 100, 0, C.byref(out)) == status


def test_null_and_alignment_errors_are_reported_before_any_launch():
    L = B.lib()
    p = B.make_params(2, 16, 64, 2, kmeans_iters=1)
    fake = C.c_void_p(0x1000)          # aligned, never dereferenced: every call below fails first
    odd = C.c_void_p(0x1008)
    # NULL x
    assert L.qvg_encode_chunk(C.byref(p), 10, None, 1280, 128, fake, fake, 0, fake, fake, fake, 0,
                              None, 0, None) == -1
    # misaligned x
    assert L.qvg_encode_chunk(C.byref(p), 10, odd, 1280, 128, fake, fake, 0, fake, fake, fake, 0,
                              None, 0, None) == -5
    # stride not a multiple of 8
    assert L.qvg_encode_chunk(C.byref(p), 10, fake, 1284, 132, fake, fake, 0, fake, fake, fake, 0,
                              None, 0, None) == -5
    # workspace missing although kmeans_iters > 0
    assert L.qvg_encode_chunk(C.byref(p), 10, fake, 1280, 128, fake, fake, 0, fake, fake, fake, 0,
                              None, 0, None) == -4
    # too many tokens for one chunk
    assert L.qvg_encode_chunk(C.byref(p), (1 << 20) + 1, fake, 1 << 28, 128, fake, fake, 0, fake,
                              fake, fake, 0, None, 0, None) == -2
    # output stride smaller than the chunk
    assert L.qvg_encode_chunk(C.byref(p), 10, fake, 1280, 128, fake, fake, 0, fake, fake, fake, 5,
                              fake, 1 << 30, None) == -2
    # decode / attention
    assert L.qvg_decode(C.byref(p), 10, 0, fake, fake, fake, fake, fake, 1280, 128, None) == -2
    assert L.qvg_decode(C.byref(p), 10, 10, None, fake, fake, fake, fake, 1280, 128, None) == -1
    assert L.qvg_attn_decode(C.byref(p), 4, fake, 0, 10, fake, fake, fake, fake, fake, fake, fake,
                             fake, C.c_float(0.1), fake, None, None, 0, None) == -2
    assert L.qvg_attn_decode(C.byref(p), 4, fake, 10, 10, fake, fake, fake, fake, fake, fake, fake,
                             fake, C.c_float(float("nan")), fake, None, None, 0, None) == -2
    assert L.qvg_attn_decode(C.byref(p), 4, None, 10, 10, fake, fake, fake, fake, fake, fake, fake,
                             fake, C.c_float(0.1), fake, None, None, 0, None) == -1
    for bad in (0.0, -0.5, float("inf")):
        assert L.qvg_attn_decode(C.byref(p), 4, fake, 10, 10, fake, fake, fake, fake, fake, fake, fake,
                                 fake, C.c_float(bad), fake, None, None, 0, None) == -2
    # decode of a range: start off a chunk boundary, capacity below the range's end
    assert L.qvg_decode_ex(C.byref(p), 10, 10, 0, 5, fake, fake, fake, fake, fake, 1280, 128, None) == -2
    assert L.qvg_decode_ex(C.byref(p), 10, 10, 15, 10, fake, fake, fake, fake, fake, 1280, 128, None) == -2
    # extended attention: capacity below the fill, misaligned rotary table
    ex = lambda cap, rope: L.qvg_attn_decode_ex(C.byref(p), 4, fake, 10, 10, cap, fake, fake, fake, fake, fake, fake,
                                                fake, fake, rope, C.c_float(0.1), fake, None, None, 0, None)
    assert ex(5, None) == -2
    assert ex(0, C.c_void_p(0x1004)) == -5
    # prefix length per query: a misaligned length array
    assert L.qvg_attn_decode_causal(C.byref(p), 4, fake, 10, 10, 0, fake, fake, fake, fake, fake, fake, fake, fake,
                                    None, C.c_void_p(0x1002), C.c_float(0.1), fake, None, None, 0, None) == -5
    assert L.qvg_attn_decode_causal(C.byref(p), 0, None, 10, 10, 0, None, None, None, None, None, None, None, None,
                                    None, None, C.c_float(0.1), None, None, None, 0, None) == 0
    # merge
    assert L.qvg_attn_merge(4, 64, fake, fake, fake, fake, fake, None, None) == -3
    assert L.qvg_attn_merge(-1, 128, fake, fake, fake, fake, fake, None, None) == -2
    assert L.qvg_attn_merge(4, 128, fake, None, fake, fake, fake, None, None) == -1
    assert L.qvg_attn_merge(4, 128, odd, fake, fake, fake, fake, None, None) == -5
    assert L.qvg_attn_merge(0, 128, None, None, None, None, None, None, None) == 0
    # zero-size calls succeed without touching the device
    assert L.qvg_decode(C.byref(p), 0, 10, None, None, None, None, None, 0, 0, None) == 0
    assert L.qvg_attn_decode(C.byref(p), 0, None, 10, 10, None, None, None, None, None, None, None,
                             None, C.c_float(0.1), None, None, None, 0, None) == 0
    assert L.qvg_kmeans_assign(C.byref(p), 0, None, 0, 0, None, None, None, 0, None) == 0
    # 16-bit ids (more than 256 centroids) must be 2-byte aligned
    pw = B.make_params(2, 512, 64, 2)
    assert L.qvg_decode(C.byref(pw), 10, 10, fake, C.c_void_p(0x1001), fake, fake, fake, 1280, 128, None) == -5
    assert L.qvg_decode(C.byref(p), 10, 0, fake, C.c_void_p(0x1001), fake, fake, fake, 1280, 128, None) == -2


def test_workspace_sizes():
    p = B.make_params(24, 256, 64, 2, kmeans_iters=0)
    # a single pass needs only the assignment's scratch: 8 bytes per centroid row, 4 per unit
    small = B.workspace_bytes(p, B.ENTRY_ENCODE, 4680)
    assert 24 * 256 * 8 + 24 * 4 <= small <= 24 * 256 * 8 + 24 * 4 + 1024
    assert B.workspace_bytes(p, B.ENTRY_KMEANS_ASSIGN, 4680) == small
    assert B.workspace_bytes(p, B.ENTRY_ENCODE, 0) == 0
    p = B.make_params(24, 256, 64, 2, kmeans_iters=3)
    need = B.workspace_bytes(p, B.ENTRY_ENCODE, 4680)
    assert need >= 2 * 24 * 256 * 256 + 24 * 4680 * 4 + 24 * 257 * 4
    assert B.workspace_bytes(p, B.ENTRY_DECODE, 4680) == 0
    # attention's optional workspace: the decoded tiles (256 B per token and unit for K and for V, in
    # tiles of 64 tokens) + the queries' running state (66 floats per query slot of 256-query blocks)
    tiles = -(-4680 // 64)
    assert B.workspace_bytes(p, B.ENTRY_ATTN, 4680, 128) == 24 * tiles * 64 * 512 + 24 * 1 * 66 * 512 * 4


def test_static_scratch_entry_rejects_what_does_not_fit_before_touching_the_gpu():
    """qvg_encode_chunk_static: sizes whose workspace exceeds QVG_STATIC_SCRATCH_BYTES are refused
    with their own status, from the host-side size arithmetic alone."""
    L = B.lib()
    text = open(os.path.join(ROOT, "include", "qvg.h")).read()
    limit = eval(re.search(r"#define QVG_STATIC_SCRATCH_BYTES \((.*?)\)", text).group(1).replace("u", ""))
    fake = C.c_void_p(0x1000)
    big = B.make_params(720, 256, 64, 2, kmeans_iters=3)            # all 30 layers at once: two 47 MB tables
    assert B.workspace_bytes(big, B.ENTRY_ENCODE, 4680) > limit
    st = L.qvg_encode_chunk_static(C.byref(big), 4680, fake, 4680 * 128, 128, fake, fake, 0, fake, fake, fake, 0, None)
    assert st == -7 and "static" in B.status_string(st)
    ok = B.make_params(24, 256, 64, 4, kmeans_iters=10)             # one layer's chunk fits
    assert B.workspace_bytes(ok, B.ENTRY_ENCODE, 4680) <= limit
    # bad parameters are reported as for qvg_encode_chunk
    assert L.qvg_encode_chunk_static(C.byref(B.make_params(0, 256, 64, 2)), 10, fake, 1280, 128, fake, fake, 0,
                                     fake, fake, fake, 0, None) == -2
