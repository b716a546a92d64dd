"""Several smoothing stages (the paper's progressive residual quantization, Sec. 4.2: k-means on
the residual of the previous k-means, S times, then the quantizer) on the GPU against the
oracle: stored tables, ids, codes and scales bit-equal, decode bit-equal, attention within the
stated tolerance."""
import numpy as np
import pytest
import torch

from oracle import qvg_oracle as O
from paper_2602_02958_amd import binding as B
from paper_2602_02958_amd import synth
from paper_2602_02958_amd.configs import CONFIGS
from conftest import bf16_bits
import parity_util as P

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _inputs(cfg, H, N, K, S, seed0=0):
    wl = CONFIGS[cfg]
    x = synth.MixtureStream(wl, H, 0, "cpu").next_chunk(N)
    init = torch.stack([synth.cold_start_centroids(x, K, seed=seed0 + s) for s in range(S)], 1)  # [H,S,K,d]
    return x, init


@pytest.mark.parametrize("cfg,H,N,K,Bg,T,S,I", [
    ("cfg1_tiny", 2, 700, 16, 64, 1, 2, 3),
    ("cfg2_window21", 3, 1500, 64, 32, 2, 3, 2),
    ("cfg3_dit_small", 2, 1000, 256, 16, 1, 4, 1),      # the paper's QVG-Pro shape: S = 4, B = 16
    ("cfg1_tiny", 1, 300, 16, 128, 2, 2, 0),            # no Lloyd iterations: start tables are final
    ("cfg2_window21", 2, 1300, 300, 64, 2, 2, 2),       # more than 256 centroids: 16-bit ids, two per token
    ("cfg3_dit_small", 2, 900, 512, 16, 1, 4, 1),       # QVG-Pro with the largest codebook
])
def test_encode_decode_with_smoothing_stages(cfg, H, N, K, Bg, T, S, I):
    x, init = _inputs(cfg, H, N, K, S)
    enc = B.encode_chunk(x.to(DEV), init.to(DEV), Bg, T, I)
    dec = B.decode(enc)
    torch.cuda.synchronize()
    ref = O.encode_batch(bf16_bits(x), bf16_bits(init), K, Bg, T, I, S=S)
    assert enc.centroids.shape == (H, 1, S, K, 128) and enc.ids.shape == (H, N, S)
    assert np.array_equal(P.to_np_u16(enc.centroids[:, 0]), ref["cent"])
    ids = P.to_np_u8(enc.ids) if K <= 256 else P.to_np_u16(enc.ids)
    assert np.array_equal(ids, ref["ids"].transpose(0, 2, 1))
    assert np.array_equal(P.to_np_u8(enc.codes), ref["codes"])
    assert np.array_equal(P.to_np_u16(enc.scales), ref["scales"])
    want = O.decode_batch(ref["cent"], ref["ids"], ref["codes"], ref["scales"], Bg)
    assert np.array_equal(P.to_np_u16(dec), want)


def test_decode_tables_in_lds_and_in_global_memory():
    """S*K*256 B <= 64 KB keeps every stage's table in LDS; beyond that the rows are gathered
    from global memory.  Random valid storage, several chunks."""
    g = torch.Generator().manual_seed(11)
    for (S, K) in ((2, 64), (4, 64), (2, 256), (4, 256)):
        H, N, L, T, Bg = 2, 1111, 400, 2, 32
        cache = B.alloc_cache(H, N, L, K, Bg, T, 128, DEV, n_smooth=S)
        cache.centroids.copy_(torch.randn(cache.centroids.shape, generator=g).to(torch.bfloat16))
        cache.ids.copy_(torch.randint(0, K, cache.ids.shape, generator=g, dtype=torch.uint8))
        f = torch.tensor([0, 1, 3], dtype=torch.uint8)[torch.randint(0, 3, cache.codes.shape + (4,), generator=g)]
        cache.codes.copy_(f[..., 0] | (f[..., 1] << 2) | (f[..., 2] << 4) | (f[..., 3] << 6))
        cache.scales.copy_(torch.rand(cache.scales.shape, generator=g).to(torch.float16))
        out = B.decode(cache)
        torch.cuda.synchronize()
        for h in range(H):
            for c in range(-(-N // L)):
                sl = slice(c * L, min((c + 1) * L, N))
                want = O.decode_unit(P.to_np_u16(cache.centroids[h, c]), P.to_np_u8(cache.ids[h, sl]).T,
                                     P.to_np_u8(cache.codes[h, sl]), P.to_np_u16(cache.scales[h, sl]), Bg)
                assert np.array_equal(P.to_np_u16(out[h, sl]), want), (S, K, h, c)


def test_attention_over_cache_with_smoothing_stages():
    wl = CONFIGS["cfg2_window21"]
    H, L, n_chunks, K, Bg, T, S, Nq = 2, 520, 3, 64, 32, 2, 2, 300
    N = L * n_chunks - 37                                   # ragged last chunk
    caches = []
    for kv in (0, 1):
        st = synth.MixtureStream(wl, H, kv, DEV)
        cache = B.alloc_cache(H, N, L, K, Bg, T, 128, DEV, n_smooth=S)
        for c in range(n_chunks):
            n = min(L, N - c * L)
            x = st.next_chunk(n)
            init = torch.stack([synth.cold_start_centroids(x, K, seed=s) for s in range(S)], 1)
            B.encode_chunk(x, init, Bg, T, 2, cache=cache, chunk_index=c)
        caches.append(cache)
    q = synth.queries(wl, H, Nq, DEV)
    out, lse = B.attn_decode(q, caches[0], caches[1], want_lse=True)
    khat, vhat = B.decode(caches[0]), B.decode(caches[1])
    torch.cuda.synchronize()
    for h in range(H):
        want, lse_w = O.attention(bf16_bits(q[h]), P.to_np_u16(khat[h]), P.to_np_u16(vhat[h]), want_lse=True)
        ok, max_abs, worst = P.attn_tolerance_ok(P.to_np_u16(out[h]), want)
        assert ok, f"head {h}: max abs err {max_abs}, worst err/tol {worst}"
        assert np.abs(lse[h].cpu().numpy() - lse_w).max() < 2e-3


@pytest.mark.parametrize("S,K,T,Bg,fmt,bits", [(2, 300, 2, 32, B.SCALE_F16, 2), (4, 384, 1, 16, B.SCALE_E4M3, 2),
                                               (2, 512, 1, 64, B.SCALE_E4M3, 4)])
def test_attention_with_16_bit_ids_and_several_stages(S, K, T, Bg, fmt, bits):
    """More than 256 centroids per stage AND several smoothing stages: a token has S 16-bit ids.  One
    kernel, with the tile workspace, and with a prefix length per query, each against the oracle."""
    wl = CONFIGS["cfg2_window21"]
    H, L, n_chunks, Nq = 2, 520, 3, 600
    N = L * n_chunks - 37
    caches = []
    for kv in (0, 1):
        st = synth.MixtureStream(wl, H, kv, DEV)
        cache = B.alloc_cache(H, N, L, K, Bg, T, 128, DEV, n_smooth=S, bits=bits, scale_format=fmt)
        for c in range(n_chunks):
            n = min(L, N - c * L)
            x = st.next_chunk(n)
            init = torch.stack([synth.cold_start_centroids(x, K, seed=s) for s in range(S)], 1)
            B.encode_chunk(x, init, Bg, T, 1, cache=cache, chunk_index=c)
        caches.append(cache)
    assert caches[0].ids.dtype == B.id_dtype(K) and caches[0].ids.shape == (H, N, S)
    q = synth.queries(wl, H, Nq, DEV)
    khat, vhat = B.decode(caches[0]), B.decode(caches[1])
    torch.cuda.synchronize()
    # the decode against the oracle's, chunk by chunk
    for h in range(H):
        for c in range(n_chunks):
            sl = slice(c * L, min((c + 1) * L, N))
            want = O.decode_unit(P.to_np_u16(caches[0].centroids[h, c]), P.to_np_u16(caches[0].ids[h, sl]).T,
                                 P.to_np_u8(caches[0].codes[h, sl]),
                                 P.to_np_u16(caches[0].scales[h, sl]) if fmt == B.SCALE_F16 else P.to_np_u8(caches[0].scales[h, sl]),
                                 Bg, bits=bits, scale_fmt=fmt)
            assert np.array_equal(P.to_np_u16(khat[h, sl]), want), (h, c)
    ws = B.attn_workspace(H, Nq, L, 2, DEV)
    lens = torch.full((Nq,), N, dtype=torch.int32, device=DEV)
    lens[:100] = L + 3
    for kw in (dict(), dict(workspace=ws), dict(q_kv_len=lens), dict(q_kv_len=lens, workspace=ws)):
        out, lse = B.attn_decode(q, caches[0], caches[1], want_lse=True, **kw)
        torch.cuda.synchronize()
        for h in range(H):
            for rows, n in ((slice(0, 100), L + 3 if "q_kv_len" in kw else N), (slice(100, Nq), N)):
                want, lse_w = O.attention(bf16_bits(q[h])[rows], P.to_np_u16(khat[h, :n]), P.to_np_u16(vhat[h, :n]), want_lse=True)
                ok, max_abs, worst = P.attn_tolerance_ok(P.to_np_u16(out[h])[rows], want)
                assert ok, f"{sorted(kw)} head {h}: max abs err {max_abs}, worst err/tol {worst}"
                assert np.abs(lse[h].cpu().numpy()[rows] - lse_w).max() < 2e-3
