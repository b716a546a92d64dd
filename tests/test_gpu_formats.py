"""Stored-format variants (Sec. 5 "Implementation": FP8 E4M3 per-group scales; Sec. 5: INT4
levels) on the GPU against the oracle: tables, ids, codes and scale bytes bit-equal, decode
bit-equal, attention within the stated tolerance."""
import numpy as np
import pytest
import torch

from oracle import qvg_oracle as O
from paper_2602_02958_amd import binding as B
from paper_2602_02958_amd import synth
from paper_2602_02958_amd.configs import CONFIGS
from conftest import bf16_bits, bits_to_f32
import parity_util as P

pytestmark = pytest.mark.gpu
DEV = "cuda"
F16, E4M3 = B.SCALE_F16, B.SCALE_E4M3


def _scales_np(enc):
    """stored scales as the oracle keeps them: uint16 (binary16 bits, or the E4M3 code)"""
    if enc.scales.dtype == torch.uint8:
        return P.to_np_u8(enc.scales).astype(np.uint16)
    return P.to_np_u16(enc.scales)


def _inputs(cfg, H, N, K, S=1):
    wl = CONFIGS[cfg]
    x = synth.MixtureStream(wl, H, 0, "cpu").next_chunk(N)
    init = torch.stack([synth.cold_start_centroids(x, K, seed=s) for s in range(S)], 1)      # [H,S,K,d]
    return x, (init if S > 1 else init[:, 0])


@pytest.mark.parametrize("cfg,H,N,K,Bg,T,S,I,bits,fmt", [
    ("cfg2_window21", 3, 1500, 64, 64, 1, 1, 2, 2, E4M3),     # the paper's QVG format: INT2, B = 64, FP8 scales
    ("cfg1_tiny", 2, 700, 16, 16, 3, 1, 3, 2, E4M3),
    ("cfg1_tiny", 2, 333, 16, 128, 2, 1, 0, 2, E4M3),
    ("cfg3_dit_small", 2, 1000, 256, 16, 1, 4, 1, 2, E4M3),   # QVG-Pro: S = 4, B = 16, FP8 scales
    ("cfg2_window21", 3, 1500, 64, 64, 1, 1, 2, 4, E4M3),     # INT4 of the same
    ("cfg1_tiny", 2, 700, 16, 32, 2, 1, 3, 4, F16),
    ("cfg1_tiny", 1, 300, 16, 128, 3, 2, 1, 4, F16),
    ("cfg3_dit_small", 2, 1000, 256, 16, 1, 4, 1, 4, E4M3),   # QVG-Pro INT4
    ("cfg1_tiny", 2, 17, 16, 64, 8, 1, 1, 4, E4M3),           # fewer tokens than a pass, 8 rounds
    ("cfg3_dit_small", 2, 1200, 512, 64, 1, 1, 2, 2, E4M3),   # the codebook-size study's K = 512: 16-bit ids
    ("cfg3_dit_small", 2, 1200, 512, 64, 1, 1, 2, 4, E4M3),
])
def test_encode_decode_in_other_formats(cfg, H, N, K, Bg, T, S, I, bits, fmt):
    x, init = _inputs(cfg, H, N, K, S)
    enc = B.encode_chunk(x.to(DEV), init.to(DEV), Bg, T, I, bits=bits, scale_format=fmt)
    dec = B.decode(enc)
    torch.cuda.synchronize()
    assert enc.codes.shape == (H, N, T, 16 * bits) and enc.bits == bits and enc.scale_format == fmt
    ref = O.encode_batch(bf16_bits(x), bf16_bits(init), K, Bg, T, I, S=S, bits=bits, scale_fmt=fmt)
    cent = P.to_np_u16(enc.centroids[:, 0]).reshape(H, S, K, 128)
    ids = P.to_np_u8(enc.ids).reshape(H, N, S).transpose(0, 2, 1)
    assert np.array_equal(cent, ref["cent"])
    assert np.array_equal(ids, ref["ids"])
    assert np.array_equal(_scales_np(enc), ref["scales"])
    assert np.array_equal(P.to_np_u8(enc.codes), ref["codes"])
    want = O.decode_batch(ref["cent"], ref["ids"], ref["codes"], ref["scales"], Bg, bits=bits, scale_fmt=fmt)
    assert np.array_equal(P.to_np_u16(dec), want)
    assert B.compressed_bytes(B.make_params(H, K, Bg, T, I, n_smooth_stages=S, bits=bits, scale_format=fmt), N) == \
        enc.codes.numel() + enc.scales.numel() * enc.scales.element_size() + enc.ids.numel() * enc.ids.element_size() + \
        enc.centroids.numel() * 2


def test_e4m3_scale_of_every_bf16_magnitude():
    """Every non-negative finite bf16 value as the maximum of a group of its own (zero centroid):
    the stored byte is the oracle's E4M3 conversion (itself pinned to torch's), over subnormals,
    all exact ties (bf16 has more mantissa bits than E4M3) and saturation beyond 448.  The second
    round sees fp32 residuals that are not bf16 values."""
    vals = np.arange(0, 0x7F80, dtype=np.uint16)                      # all finite non-negative bf16
    N = vals.size
    x = np.zeros((1, N, 128), np.uint16)
    x[0, :, 5] = vals
    x[0, :, 70] = vals ^ 0x8000                                       # second group: the negative value
    x[0, 1:, 71] = vals[:-1]                                          # and a smaller companion
    xt = torch.from_numpy(x.view(np.int16)).view(torch.bfloat16)
    init = torch.zeros(1, 1, 128, dtype=torch.bfloat16)
    for bits in (2, 4):
        enc = B.encode_chunk(xt.to(DEV), init.to(DEV), 64, 2, 0, bits=bits, scale_format=E4M3)
        dec = B.decode(enc)
        torch.cuda.synchronize()
        ref = O.encode_batch(x, bf16_bits(init), 1, 64, 2, 0, bits=bits, scale_fmt=1)
        sc = _scales_np(enc)
        assert np.array_equal(sc, ref["scales"])
        assert np.array_equal(P.to_np_u8(enc.codes), ref["codes"])
        assert sc.max() == 0x7E and (sc[0, bits_to_f32(vals) > 448.0 * (7 if bits == 4 else 1), 0, 0] == 0x7E).all()
        want = O.decode_batch(ref["cent"], ref["ids"], ref["codes"], ref["scales"], 64, bits=bits, scale_fmt=1)
        assert np.array_equal(P.to_np_u16(dec), want)


@pytest.mark.parametrize("bits,fmt", [(2, E4M3), (4, F16), (4, E4M3)])
def test_decode_random_storage_all_table_placements(bits, fmt):
    """Random valid storage (every level, every scale code incl. subnormal ones), several ragged
    chunks, tables in LDS (S = 1, 2) and in global memory (S = 4, K = 256)."""
    g = torch.Generator().manual_seed(5 + bits + fmt)
    for (S, K, T) in ((1, 64, 1), (1, 256, 3), (2, 64, 2), (4, 256, 1)):
        H, N, L, Bg = 2, 1111, 400, 32
        cache = B.alloc_cache(H, N, L, K, Bg, T, 128, DEV, n_smooth=S, bits=bits, scale_format=fmt)
        cache.centroids.copy_(torch.randn(cache.centroids.shape, generator=g).to(torch.bfloat16))
        cache.ids.copy_(torch.randint(0, K, cache.ids.shape, generator=g, dtype=torch.uint8))
        if bits == 2:
            f = torch.tensor([0, 1, 3], dtype=torch.uint8)[torch.randint(0, 3, cache.codes.shape + (4,), generator=g)]
            cache.codes.copy_(f[..., 0] | (f[..., 1] << 2) | (f[..., 2] << 4) | (f[..., 3] << 6))
        else:
            f = (torch.randint(-7, 8, cache.codes.shape + (2,), generator=g) & 15).to(torch.uint8)
            cache.codes.copy_(f[..., 0] | (f[..., 1] << 4))
        if fmt == E4M3:
            cache.scales.copy_(torch.randint(0, 0x60, cache.scales.shape, generator=g, dtype=torch.uint8))
        else:
            cache.scales.copy_(torch.rand(cache.scales.shape, generator=g).to(torch.float16))
        out = B.decode(cache)
        torch.cuda.synchronize()
        sc = _scales_np(cache)
        for h in range(H):
            for c in range(-(-N // L)):
                sl = slice(c * L, min((c + 1) * L, N))
                cent = P.to_np_u16(cache.centroids[h, c]).reshape(S, K, 128)
                ids = P.to_np_u8(cache.ids[h, sl]).reshape(-1, S).T
                want = O.decode_unit(cent, ids, P.to_np_u8(cache.codes[h, sl]), sc[h, sl], Bg, bits=bits,
                                     scale_fmt=fmt)
                assert np.array_equal(P.to_np_u16(out[h, sl]), want), (S, K, T, h, c)


@pytest.mark.parametrize("bits,fmt,S,T,Bg", [(2, E4M3, 1, 1, 64), (2, E4M3, 1, 3, 32), (4, E4M3, 1, 1, 64),
                                             (4, F16, 1, 2, 16), (2, E4M3, 2, 1, 16), (4, E4M3, 2, 2, 64)])
@pytest.mark.parametrize("trim", [37, 40])
def test_attention_over_cache_in_other_formats(bits, fmt, S, T, Bg, trim):
    """trim = 40: every unit's scale array starts on a 16-byte boundary, so the formats the staged
    kernel knows (E4M3 scales with one smoothing stage: 2-bit levels, or 4-bit levels in one round)
    run there; trim = 37: the general kernel."""
    wl = CONFIGS["cfg2_window21"]
    H, L, n_chunks, K, Nq = 2, 520, 3, 64, 300
    N = L * n_chunks - trim                                 # ragged last chunk
    caches = []
    for kv in (0, 1):
        st = synth.MixtureStream(wl, H, kv, DEV)
        cache = B.alloc_cache(H, N, L, K, Bg, T, 128, DEV, n_smooth=S, bits=bits, scale_format=fmt)
        for c in range(n_chunks):
            n = min(L, N - c * L)
            x = st.next_chunk(n)
            init = torch.stack([synth.cold_start_centroids(x, K, seed=s) for s in range(S)], 1)
            B.encode_chunk(x, init if S > 1 else init[:, 0], Bg, T, 2, cache=cache, chunk_index=c)
        caches.append(cache)
    q = synth.queries(wl, H, Nq, DEV)
    out, lse = B.attn_decode(q, caches[0], caches[1], want_lse=True)
    khat, vhat = B.decode(caches[0]), B.decode(caches[1])
    torch.cuda.synchronize()
    for h in range(H):
        # the decoded cache itself is the oracle's (bit-equal), checked on the K side here
        kc = caches[0]
        sl = slice(0, L)
        want_k = O.decode_unit(P.to_np_u16(kc.centroids[h, 0]).reshape(S, K, 128),
                               P.to_np_u8(kc.ids[h, sl]).reshape(-1, S).T, P.to_np_u8(kc.codes[h, sl]),
                               _scales_np(kc)[h, sl], Bg, bits=bits, scale_fmt=fmt)
        assert np.array_equal(P.to_np_u16(khat[h, sl]), want_k)
        want, lse_w = O.attention(bf16_bits(q[h]), P.to_np_u16(khat[h]), P.to_np_u16(vhat[h]), want_lse=True)
        ok, max_abs, worst = P.attn_tolerance_ok(P.to_np_u16(out[h]), want)
        assert ok, f"head {h}: max abs err {max_abs}, worst err/tol {worst}"
        assert np.abs(lse[h].cpu().numpy() - lse_w).max() < 2e-3


def test_more_levels_and_more_rounds_reconstruct_better():
    """Sec. 5 (INT4 rows against INT2 rows) and Sec. 4.2 (coarse to fine): the error of the decoded
    cache falls with the bit width and with the number of rounds; FP8 scales cost little."""
    x, init = _inputs("cfg2_window21", 2, 2000, 64)
    xf = x.float()
    err = {}
    for bits in (2, 4):
        for fmt in (F16, E4M3):
            for T in (1, 2):
                enc = B.encode_chunk(x.to(DEV), init.to(DEV), 64, T, 3, bits=bits, scale_format=fmt)
                err[bits, fmt, T] = float((B.decode(enc).float().cpu() - xf).pow(2).mean())
    for fmt in (F16, E4M3):
        assert err[4, fmt, 1] < 0.2 * err[2, fmt, 1]
        for bits in (2, 4):
            assert err[bits, fmt, 2] < 0.5 * err[bits, fmt, 1]
    for bits in (2, 4):
        assert err[bits, E4M3, 1] < 1.25 * err[bits, F16, 1]


def test_seeded_sweep_over_parameter_combinations():
    """Forty seeded draws of (H, N, chunk length, K, B, T, S, bits, scale format, Lloyd iterations):
    a cache filled chunk by chunk, every stored array and the decode bit-equal to the oracle, the
    fused attention over a random prefix within tolerance.  Small sizes, many shapes: ragged
    chunks, K not a multiple of 32, N < K, single tokens."""
    rng = np.random.default_rng(77)
    wl = CONFIGS["cfg1_tiny"]
    for draw in range(40):
        H = int(rng.integers(1, 4))
        K = int(rng.choice([1, 3, 16, 33, 64, 100, 256]))
        Bg = int(rng.choice([16, 32, 64, 128]))
        T = int(rng.integers(1, 5)) if draw % 5 else int(rng.integers(5, 9))
        S = int(rng.choice([1, 1, 1, 2, 3]))
        bits = int(rng.choice([2, 4]))
        fmt = int(rng.choice([F16, E4M3]))
        I = int(rng.integers(0, 3))
        n_chunks = int(rng.integers(1, 4))
        # f16 scale arrays are written with 16-byte stores: chunks must start on such a boundary
        step = 8 if fmt == F16 else 1
        L = int(rng.integers(1, 40)) * step
        last = int(rng.integers(1, L + 1))
        N = L * (n_chunks - 1) + last
        tag = dict(draw=draw, H=H, K=K, B=Bg, T=T, S=S, bits=bits, fmt=fmt, I=I, L=L, N=N)
        caches, xs = [], []
        for kv in (0, 1):
            st = synth.MixtureStream(wl, H, kv, DEV)
            cache = B.alloc_cache(H, N, L, K, Bg, T, 128, DEV, n_smooth=S, bits=bits, scale_format=fmt)
            for c in range(n_chunks):
                n = min(L, N - c * L)
                x = st.next_chunk(n)
                init = torch.randn(H, S, K, 128, device=DEV).to(torch.bfloat16)
                B.encode_chunk(x, init if S > 1 else init[:, 0].contiguous(), Bg, T, I, cache=cache, chunk_index=c)
                ref = O.encode_batch(bf16_bits(x), bf16_bits(init), K, Bg, T, I, S=S, bits=bits, scale_fmt=fmt)
                sl = slice(c * L, c * L + n)
                assert np.array_equal(P.to_np_u16(cache.centroids[:, c]).reshape(H, S, K, 128), ref["cent"]), tag
                assert np.array_equal(P.to_np_u8(cache.ids[:, sl]).reshape(H, n, S).transpose(0, 2, 1), ref["ids"]), tag
                assert np.array_equal(P.to_np_u8(cache.codes[:, sl]), ref["codes"]), tag
                assert np.array_equal(_scales_np(cache)[:, sl], ref["scales"]), tag
                want = O.decode_batch(ref["cent"], ref["ids"], ref["codes"], ref["scales"], Bg, bits=bits, scale_fmt=fmt)
                got = B.decode(cache, n_tokens=n, first_token=c * L)
                assert np.array_equal(P.to_np_u16(got), want), tag
            caches.append(cache)
        n_kv = int(rng.integers(1, N + 1))
        Nq = int(rng.integers(1, 70))
        q = synth.queries(wl, H, Nq, DEV)
        out, lse = B.attn_decode(q, caches[0], caches[1], want_lse=True, n_kv=n_kv)
        khat, vhat = B.decode(caches[0]), B.decode(caches[1])
        torch.cuda.synchronize()
        for h in range(H):
            want, lse_w = O.attention(bf16_bits(q[h]), P.to_np_u16(khat[h, :n_kv]), P.to_np_u16(vhat[h, :n_kv]), want_lse=True)
            # this workload has channels scaled x8: the tolerance with the f16-probability term
            ok, max_abs, worst = P.attn_tolerance_wide_range_ok(P.to_np_u16(out[h]), want, bf16_bits(q[h]),
                                                                P.to_np_u16(khat[h, :n_kv]), P.to_np_u16(vhat[h, :n_kv]))
            assert ok, (tag, h, max_abs, worst)
            assert np.abs(lse[h].cpu().numpy() - lse_w).max() < 2e-3, tag
