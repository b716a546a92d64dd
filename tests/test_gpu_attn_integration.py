"""What a generation step needs around the fused attention (Sec. 3.1: a chunk attends to the
cached chunks and to itself; Sec. 5 "Implementation": keys are cached before the rotary
embedding): reading a prefix of a cache allocated for more tokens, rotating the decoded keys,
and merging with a second partial attention - each against the oracle."""
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


def _filled_caches(H, L, capacity_chunks, filled, K, Bg, T, S=1, bits=2, fmt=B.SCALE_F16):
    """K and V caches with room for capacity_chunks chunks of L tokens, the first `filled` tokens
    encoded (the rest zero bytes)."""
    wl = CONFIGS["cfg2_window21"]
    caches = []
    for kv in (0, 1):
        st = synth.MixtureStream(wl, H, kv, DEV)
        cache = B.alloc_cache(H, L * capacity_chunks, L, K, Bg, T, 128, DEV, n_smooth=S, bits=bits, scale_format=fmt)
        for t in (cache.centroids, cache.ids, cache.codes, cache.scales):
            t.zero_()
        c = 0
        while c * L < filled:
            n = min(L, filled - c * L)
            x = st.next_chunk(n)
            init = torch.stack([synth.cold_start_centroids(x, K, seed=s) for s in range(S)], 1)
            B.encode_chunk(x, init if S > 1 else init[:, 0], Bg, T, 2, cache=cache, chunk_index=c)
            c += 1
        caches.append(cache)
    return caches


def _rope_table(n, d=128, theta=10000.0, offset=0):
    pos = torch.arange(offset, offset + n, dtype=torch.float64)
    freq = theta ** (-torch.arange(d // 2, dtype=torch.float64) / (d // 2))
    ang = pos[:, None] * freq[None]
    return torch.stack([ang.cos(), ang.sin()], -1).to(torch.float16).contiguous()      # [n, d/2, 2]


def _check_against_oracle(q, out, lse, khat_bits, vhat_bits, h):
    want, lse_w = O.attention(bf16_bits(q[h]), khat_bits, vhat_bits, want_lse=True)
    ok, max_abs, worst = P.attn_tolerance_ok(P.to_np_u16(out[h]), want)
    assert ok, f"head {h}: max abs err {max_abs}, worst err/tol {worst}"
    assert np.abs(lse[h].cpu().numpy() - lse_w).max() < 2e-3


@pytest.mark.parametrize("L,T,Bg,bits,fmt", [(520, 2, 32, 2, B.SCALE_F16),      # staged kernel
                                             (516, 3, 64, 2, B.SCALE_F16),      # general kernel (chunks not on 16-byte scale boundaries)
                                             (520, 1, 64, 4, B.SCALE_E4M3)])
def test_attention_over_a_prefix_of_a_larger_cache(L, T, Bg, bits, fmt):
    H, K, Nq = 2, 64, 300
    filled = 2 * L + 133
    kc, vc = _filled_caches(H, L, 4, filled, K, Bg, T, bits=bits, fmt=fmt)
    q = synth.queries(CONFIGS["cfg2_window21"], H, Nq, DEV)
    khat, vhat = B.decode(kc), B.decode(vc)
    for n_kv in (filled, 2 * L, L + 7, 64, 1):
        out, lse = B.attn_decode(q, kc, vc, want_lse=True, n_kv=n_kv)
        torch.cuda.synchronize()
        for h in range(H):
            _check_against_oracle(q, out, lse, P.to_np_u16(khat[h, :n_kv]), P.to_np_u16(vhat[h, :n_kv]), h)


@pytest.mark.parametrize("L,T,Bg,S,bits,fmt", [(520, 2, 32, 1, 2, B.SCALE_F16),     # staged kernel
                                               (520, 4, 64, 1, 2, B.SCALE_F16),
                                               (516, 3, 64, 1, 2, B.SCALE_F16),     # general kernel
                                               (520, 1, 64, 1, 2, B.SCALE_E4M3),    # the paper's QVG format
                                               (520, 1, 16, 2, 4, B.SCALE_E4M3)])
def test_attention_with_rotary_embedding_of_decoded_keys(L, T, Bg, S, bits, fmt):
    H, K, Nq = 2, 64, 300
    filled = 2 * L + 133
    kc, vc = _filled_caches(H, L, 3, filled, K, Bg, T, S=S, bits=bits, fmt=fmt)
    q = synth.queries(CONFIGS["cfg2_window21"], H, Nq, DEV)
    rope = _rope_table(filled, offset=3)
    out, lse = B.attn_decode(q, kc, vc, want_lse=True, n_kv=filled, k_rope=rope.to(DEV))
    plain = B.attn_decode(q, kc, vc, n_kv=filled)
    khat, vhat = B.decode(kc), B.decode(vc)
    torch.cuda.synchronize()
    rope_bits = rope.view(torch.int16).numpy().view(np.uint16)
    for h in range(H):
        krot = O.rope_keys(P.to_np_u16(khat[h, :filled]), rope_bits)
        _check_against_oracle(q, out, lse, krot, P.to_np_u16(vhat[h, :filled]), h)
    assert (out.float() - plain.float()).abs().max() > 0.05          # the rotation is not a no-op
    # the identity rotation (cos 1, sin 0) reproduces the plain call bit for bit
    ident = torch.zeros(filled, 64, 2, dtype=torch.float16); ident[..., 0] = 1.0
    same = B.attn_decode(q, kc, vc, n_kv=filled, k_rope=ident.to(DEV))
    torch.cuda.synchronize()
    assert torch.equal(same, plain)


def test_merge_with_the_current_chunks_own_attention():
    """Cache part from the fused kernel, the current chunk's bf16 part from the oracle (standing in
    for the model's own attention kernel), merged on the GPU: equals attention over the union."""
    H, L, K, Bg, T, Nq, Ntail = 2, 520, 64, 32, 2, 333, 200
    filled = 2 * L + 50
    kc, vc = _filled_caches(H, L, 3, filled, K, Bg, T)
    wl = CONFIGS["cfg2_window21"]
    q = synth.queries(wl, H, Nq, DEV)
    tail_k = synth.MixtureStream(wl, H, 0, "cpu").next_chunk(Ntail)
    tail_v = synth.MixtureStream(wl, H, 1, "cpu").next_chunk(Ntail)
    out_a, lse_a = B.attn_decode(q, kc, vc, want_lse=True, n_kv=filled)
    khat, vhat = B.decode(kc), B.decode(vc)
    torch.cuda.synchronize()
    ob = np.empty((H, Nq, 128)); lb = np.empty((H, Nq))
    for h in range(H):
        ob[h], lb[h] = O.attention(bf16_bits(q[h]), bf16_bits(tail_k[h]), bf16_bits(tail_v[h]), want_lse=True)
    out_b = torch.from_numpy(ob).to(torch.bfloat16).to(DEV)
    lse_b = torch.from_numpy(lb).float().to(DEV)
    out, lse = B.attn_merge(out_a, lse_a, out_b, lse_b, want_lse=True)
    torch.cuda.synchronize()
    for h in range(H):
        ku = np.concatenate([P.to_np_u16(khat[h, :filled]), bf16_bits(tail_k[h])])
        vu = np.concatenate([P.to_np_u16(vhat[h, :filled]), bf16_bits(tail_v[h])])
        want, lse_w = O.attention(bf16_bits(q[h]), ku, vu, want_lse=True)
        # each partial result carries its own bf16 rounding (2^-9 relative) into the convex
        # combination, the merged row is rounded once more: 2e-3 + 2^-7 max(|o_a|, |o_b|, |o|)
        got = bits_to_f32(P.to_np_u16(out[h])).astype(np.float64)
        mag = np.maximum(np.maximum(np.abs(bits_to_f32(P.to_np_u16(out_a[h]))), np.abs(ob[h])), np.abs(want))
        assert (np.abs(got - want) <= 2e-3 + 2.0 ** -7 * mag).all()
        assert np.abs(lse[h].cpu().numpy() - lse_w).max() < 2e-3
        # against the oracle's merge of the very same partial results: only fp32 arithmetic and
        # the final bf16 rounding remain
        om, lm = O.attn_merge(bits_to_f32(P.to_np_u16(out_a[h])).astype(np.float64), lse_a[h].cpu().double().numpy(),
                              bits_to_f32(P.to_np_u16(out_b[h])).astype(np.float64), lse_b[h].cpu().double().numpy())
        assert (np.abs(got - om) <= 2.0 ** -8 * np.abs(om) + 1e-5).all()
        assert np.abs(lse[h].cpu().numpy() - lm).max() < 1e-4
    # in place, and with a second set that carries no weight
    out2 = B.attn_merge(out_a.clone(), lse_a, out_b, lse_b - 200.0)
    torch.cuda.synchronize()
    assert torch.equal(out2, out_a)
    buf = out_a.clone()
    B.attn_merge(buf, lse_a, out_b, lse_b, out=buf)
    torch.cuda.synchronize()
    assert torch.equal(buf, out)


@pytest.mark.parametrize("T,Bg,S,bits,fmt", [(2, 32, 1, 2, B.SCALE_F16), (1, 16, 2, 4, B.SCALE_E4M3)])
def test_decode_of_a_token_range_of_a_larger_cache(T, Bg, S, bits, fmt):
    H, L, K = 3, 520, 64
    filled = 3 * L + 77
    kc, _ = _filled_caches(H, L, 5, filled, K, Bg, T, S=S, bits=bits, fmt=fmt)
    whole = B.decode(kc)                                     # all 5 chunk slots (the unfilled ones hold zero bytes)
    torch.cuda.synchronize()
    sc = P.to_np_u8(kc.scales).astype(np.uint16) if fmt == B.SCALE_E4M3 else P.to_np_u16(kc.scales)
    for h in range(H):                                       # the filled part is the oracle's decode
        for c in range(4):
            sl = slice(c * L, min((c + 1) * L, filled))
            want = O.decode_unit(P.to_np_u16(kc.centroids[h, c]).reshape(S, K, 128),
                                 P.to_np_u8(kc.ids[h, sl]).reshape(-1, S).T, P.to_np_u8(kc.codes[h, sl]), sc[h, sl],
                                 Bg, bits=bits, scale_fmt=fmt)
            assert np.array_equal(P.to_np_u16(whole[h, sl]), want)
    for first, n in ((0, filled), (L, 2 * L + 77), (2 * L, 100), (3 * L, 77), (L, 0)):
        part = B.decode(kc, n_tokens=n, first_token=first)
        torch.cuda.synchronize()
        assert part.shape == (H, n, 128) and torch.equal(part, whole[:, first:first + n])
    with pytest.raises(B.QvgError):
        B.decode(kc, n_tokens=10, first_token=7)             # not on a chunk boundary


def test_streaming_cache_append_attend_decode():
    """The rollout object: a cache allocated for five chunks, three and a bit appended with
    centroid caching; every appended chunk equals a stand-alone encode from the same start, the
    attention over what has been appended so far equals the oracle's over the decoded prefix."""
    wl = CONFIGS["cfg2_window21"]
    heads, L, K, Bg, T = 2, 520, 64, 32, 2
    sc = B.StreamingCache(heads, 5 * L, L, K, Bg, T, warm_iters=2, cold_iters=4)
    sk, sv = synth.MixtureStream(wl, heads, 0, DEV), synth.MixtureStream(wl, heads, 1, DEV)
    q = synth.queries(wl, heads, 200, DEV)
    prev = None
    for c, n in enumerate((L, L, L, 133)):
        x = torch.cat([sk.next_chunk(n), sv.next_chunk(n)], 0)
        init = synth.cold_start_centroids(x, K) if c == 0 else None
        assert sc.append(x, init=init) == c
        start = init if c == 0 else prev
        alone = B.encode_chunk(x, start, Bg, T, 4 if c == 0 else 2)
        lo = c * L
        assert torch.equal(sc.cache.centroids[:, c], alone.centroids[:, 0])
        assert torch.equal(sc.cache.ids[:, lo:lo + n], alone.ids) and torch.equal(sc.cache.codes[:, lo:lo + n], alone.codes)
        assert torch.equal(sc.cache.scales[:, lo:lo + n], alone.scales)
        prev = sc.cache.centroids[:, c].clone()
        out, lse = sc.attend(q, want_lse=True)
        dec = sc.decode()
        torch.cuda.synchronize()
        assert dec.shape == (2 * heads, sc.n_tokens, 128)
        for h in range(heads):
            _check_against_oracle(q, out, lse, P.to_np_u16(dec[h]), P.to_np_u16(dec[heads + h]), h)
    assert sc.n_tokens == 3 * L + 133
    assert sc.stored_bytes() == B.compressed_bytes(B.make_params(2 * heads, K, Bg, T), L) * 3 + \
        B.compressed_bytes(B.make_params(2 * heads, K, Bg, T), 133)
    with pytest.raises(ValueError):
        sc.append(torch.zeros(2 * heads, 10, 128, dtype=torch.bfloat16, device=DEV))      # after a partial chunk
    assert torch.equal(sc.decode(first_chunk=2), sc.decode()[:, 2 * L:])


@pytest.mark.parametrize("L,T,Bg,S,bits,fmt,rope", [(520, 2, 32, 1, 2, B.SCALE_F16, False), (520, 4, 64, 1, 2, B.SCALE_F16, True),
                                                    (520, 3, 32, 1, 2, B.SCALE_F16, False), (260, 1, 16, 4, 2, B.SCALE_E4M3, False),
                                                    (516, 3, 64, 1, 4, B.SCALE_F16, True), (520, 1, 64, 2, 4, B.SCALE_E4M3, True)])
def test_attention_with_a_prefix_length_per_query(L, T, Bg, S, bits, fmt, rope):
    """qvg_attn_decode_causal: the queries of several chunks in one call, each seeing the chunks
    before its own (lengths on chunk boundaries), plus lengths inside a chunk, the whole cache,
    a single token, out-of-range values (clamped) and empty prefixes (a zero row, lse = -inf).  Every
    other query is checked against the oracle's attention over its own prefix.  Query blocks with short prefixes stop early: more than 256
    queries, sorted and unsorted."""
    H, K = 2, 64
    n_chunks, filled = 4, 3 * L + 77
    kc, vc = _filled_caches(H, L, n_chunks, filled, K, Bg, T, S, bits, fmt)
    wl = CONFIGS["cfg2_window21"]
    Nq = 300
    q = synth.queries(wl, H, Nq, DEV)
    g = torch.Generator().manual_seed(3)
    lens = torch.empty(Nq, dtype=torch.int64)
    lens[:100] = L                                   # queries of chunk 1 see chunk 0
    lens[100:200] = 2 * L                            # queries of chunk 2 see chunks 0-1
    lens[200:260] = torch.randint(1, filled + 1, (60,), generator=g)
    lens[260:] = torch.tensor([1, 2, 63, 64, 65, L - 1, L + 1, filled, filled - 1, filled + 50, 0, -5] + [3 * L] * 28)
    if T == 3:
        lens = lens[torch.randperm(Nq, generator=g)]              # unsorted: every block walks to its longest prefix
    table = _rope_table(filled).to(DEV) if rope else None
    out, lse = B.attn_decode(q, kc, vc, want_lse=True, n_kv=filled, k_rope=table,
                             q_kv_len=lens.to(torch.int32).to(DEV))
    khat, vhat = B.decode(kc, n_tokens=filled), B.decode(vc, n_tokens=filled)
    torch.cuda.synchronize()
    eff = lens.clamp(0, filled).numpy()
    assert (eff == 0).sum() == 2
    for h in range(H):
        kb = P.to_np_u16(khat[h])
        if rope:
            kb = O.rope_keys(kb, table.cpu().numpy().view(np.uint16))
        vb = P.to_np_u16(vhat[h])
        qb = bf16_bits(q[h])
        og, lg = P.to_np_u16(out[h]), lse[h].cpu().numpy()
        for n in np.unique(eff):
            rows = np.flatnonzero(eff == n)
            if n == 0:                                   # nothing cached before these queries
                assert (og[rows] == 0).all() and np.isneginf(lg[rows]).all()
                continue
            want, lse_w = O.attention(qb[rows], kb[:n], vb[:n], want_lse=True)
            ok, max_abs, worst = P.attn_tolerance_ok(og[rows], want)
            assert ok, f"head {h}, prefix {n}: max abs err {max_abs}, worst err/tol {worst}"
            assert np.abs(lg[rows] - lse_w).max() < 2e-3, (h, n)
    # every length = the whole cache: the result of the call without a length array (which may
    # run on the other kernel), within the tolerance of either
    full = torch.full((Nq,), filled, dtype=torch.int32, device=DEV)
    a = B.attn_decode(q, kc, vc, n_kv=filled, k_rope=table, q_kv_len=full)
    b = B.attn_decode(q, kc, vc, n_kv=filled, k_rope=table)
    torch.cuda.synchronize()
    for h in range(H):
        assert P.attn_tolerance_ok(P.to_np_u16(a[h]), bits_to_f32(P.to_np_u16(b[h])).astype(np.float64))[0]


@pytest.mark.parametrize("L,T,Bg,S,bits,fmt", [(520, 2, 32, 1, 2, B.SCALE_F16),      # staged kernel
                                               (516, 3, 64, 1, 2, B.SCALE_F16),      # general kernel, one table per chunk
                                               (260, 1, 16, 4, 2, B.SCALE_E4M3)])    # general kernel, four tables per chunk
def test_ids_beyond_the_table_read_its_last_row(L, T, Bg, S, bits, fmt):
    """A cache the library did not write may hold ids >= K (a byte holds up to 255, K is 64
    here).  Decode and attention must treat such an id as K - 1, the table's last row, and not
    read past the table: the outputs equal, bit for bit, those of the same cache with these ids
    set to K - 1, and that cache's attention agrees with the oracle."""
    H, K, Nq = 2, 64, 200
    filled = 2 * L + 77
    kc, vc = _filled_caches(H, L, 3, filled, K, Bg, T, S=S, bits=bits, fmt=fmt)
    q = synth.queries(CONFIGS["cfg2_window21"], H, Nq, DEV)
    g = torch.Generator(device="cpu").manual_seed(5)
    bad_k = (torch.rand(kc.ids.shape, generator=g) < 0.05).to(DEV)
    bad_v = (torch.rand(vc.ids.shape, generator=g) < 0.05).to(DEV)
    big = torch.randint(K, 256, kc.ids.shape, generator=g, dtype=torch.int32).to(torch.uint8).to(DEV)
    ids_k, ids_v = kc.ids.clone(), vc.ids.clone()

    kc.ids.copy_(torch.where(bad_k, torch.full_like(ids_k, K - 1), ids_k))
    vc.ids.copy_(torch.where(bad_v, torch.full_like(ids_v, K - 1), ids_v))
    khat, vhat = B.decode(kc, n_tokens=filled), B.decode(vc, n_tokens=filled)
    out, lse = B.attn_decode(q, kc, vc, want_lse=True, n_kv=filled)
    torch.cuda.synchronize()
    for h in range(H):
        _check_against_oracle(q, out, lse, P.to_np_u16(khat[h]), P.to_np_u16(vhat[h]), h)

    kc.ids.copy_(torch.where(bad_k, big, ids_k))
    vc.ids.copy_(torch.where(bad_v, big, ids_v))
    assert int((kc.ids >= K).sum()) > 0 and int((vc.ids >= K).sum()) > 0
    khat2, vhat2 = B.decode(kc, n_tokens=filled), B.decode(vc, n_tokens=filled)
    out2, lse2 = B.attn_decode(q, kc, vc, want_lse=True, n_kv=filled)
    torch.cuda.synchronize()
    assert torch.equal(khat2.view(torch.int16), khat.view(torch.int16))
    assert torch.equal(vhat2.view(torch.int16), vhat.view(torch.int16))
    assert torch.equal(out2.view(torch.int16), out.view(torch.int16))
    assert torch.equal(lse2, lse)


@pytest.mark.parametrize("S", [2, 4])
def test_id_arrays_at_any_byte_address(S):
    """Byte ids need no alignment (include/qvg.h asks for none): with several smoothing stages a
    token's S id bytes are read as one word when the array allows it and byte by byte otherwise.
    The same caches with their id arrays moved to an odd address must decode and attend to the
    same bits."""
    import dataclasses
    H, K, L, T, Bg, Nq = 2, 64, 260, 1, 16, 200
    filled = 2 * L + 31
    kc, vc = _filled_caches(H, L, 3, filled, K, Bg, T, S=S, bits=2, fmt=B.SCALE_E4M3)
    q = synth.queries(CONFIGS["cfg2_window21"], H, Nq, DEV)
    khat, vhat = B.decode(kc, n_tokens=filled), B.decode(vc, n_tokens=filled)
    out, lse = B.attn_decode(q, kc, vc, want_lse=True, n_kv=filled)

    def moved(c):
        buf = torch.zeros(c.ids.numel() + 1, dtype=torch.uint8, device=DEV)
        ids = buf[1:].view(c.ids.shape)
        ids.copy_(c.ids)
        assert ids.data_ptr() % 2 == 1 and ids.is_contiguous()
        return dataclasses.replace(c, ids=ids)
    kc2, vc2 = moved(kc), moved(vc)
    khat2, vhat2 = B.decode(kc2, n_tokens=filled), B.decode(vc2, n_tokens=filled)
    out2, lse2 = B.attn_decode(q, kc2, vc2, want_lse=True, n_kv=filled)
    torch.cuda.synchronize()
    assert torch.equal(khat2.view(torch.int16), khat.view(torch.int16))
    assert torch.equal(vhat2.view(torch.int16), vhat.view(torch.int16))
    assert torch.equal(out2.view(torch.int16), out.view(torch.int16))
    assert torch.equal(lse2, lse)
    for h in range(H):
        _check_against_oracle(q, out2, lse2, P.to_np_u16(khat2[h]), P.to_np_u16(vhat2[h]), h)


def test_empty_prefix_rows_merge_as_weightless():
    """A query that sees no cached token (prefix length 0) returns a zero row with lse = -inf; merged
    with the current chunk's own attention it must give exactly that second result."""
    H, K, L, T, Bg, Nq = 2, 64, 520, 2, 32, 70
    kc, vc = _filled_caches(H, L, 2, L + 40, K, Bg, T)
    q = synth.queries(CONFIGS["cfg2_window21"], H, Nq, DEV)
    lens = torch.zeros(Nq, dtype=torch.int32, device=DEV)
    lens[35:] = L
    out, lse = B.attn_decode(q, kc, vc, want_lse=True, n_kv=L + 40, q_kv_len=lens)
    g = torch.Generator(device=DEV).manual_seed(2)
    own = torch.randn(H, Nq, 128, generator=g, device=DEV).to(torch.bfloat16)
    own_lse = torch.randn(H, Nq, generator=g, device=DEV)
    merged, mlse = B.attn_merge(out, lse, own, own_lse, want_lse=True)
    torch.cuda.synchronize()
    assert (out[:, :35] == 0).all() and torch.isneginf(lse[:, :35]).all()
    assert torch.equal(merged[:, :35], own[:, :35]) and torch.equal(mlse[:, :35], own_lse[:, :35])
    assert not torch.equal(merged[:, 35:], own[:, 35:])


@pytest.mark.parametrize("L,T,Bg,S", [(520, 3, 32, 1),      # staged kernel
                                      (516, 2, 64, 1),      # general kernel
                                      (520, 1, 16, 2)])     # general kernel, two smoothing stages
def test_attention_fp32_output_meets_the_plain_bound(L, T, Bg, S):
    """qvg_attn_decode_f32: the result before the rounding to bf16, against the fp64 oracle at a
    plain 2e-3 maximum absolute error (no term relative to the output) on the configurations' own
    data; the bf16 entry point returns this result rounded to nearest even."""
    H, K, Nq = 2, 64, 300
    filled = 5 * L + 133
    kc, vc = _filled_caches(H, L, 6, filled, K, Bg, T, S=S)
    q = synth.queries(CONFIGS["cfg2_window21"], H, Nq, DEV)
    o32, lse = B.attn_decode(q, kc, vc, n_kv=filled, f32_out=True, want_lse=True)
    o16 = B.attn_decode(q, kc, vc, n_kv=filled)
    khat, vhat = B.decode(kc, n_tokens=filled), B.decode(vc, n_tokens=filled)
    torch.cuda.synchronize()
    assert o32.dtype == torch.float32
    assert torch.equal(o32.to(torch.bfloat16), o16)
    for h in range(H):
        want, lse_w = O.attention(bf16_bits(q[h]), P.to_np_u16(khat[h]), P.to_np_u16(vhat[h]), want_lse=True)
        err = np.abs(o32[h].cpu().numpy().astype(np.float64) - want).max()
        assert err <= 2e-3, f"head {h}: max abs err {err}"
        assert np.abs(lse[h].cpu().numpy() - lse_w).max() < 2e-3


def test_attention_with_values_of_magnitude_1e3():
    """The paper reports |V| up to about 1e3 (Sec. 3.2).  With values of that size the binary16
    probabilities (11 significant bits) move an output by up to 2^-10 * sum_j p_j |v_j| wherever the
    terms cancel, so the bound that holds is 2e-3 + 2^-8 |o| + 2^-10 E_p|v|; the fp32 result is
    checked against the last term alone, which is the kernel's own error."""
    wl = CONFIGS["cfg2_window21"]
    H, K, L, T, Bg, Nq = 2, 64, 520, 2, 64, 200
    filled = 3 * L + 77
    caches = []
    for kv, gain in ((0, 10.0), (1, 120.0)):             # max |K| ~ 1e2, max |V| ~ 1e3
        st = synth.MixtureStream(wl, H, kv, DEV)
        cache = B.alloc_cache(H, 4 * L, L, K, Bg, T, 128, DEV)
        for t in (cache.centroids, cache.ids, cache.codes, cache.scales):
            t.zero_()
        c = 0
        while c * L < filled:
            x = (st.next_chunk(min(L, filled - c * L)).float() * gain).to(torch.bfloat16)
            B.encode_chunk(x, synth.cold_start_centroids(x, K), Bg, T, 2, cache=cache, chunk_index=c)
            c += 1
        caches.append(cache)
    kc, vc = caches
    q = (synth.queries(wl, H, Nq, DEV).float() * 0.1).to(torch.bfloat16)      # keeps the soft-max from collapsing onto one key
    o16 = B.attn_decode(q, kc, vc, n_kv=filled)
    o32 = B.attn_decode(q, kc, vc, n_kv=filled, f32_out=True)
    khat, vhat = B.decode(kc, n_tokens=filled), B.decode(vc, n_tokens=filled)
    torch.cuda.synchronize()
    assert float(vhat.float().abs().max()) > 500.0
    for h in range(H):
        qb, kb, vb = bf16_bits(q[h]), P.to_np_u16(khat[h]), P.to_np_u16(vhat[h])
        want = O.attention(qb, kb, vb)
        ok, max_abs, worst = P.attn_tolerance_wide_range_ok(P.to_np_u16(o16[h]), want, qb, kb, vb)
        assert ok, f"head {h}: max abs err {max_abs}, worst err/tol {worst}"
        qf, kf, vf = (bits_to_f32(t).astype(np.float64) for t in (qb, kb, vb))
        s = (qf @ kf.T) / np.sqrt(128.0)
        pr = np.exp(s - s.max(1, keepdims=True)); pr /= pr.sum(1, keepdims=True)
        spread = pr @ np.abs(vf)
        err = np.abs(o32[h].cpu().numpy().astype(np.float64) - want)
        assert (err <= 1e-4 + 2.0 ** -10 * spread).all(), f"head {h}: worst {(err / (1e-4 + 2.0 ** -10 * spread)).max()}"


@pytest.mark.parametrize("L,T,Bg", [(100, 1, 128), (100, 3, 128), (35, 1, 32)])
def test_unit_scale_arrays_off_16_byte_boundaries(L, T, Bg):
    """Several units whose binary16 scale arrays do not start on 16-byte boundaries (capacity x T x
    d/B x 2 bytes is no multiple of 16): the wide-load kernel must not be chosen; every unit
    against the oracle."""
    H, K, Nq = 3, 16, 70
    assert (L * T * (128 // Bg) * 2) % 16 != 0
    kc, vc = _filled_caches(H, L, 1, L, K, Bg, T)
    q = synth.queries(CONFIGS["cfg2_window21"], H, Nq, DEV)
    out, lse = B.attn_decode(q, kc, vc, want_lse=True)
    khat, vhat = B.decode(kc), B.decode(vc)
    torch.cuda.synchronize()
    for h in range(H):
        _check_against_oracle(q, out, lse, P.to_np_u16(khat[h]), P.to_np_u16(vhat[h]), h)
