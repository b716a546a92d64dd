"""Full-size parity in the launch configuration bench.py times (cfg2_window21: 24 units, a
37440-token cache in 8 chunks, 4680 queries): the outputs of one benchmark step are compared
with the oracle on sampled units, tokens and queries that the oracle can afford."""
import numpy as np
import pytest
import torch

from oracle import qvg_oracle as O
from paper_2602_02958_amd import binding as B
from paper_2602_02958_amd import workload
from paper_2602_02958_amd.configs import CONFIGS
from conftest import bf16_bits, bits_to_f32
import parity_util as P

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def stepped():
    wl = CONFIGS["cfg2_window21"]
    n_chunks = wl.n_chunks
    s = workload.build_streaming(wl, keep_inputs=(n_chunks - 1,))
    workload.step(s)
    torch.cuda.synchronize()
    return wl, s


def test_step_encode_matches_oracle_on_sampled_units(stepped):
    wl, s = stepped
    c = s.new_index
    lo = c * wl.chunk
    x = s.kept_chunks[c]
    units = [0, 7, 12, 23]                       # K heads 0 and 7, V heads 0 and 11
    for u in units:
        xb = bf16_bits(x[u])
        cent_g = P.to_np_u16(s.cache.centroids[u, c])
        # (1) stored ids / codes / scales are the oracle's for the GPU's own final centroids
        ties = P.check_encoded_unit(xb, cent_g, P.gpu_unit(s.cache, u, lo, lo + x.shape[1]),
                                    wl.group_size, wl.n_stages)
        assert ties <= 1
    # (2) the whole warm-started Lloyd fit equals the oracle's, unit by unit
    sel = [0, 23]
    init = P.to_np_u16(s.init_new[sel])
    ref = O.encode_batch(bf16_bits(x[sel]), init, wl.n_clusters, wl.group_size, wl.n_stages,
                         wl.kmeans_iters_warm)
    assert np.array_equal(P.to_np_u16(s.cache.centroids[sel, c]), ref["cent"][:, 0])
    assert np.array_equal(P.to_np_u8(s.cache.ids[sel, lo:lo + x.shape[1]]), ref["ids"][:, 0])
    assert np.array_equal(P.to_np_u8(s.cache.codes[sel, lo:lo + x.shape[1]]), ref["codes"])


def test_step_decode_bit_exact_on_sampled_units(stepped):
    wl, s = stepped
    for u in (1, 13, 22):
        want = np.concatenate([
            O.decode_unit(P.to_np_u16(s.cache.centroids[u, c]),
                          P.to_np_u8(s.cache.ids[u, c * wl.chunk:(c + 1) * wl.chunk]),
                          P.to_np_u8(s.cache.codes[u, c * wl.chunk:(c + 1) * wl.chunk]),
                          P.to_np_u16(s.cache.scales[u, c * wl.chunk:(c + 1) * wl.chunk]), wl.group_size)
            for c in range(wl.n_chunks)])
        assert np.array_equal(P.to_np_u16(s.decoded[u]), want)


def test_step_attention_on_sampled_queries(stepped):
    wl, s = stepped
    rng = np.random.default_rng(3)
    for head in (0, 11):
        k_hat = P.to_np_u16(s.decoded[head])                 # verified bit-exact by the test above
        v_hat = P.to_np_u16(s.decoded[wl.heads + head])
        qi = np.sort(rng.choice(wl.n_queries, 24, replace=False))
        qi[0], qi[-1] = 0, wl.n_queries - 1                  # first and last (ragged tail of the last block)
        want = O.attention(bf16_bits(s.q[head])[qi], k_hat, v_hat)
        ok, max_abs, worst = P.attn_tolerance_ok(P.to_np_u16(s.attn_out[head])[qi], want)
        assert ok, f"head {head}: max abs err {max_abs}, worst err/tol {worst}"


def test_step_is_deterministic(stepped):
    wl, s = stepped
    first = [P.to_np_u16(s.cache.centroids).copy(), P.to_np_u8(s.cache.codes).copy(),
             P.to_np_u16(s.decoded[:4]).copy(), P.to_np_u16(s.attn_out).copy()]
    workload.step(s)
    torch.cuda.synchronize()
    again = [P.to_np_u16(s.cache.centroids), P.to_np_u8(s.cache.codes), P.to_np_u16(s.decoded[:4]),
             P.to_np_u16(s.attn_out)]
    for a, b in zip(first, again):
        assert np.array_equal(a, b)


def test_cfg3_chunk_encode_decode_sampled():
    """One chunk at the cfg3 shape (K = 256, T = 2, B = 64), 48 units in one call."""
    wl = CONFIGS["cfg3_dit_small"]
    from paper_2602_02958_amd import synth
    units = 48
    x = synth.MixtureStream(wl, units, 0, "cuda").next_chunk(wl.chunk)
    init = synth.cold_start_centroids(x, wl.n_clusters)
    enc = B.encode_chunk(x, init, wl.group_size, wl.n_stages, 2)
    dec = B.decode(enc)
    torch.cuda.synchronize()
    for u in (0, 47):
        xb = bf16_bits(x[u])
        cent_g = P.to_np_u16(enc.centroids[u, 0])
        ties = P.check_encoded_unit(xb, cent_g, P.gpu_unit(enc, u), wl.group_size, wl.n_stages)
        assert ties <= 1
        want = O.decode_unit(cent_g, P.to_np_u8(enc.ids[u]), P.to_np_u8(enc.codes[u]),
                             P.to_np_u16(enc.scales[u]), wl.group_size)
        assert np.array_equal(P.to_np_u16(dec[u]), want)
        # reconstruction error within the staged-quantization bound (Eq. 3 applied T times)
        xf, df = bits_to_f32(xb).astype(np.float64), bits_to_f32(want).astype(np.float64)
        r0 = xf - bits_to_f32(cent_g)[P.to_np_u8(enc.ids[u])]
        gmax = np.repeat(np.abs(r0).reshape(-1, 2, 64).max(-1), 64, axis=1)
        # each stage halves the group's largest residual; the bf16 output adds half an ulp (2^-8 relative)
        assert (np.abs(xf - df) <= gmax / 4 * (1 + 2.0 ** -9) + 2.0 ** -8 * np.maximum(np.abs(xf), np.abs(df)) + 1e-6).all()
    # one unit end to end against the oracle's own Lloyd iterations
    ref = O.encode_batch(bf16_bits(x[5:6]), bf16_bits(init[5:6]), wl.n_clusters, wl.group_size, wl.n_stages, 2)
    assert np.array_equal(P.to_np_u16(enc.centroids[5, 0]), ref["cent"][0, 0])
    assert np.array_equal(P.to_np_u8(enc.ids[5]), ref["ids"][0, 0])
    assert np.array_equal(P.to_np_u8(enc.codes[5]), ref["codes"][0])


def test_cfg3_all_layers_chunk_in_bench_launch_shape():
    """The large-shape supplement of bench.py: one 4680-token chunk of all 30 layers of cfg3
    (720 units in one call, which makes the encoder take several 256-token steps per workgroup),
    warm-started Lloyd iterations included; sampled units against the oracle."""
    wl = CONFIGS["cfg3_dit_small"]
    from paper_2602_02958_amd import synth
    units = 2 * wl.layers * wl.heads
    x = synth.MixtureStream(wl, units, 0, "cuda").next_chunk(wl.chunk)
    init = synth.cold_start_centroids(x, wl.n_clusters)
    enc = B.encode_chunk(x, init, wl.group_size, wl.n_stages, 2)
    dec = B.decode(enc)
    torch.cuda.synchronize()
    for u in (0, 359, 719):
        xb = bf16_bits(x[u])
        cent_g = P.to_np_u16(enc.centroids[u, 0])
        ties = P.check_encoded_unit(xb, cent_g, P.gpu_unit(enc, u), wl.group_size, wl.n_stages)
        assert ties <= 1
        want = O.decode_unit(cent_g, P.to_np_u8(enc.ids[u]), P.to_np_u8(enc.codes[u]),
                             P.to_np_u16(enc.scales[u]), wl.group_size)
        assert np.array_equal(P.to_np_u16(dec[u]), want)
    sel = [1, 718]
    ref = O.encode_batch(bf16_bits(x[sel]), bf16_bits(init[sel]), wl.n_clusters, wl.group_size, wl.n_stages, 2)
    assert np.array_equal(P.to_np_u16(enc.centroids[sel, 0]), ref["cent"][:, 0])
    assert np.array_equal(P.to_np_u8(enc.ids[sel]), ref["ids"][:, 0])
    assert np.array_equal(P.to_np_u8(enc.codes[sel]), ref["codes"])
    assert np.array_equal(P.to_np_u16(enc.scales[sel]), ref["scales"])


def test_cfg3_full_cache_decode_sampled():
    """Decode of a 126360-token cache (27 chunks) of 72 units, the launch bench.py times for the
    decode roofline: random valid storage, sampled (unit, chunk) pairs against the oracle."""
    wl = CONFIGS["cfg3_dit_small"]
    units, n = 2 * 3 * wl.heads, wl.tokens_per_layer
    big = B.alloc_cache(units, n, wl.chunk, wl.n_clusters, wl.group_size, wl.n_stages, wl.head_dim, "cuda")
    g = torch.Generator(device="cuda"); g.manual_seed(5)
    big.ids.copy_(torch.randint(0, wl.n_clusters, big.ids.shape, generator=g, device="cuda", dtype=torch.uint8))
    f = torch.randint(0, 3, big.codes.shape + (4,), generator=g, device="cuda", dtype=torch.uint8)
    two = torch.tensor([0, 1, 3], dtype=torch.uint8, device="cuda")[f.long()]     # levels 0, +1, -1
    big.codes.copy_(two[..., 0] | (two[..., 1] << 2) | (two[..., 2] << 4) | (two[..., 3] << 6)); del f, two
    big.scales.copy_(torch.rand(big.scales.shape, generator=g, device="cuda").to(torch.float16))
    big.centroids.copy_(torch.randn(big.centroids.shape, generator=g, device="cuda").to(torch.bfloat16))
    out = B.decode(big)
    torch.cuda.synchronize()
    L = wl.chunk
    for u, c in ((0, 0), (35, 13), (71, 26)):
        sl = slice(c * L, min((c + 1) * L, n))
        want = O.decode_unit(P.to_np_u16(big.centroids[u, c]), P.to_np_u8(big.ids[u, sl]),
                             P.to_np_u8(big.codes[u, sl]), P.to_np_u16(big.scales[u, sl]), wl.group_size)
        assert np.array_equal(P.to_np_u16(out[u, sl]), want)


def test_cfg4_layer_chunk_heavy_tails():
    """One 10800-token chunk of one cfg4 layer (40 K heads + 40 V heads, K = 128, T = 3, B = 32,
    Student-t outlier channels): encode with Lloyd iterations, decode, attention of 300 queries,
    sampled units against the oracle."""
    wl = CONFIGS["cfg4_dit_large"]
    from paper_2602_02958_amd import synth
    heads = wl.heads
    xk = synth.MixtureStream(wl, heads, 0, "cuda").next_chunk(wl.chunk)
    xv = synth.MixtureStream(wl, heads, 1, "cuda").next_chunk(wl.chunk)
    x = torch.cat([xk, xv], 0)
    init = synth.cold_start_centroids(x, wl.n_clusters)
    enc = B.encode_chunk(x, init, wl.group_size, wl.n_stages, 2)
    dec = B.decode(enc)
    q = synth.queries(wl, heads, 300, "cuda")
    k = B.Encoded(enc.centroids[:heads], enc.ids[:heads], enc.codes[:heads], enc.scales[:heads], enc.chunk_len)
    v = B.Encoded(enc.centroids[heads:], enc.ids[heads:], enc.codes[heads:], enc.scales[heads:], enc.chunk_len)
    out = B.attn_decode(q, k, v)
    torch.cuda.synchronize()
    for u in (3, 77):
        xb = bf16_bits(x[u])
        cent_g = P.to_np_u16(enc.centroids[u, 0])
        assert P.check_encoded_unit(xb, cent_g, P.gpu_unit(enc, u), wl.group_size, wl.n_stages) <= 1
        want = O.decode_unit(cent_g, P.to_np_u8(enc.ids[u]), P.to_np_u8(enc.codes[u]),
                             P.to_np_u16(enc.scales[u]), wl.group_size)
        assert np.array_equal(P.to_np_u16(dec[u]), want)
    ref = O.encode_batch(bf16_bits(x[40:41]), bf16_bits(init[40:41]), wl.n_clusters, wl.group_size, wl.n_stages, 2)
    assert np.array_equal(P.to_np_u16(enc.centroids[40, 0]), ref["cent"][0, 0])
    assert np.array_equal(P.to_np_u8(enc.ids[40]), ref["ids"][0, 0])
    assert np.array_equal(P.to_np_u8(enc.codes[40]), ref["codes"][0])
    for h in (0, 39):
        want = O.attention(bf16_bits(q[h]), P.to_np_u16(dec[h]), P.to_np_u16(dec[heads + h]))
        ok, max_abs, worst = P.attn_tolerance_ok(P.to_np_u16(out[h]), want)
        assert ok, f"head {h}: max abs err {max_abs}, worst err/tol {worst}"


def test_cfg5_drifting_stream_four_rounds():
    """cfg5 (K = 256, T = 4, B = 64, mixture centres drifting from chunk to chunk): three chunks
    appended with warm starts; the last one against the oracle for a sampled unit."""
    wl = CONFIGS["cfg5_long"]
    from paper_2602_02958_amd import synth
    units, L = 2 * wl.heads, wl.chunk
    sk, sv = synth.MixtureStream(wl, wl.heads, 0, "cuda"), synth.MixtureStream(wl, wl.heads, 1, "cuda")
    cache = B.alloc_cache(units, 3 * L, L, wl.n_clusters, wl.group_size, wl.n_stages, wl.head_dim, "cuda")
    x = init = None
    for c in range(3):
        x = torch.cat([sk.next_chunk(L), sv.next_chunk(L)], 0)
        init = synth.cold_start_centroids(x, wl.n_clusters) if c == 0 else cache.centroids[:, c - 1].contiguous()
        B.encode_chunk(x, init, wl.group_size, wl.n_stages, wl.kmeans_iters_cold if c == 0 else wl.kmeans_iters_warm,
                       cache=cache, chunk_index=c)
    dec = B.decode(cache)
    torch.cuda.synchronize()
    u = 17
    ref = O.encode_batch(bf16_bits(x[u:u + 1]), bf16_bits(init[u:u + 1]), wl.n_clusters, wl.group_size,
                         wl.n_stages, wl.kmeans_iters_warm)
    sl = slice(2 * L, 3 * L)
    assert np.array_equal(P.to_np_u16(cache.centroids[u, 2]), ref["cent"][0, 0])
    assert np.array_equal(P.to_np_u8(cache.ids[u, sl]), ref["ids"][0, 0])
    assert np.array_equal(P.to_np_u8(cache.codes[u, sl]), ref["codes"][0])
    assert np.array_equal(P.to_np_u16(cache.scales[u, sl]), ref["scales"][0])
    want = O.decode_batch(ref["cent"], ref["ids"], ref["codes"], ref["scales"], wl.group_size)
    assert np.array_equal(P.to_np_u16(dec[u, sl]), want[0])


@pytest.mark.parametrize("S,Bg,bits,with_rope", [(1, 64, 2, True), (4, 16, 4, False)])
def test_paper_presets_on_the_cfg2_window_sampled(S, Bg, bits, with_rope):
    """The paper's presets (one round, K = 256, E4M3 scales; QVG INT2 and QVG-Pro INT4) at the size
    and in the launches bench.py's `paper_presets` times: 24 units, 8 chunks of 4680 tokens, 4680
    queries.  Sampled: the last chunk's encode on two units (whole Lloyd fit), the decode of two
    units, the attention of 24 queries of two heads over the full cache (with the rotary embedding
    of the decoded keys for the first preset)."""
    from paper_2602_02958_amd import synth
    wl = CONFIGS["cfg2_window21"]
    heads, units, L, n, K = wl.heads, 2 * wl.heads, wl.chunk, wl.tokens_per_layer, 256
    cache = B.alloc_cache(units, n, L, K, Bg, 1, 128, "cuda", n_smooth=S, bits=bits, scale_format=B.SCALE_E4M3)
    sk, sv = synth.MixtureStream(wl, heads, 0, "cuda"), synth.MixtureStream(wl, heads, 1, "cuda")
    x = init = None
    for c in range(wl.n_chunks):
        x = torch.cat([sk.next_chunk(L), sv.next_chunk(L)], 0)
        if c > 0:
            init = cache.centroids[:, c - 1].contiguous()
        elif S > 1:
            init = torch.stack([synth.cold_start_centroids(x, K, seed=st) for st in range(S)], 1)
        else:
            init = synth.cold_start_centroids(x, K, seed=0)
        B.encode_chunk(x, init, Bg, 1, 10 if c == 0 else 3, cache=cache, chunk_index=c)
    dec = B.decode(cache)
    q = synth.queries(wl, heads, wl.n_queries, "cuda")
    rope = bench_rope(n) if with_rope else None
    k = B.Encoded(cache.centroids[:heads], cache.ids[:heads], cache.codes[:heads], cache.scales[:heads], L, S)
    v = B.Encoded(cache.centroids[heads:], cache.ids[heads:], cache.codes[heads:], cache.scales[heads:], L, S)
    out = B.attn_decode(q, k, v, k_rope=rope)
    torch.cuda.synchronize()
    c = wl.n_chunks - 1
    lo = c * L
    sel = [3, 20]
    ref = O.encode_batch(bf16_bits(x[sel]), P.to_np_u16(init[sel]), K, Bg, 1, 3, S=S, bits=bits, scale_fmt=1)
    assert np.array_equal(P.to_np_u16(cache.centroids[sel, c]).reshape(2, S, K, 128), ref["cent"])
    assert np.array_equal(P.to_np_u8(cache.ids[sel, lo:]).reshape(2, L, S).transpose(0, 2, 1), ref["ids"])
    assert np.array_equal(P.to_np_u8(cache.codes[sel, lo:]), ref["codes"])
    assert np.array_equal(P.to_np_u8(cache.scales[sel, lo:]).astype(np.uint16), ref["scales"])
    for u in (0, heads):                                     # K of head 0, V of head 0: the whole cache
        want = np.concatenate([
            O.decode_unit(P.to_np_u16(cache.centroids[u, cc]).reshape(S, K, 128),
                          P.to_np_u8(cache.ids[u, cc * L:(cc + 1) * L]).reshape(L, S).T,
                          P.to_np_u8(cache.codes[u, cc * L:(cc + 1) * L]),
                          P.to_np_u8(cache.scales[u, cc * L:(cc + 1) * L]).astype(np.uint16), Bg, bits=bits, scale_fmt=1)
            for cc in range(wl.n_chunks)])
        assert np.array_equal(P.to_np_u16(dec[u]), want)
    rng = np.random.default_rng(4)
    qi = np.sort(rng.choice(wl.n_queries, 24, replace=False))
    qi[0], qi[-1] = 0, wl.n_queries - 1
    k_hat = P.to_np_u16(dec[0])
    if with_rope:
        k_hat = O.rope_keys(k_hat, rope.cpu().view(torch.int16).numpy().view(np.uint16))
    want = O.attention(bf16_bits(q[0])[qi], k_hat, P.to_np_u16(dec[heads]))
    ok, max_abs, worst = P.attn_tolerance_ok(P.to_np_u16(out[0])[qi], want)
    assert ok, f"max abs err {max_abs}, worst err/tol {worst}"


def bench_rope(n, d=128):
    pos = torch.arange(n, dtype=torch.float64, device="cuda")
    freq = 10000.0 ** (-torch.arange(d // 2, dtype=torch.float64, device="cuda") / (d // 2))
    ang = pos[:, None] * freq[None]
    return torch.stack([ang.cos(), ang.sin()], -1).to(torch.float16).contiguous()
