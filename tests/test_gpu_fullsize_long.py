"""Full-size parity at the two largest configurations, in the launches bench.py times: one layer of
cfg5_long (24 units, 160 chunks of 4680 tokens = 748800 cached tokens per unit, K = 256, T = 4,
4680 queries) and one layer of cfg4_dit_large (80 units, 10 chunks of 10800 tokens, K = 128, T = 3,
B = 32, 10800 queries).  The cache is filled chunk by chunk with warm starts exactly as the
benchmark does, one benchmark step is run, and its outputs are compared with the oracle on
sampled units, chunks and queries that the oracle can afford: the last chunk's encode, the
decode of whole units (chunk 159 of unit 23 among them: the largest token offsets and the last
centroid table), and the attention of sampled queries over ALL cached tokens."""
import numpy as np
import pytest
import torch

from oracle import qvg_oracle as O
from paper_2602_02958_amd import workload
from paper_2602_02958_amd.configs import CONFIGS
from conftest import bf16_bits
import parity_util as P

pytestmark = pytest.mark.gpu


def _stepped(name):
    wl = CONFIGS[name]
    s = workload.build_streaming(wl, keep_inputs=(wl.n_chunks - 1,))
    workload.step(s)
    torch.cuda.synchronize()
    return wl, s


@pytest.fixture(scope="module")
def cfg5():
    out = _stepped("cfg5_long")
    yield out
    del out
    torch.cuda.empty_cache()


@pytest.fixture(scope="module")
def cfg4():
    out = _stepped("cfg4_dit_large")
    yield out
    del out
    torch.cuda.empty_cache()


def _oracle_decode_unit(wl, s, u, chunks=None):
    """Oracle decode of unit u (all chunks, or the listed ones) from the GPU's stored arrays; the
    chunks go through the batched driver as independent units, one table each."""
    L = wl.chunk
    chunks = list(range(wl.n_chunks)) if chunks is None else list(chunks)
    cent = P.to_np_u16(s.cache.centroids[u])[chunks][:, None]                    # [C, 1, K, d]
    ids = np.stack([P.to_np_u8(s.cache.ids[u, c * L:(c + 1) * L]) for c in chunks])[:, None]
    codes = np.stack([P.to_np_u8(s.cache.codes[u, c * L:(c + 1) * L]) for c in chunks])
    scales = np.stack([P.to_np_u16(s.cache.scales[u, c * L:(c + 1) * L]) for c in chunks])
    return O.decode_batch(cent, ids, codes, scales, wl.group_size)              # [C, L, d]


def _check_last_chunk_encode(wl, s, units, full_fit_unit):
    c = s.new_index
    lo = c * wl.chunk
    x = s.kept_chunks[c]
    for u in units:
        ties = P.check_encoded_unit(bf16_bits(x[u]), P.to_np_u16(s.cache.centroids[u, c]),
                                    P.gpu_unit(s.cache, u, lo, lo + x.shape[1]), wl.group_size, wl.n_stages)
        assert ties <= 1
    u = full_fit_unit                                # the whole warm-started Lloyd fit of one unit
    ref = O.encode_batch(bf16_bits(x[u:u + 1]), P.to_np_u16(s.init_new[u:u + 1]), wl.n_clusters, wl.group_size,
                         wl.n_stages, wl.kmeans_iters_warm)
    assert np.array_equal(P.to_np_u16(s.cache.centroids[u, c]), ref["cent"][0, 0])
    assert np.array_equal(P.to_np_u8(s.cache.ids[u, lo:lo + x.shape[1]]), ref["ids"][0, 0])
    assert np.array_equal(P.to_np_u8(s.cache.codes[u, lo:lo + x.shape[1]]), ref["codes"][0])
    assert np.array_equal(P.to_np_u16(s.cache.scales[u, lo:lo + x.shape[1]]), ref["scales"][0])


def _check_attention(wl, s, heads, n_sample, seed):
    """Sampled queries (first, last, random) of the given heads over the whole cache; K_hat and
    V_hat are the oracle's decode of the GPU's stored arrays, which must also equal the GPU decode."""
    rng = np.random.default_rng(seed)
    n = wl.tokens_per_layer
    for head in heads:
        kv = []
        for u in (head, wl.heads + head):
            want = _oracle_decode_unit(wl, s, u).reshape(n, wl.head_dim)
            assert np.array_equal(P.to_np_u16(s.decoded[u]), want), f"decode of unit {u}"
            kv.append(want)
        qi = np.sort(rng.choice(wl.n_queries, n_sample, replace=False))
        qi[0], qi[-1] = 0, wl.n_queries - 1
        want = O.attention(bf16_bits(s.q[head])[qi], kv[0], kv[1])
        ok, max_abs, worst = P.attn_tolerance_ok(P.to_np_u16(s.attn_out[head])[qi], want)
        assert ok, f"head {head}: max abs err {max_abs}, worst err/tol {worst}"


# ------------------------------------------------------------------ cfg5: 748800 tokens per unit
def test_cfg5_layer_last_chunk_encode(cfg5):
    wl, s = cfg5
    assert s.new_index == 159 and s.cache.ids.shape == (24, 748800)
    _check_last_chunk_encode(wl, s, units=(0, 23), full_fit_unit=12)


def test_cfg5_layer_decode_sampled_chunks(cfg5):
    wl, s = cfg5
    L = wl.chunk
    for u, chunks in ((23, (159, 158, 0)), (0, (0, 1, 159)), (11, (80,)), (12, (157, 33))):
        want = _oracle_decode_unit(wl, s, u, chunks)
        for i, c in enumerate(chunks):
            assert np.array_equal(P.to_np_u16(s.decoded[u, c * L:(c + 1) * L]), want[i]), (u, c)


def test_cfg5_layer_attention_over_the_whole_cache(cfg5):
    wl, s = cfg5
    _check_attention(wl, s, heads=(0, 11), n_sample=16, seed=5)


# ------------------------------------------------------------------ cfg4: 80 units x 108000 tokens
def test_cfg4_layer_last_chunk_encode(cfg4):
    wl, s = cfg4
    assert s.new_index == 9 and s.cache.ids.shape == (80, 108000)
    _check_last_chunk_encode(wl, s, units=(0, 79), full_fit_unit=41)


def test_cfg4_layer_decode_sampled_chunks(cfg4):
    wl, s = cfg4
    L = wl.chunk
    for u, chunks in ((79, (9, 0)), (0, (0, 9)), (40, (5,))):
        want = _oracle_decode_unit(wl, s, u, chunks)
        for i, c in enumerate(chunks):
            assert np.array_equal(P.to_np_u16(s.decoded[u, c * L:(c + 1) * L]), want[i]), (u, c)


def test_cfg4_layer_attention_over_the_whole_cache(cfg4):
    wl, s = cfg4
    _check_attention(wl, s, heads=(0, 39), n_sample=16, seed=4)
