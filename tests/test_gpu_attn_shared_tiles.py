"""Attention with a workspace: every tile is decoded once per unit into the workspace and shared by
all query blocks (a slab of chunks at a time, the queries' soft-max state carried between slabs).
The arithmetic per tile is that of the fused kernels, so the result must equal theirs bit for bit
and meet the same bound against the oracle."""
import numpy as np
import pytest
import torch

from oracle import qvg_oracle as O
from paper_2602_02958_amd import binding as B
from paper_2602_02958_amd import synth
from paper_2602_02958_amd.configs import CONFIGS
from conftest import bf16_bits
import parity_util as P
from test_gpu_attn_integration import _filled_caches, _rope_table, _check_against_oracle

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _ws(H, Nq, L, n_chunks):
    return B.attn_workspace(H, Nq, L, n_chunks, DEV)


@pytest.mark.parametrize("L,T,Bg,S,bits,fmt,K", [
    (200, 3, 64, 1, 2, B.SCALE_F16, 32),      # chunks of 3 tiles + 8 tokens
    (520, 4, 64, 1, 2, B.SCALE_F16, 256),
    (516, 2, 32, 1, 2, B.SCALE_F16, 64),
    (520, 1, 64, 1, 2, B.SCALE_E4M3, 64),     # the paper's QVG format
    (520, 1, 16, 4, 2, B.SCALE_E4M3, 64),     # QVG-Pro: four smoothing stages
    (520, 1, 16, 2, 4, B.SCALE_E4M3, 64),
    (520, 1, 64, 1, 4, B.SCALE_E4M3, 64),     # INT4
    (136, 5, 128, 1, 2, B.SCALE_F16, 16),     # run-time round count
    (64, 2, 64, 1, 2, B.SCALE_F16, 16),       # a chunk is exactly one tile
    (40, 2, 64, 1, 2, B.SCALE_F16, 16),       # every tile is a partial one
])
def test_shared_tiles_equal_the_fused_kernels(L, T, Bg, S, bits, fmt, K):
    H, Nq = 3, 600                             # three query blocks per unit, the last one partial
    filled = (2 * L + 133) if L >= 136 else (9 * L + 17)    # the last chunk is short
    kc, vc = _filled_caches(H, L, -(-filled // L) + 1, filled, K, Bg, T, S=S, bits=bits, fmt=fmt)
    q = synth.queries(CONFIGS["cfg2_window21"], H, Nq, DEV)
    khat, vhat = B.decode(kc), B.decode(vc)
    for n_kv in (filled, 2 * L, L + 7, 64, 1):
        fused, lse_f = B.attn_decode(q, kc, vc, want_lse=True, n_kv=n_kv)
        n_chunks = -(-n_kv // L)
        # one slab; one chunk per slab (state carried n_chunks - 1 times); slabs of two and of three chunks
        for slab_chunks in sorted({n_chunks, 1, min(2, n_chunks), min(3, n_chunks)}):
            ws = _ws(H, Nq, L, slab_chunks)
            out, lse = B.attn_decode(q, kc, vc, want_lse=True, n_kv=n_kv, workspace=ws)
            out2, lse2 = B.attn_decode(q, kc, vc, want_lse=True, n_kv=n_kv, workspace=ws)   # straight after, same workspace
            torch.cuda.synchronize()
            assert torch.equal(out, fused), (n_kv, slab_chunks)
            assert torch.equal(lse, lse_f), (n_kv, slab_chunks)
            assert torch.equal(out2, fused) and torch.equal(lse2, lse_f), (n_kv, slab_chunks)
        for h in range(H):
            _check_against_oracle(q, out, lse, P.to_np_u16(khat[h, :n_kv]), P.to_np_u16(vhat[h, :n_kv]), h)


def test_shared_tiles_with_rotary_embedding():
    H, L, K, Bg, T, Nq = 2, 520, 64, 32, 2, 700
    filled = 2 * L + 133
    kc, vc = _filled_caches(H, L, 3, filled, K, Bg, T)
    q = synth.queries(CONFIGS["cfg2_window21"], H, Nq, DEV)
    rope = _rope_table(filled, offset=3).to(DEV)
    fused = B.attn_decode(q, kc, vc, n_kv=filled, k_rope=rope)
    out, lse = B.attn_decode(q, kc, vc, want_lse=True, n_kv=filled, k_rope=rope, workspace=_ws(H, Nq, L, 2))
    torch.cuda.synchronize()
    assert torch.equal(out, fused)
    khat, vhat = B.decode(kc), B.decode(vc)
    rope_bits = rope.cpu().view(torch.int16).numpy().view(np.uint16)
    for h in range(H):
        krot = O.rope_keys(P.to_np_u16(khat[h, :filled]), rope_bits)
        _check_against_oracle(q, out, lse, krot, P.to_np_u16(vhat[h, :filled]), h)


def test_a_workspace_too_small_for_one_chunk_is_ignored():
    H, L, K, Bg, T, Nq = 2, 520, 64, 64, 2, 600
    kc, vc = _filled_caches(H, L, 2, 2 * L, K, Bg, T)
    q = synth.queries(CONFIGS["cfg2_window21"], H, Nq, DEV)
    fused = B.attn_decode(q, kc, vc)
    small = torch.empty(4096, dtype=torch.uint8, device=DEV)
    out = B.attn_decode(q, kc, vc, workspace=small)
    torch.cuda.synchronize()
    assert torch.equal(out, fused)


def test_a_misaligned_workspace_is_refused():
    H, L, K, Bg, T, Nq = 2, 520, 64, 64, 2, 600
    kc, vc = _filled_caches(H, L, 2, 2 * L, K, Bg, T)
    q = synth.queries(CONFIGS["cfg2_window21"], H, Nq, DEV)
    ws = _ws(H, Nq, L, 2)
    odd = torch.empty(ws.numel() + 16, dtype=torch.uint8, device=DEV)[4:]
    assert odd.data_ptr() % 16 != 0
    with pytest.raises(B.QvgError) as e:
        B.attn_decode(q, kc, vc, workspace=odd)
    assert e.value.status == -5


def test_shared_tiles_16_bit_ids():
    H, L, K, Bg, T, Nq = 2, 520, 300, 64, 1, 600
    filled = L + 77
    kc, vc = _filled_caches(H, L, 2, filled, K, Bg, T, fmt=B.SCALE_E4M3)
    q = synth.queries(CONFIGS["cfg2_window21"], H, Nq, DEV)
    fused = B.attn_decode(q, kc, vc, n_kv=filled)
    out = B.attn_decode(q, kc, vc, n_kv=filled, workspace=_ws(H, Nq, L, 1))
    torch.cuda.synchronize()
    assert torch.equal(out, fused)


@pytest.mark.parametrize("L,T,Bg,S,bits,fmt,rope", [(520, 2, 32, 1, 2, B.SCALE_F16, False), (520, 4, 64, 1, 2, B.SCALE_F16, True),
                                                    (260, 1, 16, 4, 2, B.SCALE_E4M3, False)])
def test_shared_tiles_with_a_prefix_length_per_query(L, T, Bg, S, bits, fmt, rope):
    """A prefix length per query on the shared-tile path: chunk groups, lengths inside a chunk, the
    whole cache, one token, empty prefixes; sorted (query blocks stop early) and unsorted.  Equal to
    the one-kernel form bit for bit, and every query against the oracle over its own prefix."""
    H, K, Nq = 2, 64, 700
    n_chunks, filled = 4, 3 * L + 77
    kc, vc = _filled_caches(H, L, n_chunks, filled, K, Bg, T, S, bits, fmt)
    q = synth.queries(CONFIGS["cfg2_window21"], H, Nq, DEV)
    g = torch.Generator().manual_seed(5)
    lens = torch.empty(Nq, dtype=torch.int64)
    lens[:256] = 0                                   # a whole query block that sees nothing
    lens[256:400] = L
    lens[400:560] = 2 * L
    lens[560:660] = torch.randint(1, filled + 1, (100,), generator=g)
    lens[660:] = torch.tensor([1, 2, 63, 64, 65, L - 1, L + 1, filled, filled - 1, filled + 50, 0, -5] + [3 * L] * 28)
    table = _rope_table(filled).to(DEV) if rope else None
    khat, vhat = B.decode(kc, n_tokens=filled), B.decode(vc, n_tokens=filled)
    for order in ("sorted", "shuffled"):
        if order == "shuffled":
            lens = lens[torch.randperm(Nq, generator=g)]
        ql = lens.to(torch.int32).to(DEV)
        one, lse_one = B.attn_decode(q, kc, vc, want_lse=True, n_kv=filled, k_rope=table, q_kv_len=ql)
        for slab_chunks in (n_chunks, 1):
            out, lse = B.attn_decode(q, kc, vc, want_lse=True, n_kv=filled, k_rope=table, q_kv_len=ql,
                                     workspace=_ws(H, Nq, L, slab_chunks))
            torch.cuda.synchronize()
            assert torch.equal(out, one), (order, slab_chunks)
            assert torch.equal(lse, lse_one), (order, slab_chunks)
    eff = lens.clamp(0, filled).numpy()
    for h in range(H):
        kb = P.to_np_u16(khat[h])
        if rope:
            kb = O.rope_keys(kb, table.cpu().numpy().view(np.uint16))
        vb = P.to_np_u16(vhat[h])
        qb = bf16_bits(q[h])
        og, lg = P.to_np_u16(out[h]), lse[h].cpu().numpy()
        for n in np.unique(eff):
            rows = np.flatnonzero(eff == n)
            if n == 0:
                assert (og[rows] == 0).all() and np.isneginf(lg[rows]).all()
                continue
            want, lse_w = O.attention(qb[rows], kb[:n], vb[:n], want_lse=True)
            ok, max_abs, worst = P.attn_tolerance_ok(og[rows], want)
            assert ok, f"head {h}, prefix {n}: max abs err {max_abs}, worst err/tol {worst}"
            assert np.abs(lg[rows] - lse_w).max() < 2e-3, (h, n)


def test_calls_back_to_back_on_two_streams_share_one_workspace():
    """A cache of 9 chunks with a workspace for 4 (three slabs, the last one short or not), calls
    following each other without a synchronisation, on the current and on another stream: every
    call's kernels are ordered by the stream they are enqueued on, the workspace keeps nothing
    that a later call relies on."""
    H, L, K, Bg, T, Nq = 3, 330, 64, 64, 2, 900
    q = synth.queries(CONFIGS["cfg2_window21"], H, Nq, DEV)
    ws = _ws(H, Nq, L, 4)
    results = []
    for stream in (torch.cuda.current_stream(), torch.cuda.Stream()):
        with torch.cuda.stream(stream):
            for filled in (8 * L + 100, 7 * L + 1, 9 * L):             # 3, 2 and 3 slabs; the caches differ in length
                kc, vc = _filled_caches(H, L, 9, filled, K, Bg, T)
                out, lse = B.attn_decode(q, kc, vc, want_lse=True, n_kv=filled, workspace=ws)
                fused, lse_f = B.attn_decode(q, kc, vc, want_lse=True, n_kv=filled)
                results.append((out, lse, fused, lse_f))
    torch.cuda.synchronize()
    for out, lse, fused, lse_f in results:
        assert torch.equal(out, fused) and torch.equal(lse, lse_f)
    assert not torch.equal(results[0][0], results[1][0])             # different prefixes, different results
