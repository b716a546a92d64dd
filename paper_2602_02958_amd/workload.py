"""The benchmark workload: a streaming KV cache of one layer held in compressed form.

One "step" is one pass of the whole hot path (paper Sec. 4.1-4.3) over one batch:
  1. encode the newly generated chunk of K and V (all heads in one call, warm-started from the
     previous chunk's centroids, Sec. 4.3) straight into the cache,
  2. decode the whole cache back to bf16,
  3. attention of the new chunk's queries over the compressed cache (decode fused in; with a
     workspace for the decoded tiles of a slab of chunks, so that every tile is decoded once per
     unit instead of once per block of 256 queries).
K heads and V heads are stacked as independent units: units [0, heads) are K, [heads, 2*heads) V.
Used by bench.py and by the full-size parity test, so that both run the same launches.
"""
from __future__ import annotations

from dataclasses import dataclass

import torch

from . import binding as B
from . import synth
from .configs import Workload


@dataclass
class Streaming:
    wl: Workload
    heads: int
    cache: B.Encoded            # [2*heads] units, all chunks
    x_new: torch.Tensor         # [2*heads, chunk, d] bf16: the chunk the step encodes
    init_new: torch.Tensor      # [2*heads, K, d]: previous chunk's centroids
    q: torch.Tensor             # [heads, n_q, d]
    new_index: int              # chunk slot the step writes
    decoded: torch.Tensor       # [2*heads, n_tokens, d] bf16 output buffer of step part 2
    attn_out: torch.Tensor
    workspace: torch.Tensor
    kept_chunks: dict           # chunk index -> bf16 input kept for parity sampling
    attn_ws: torch.Tensor = None    # workspace of the attention (decoded tiles of a slab of chunks), or None

    @property
    def k(self) -> B.Encoded:
        h = self.heads
        c = self.cache
        return B.Encoded(c.centroids[:h], c.ids[:h], c.codes[:h], c.scales[:h], c.chunk_len)

    @property
    def v(self) -> B.Encoded:
        h = self.heads
        c = self.cache
        return B.Encoded(c.centroids[h:], c.ids[h:], c.codes[h:], c.scales[h:], c.chunk_len)


ATTN_SLAB_CHUNKS = 32          # chunks whose decoded tiles the attention workspace holds (0: no workspace)


def build_streaming(wl: Workload, device="cuda", layer: int = 0, keep_inputs=(), n_tokens=None,
                    n_q=None, attn_slab_chunks=None) -> Streaming:
    """Fill all but the last chunk of the cache (cold start on the first chunk, warm afterwards),
    and leave the last chunk ready to be encoded by step()."""
    heads = wl.heads
    units = 2 * heads
    n_tokens = wl.tokens_per_layer if n_tokens is None else n_tokens
    n_q = wl.n_queries if n_q is None else n_q
    L = wl.chunk
    n_chunks = -(-n_tokens // L)
    cache = B.alloc_cache(units, n_tokens, L, wl.n_clusters, wl.group_size, wl.n_stages,
                          wl.head_dim, device)
    sk = synth.MixtureStream(wl, heads, 0, device, layer)
    sv = synth.MixtureStream(wl, heads, 1, device, layer)
    p = B.make_params(units, wl.n_clusters, wl.group_size, wl.n_stages, wl.kmeans_iters_cold)
    ws = torch.empty(max(B.workspace_bytes(p, B.ENTRY_ENCODE, L), 16), dtype=torch.uint8, device=device)
    kept = {}
    init = None
    x = None
    for c in range(n_chunks):
        n = min(L, n_tokens - c * L)
        x = torch.cat([sk.next_chunk(n), sv.next_chunk(n)], 0)
        if c in keep_inputs:
            kept[c] = x.clone()
        if c == 0:
            init = synth.cold_start_centroids(x, wl.n_clusters)
            iters = wl.kmeans_iters_cold
        else:
            init = cache.centroids[:, c - 1].contiguous()
            iters = wl.kmeans_iters_warm
        if c < n_chunks - 1 or n_chunks == 1:
            B.encode_chunk(x, init, wl.group_size, wl.n_stages, iters, cache=cache, chunk_index=c,
                           workspace=ws)
    if n_chunks == 1:
        init = synth.cold_start_centroids(x, wl.n_clusters)
    q = synth.queries(wl, heads, n_q, device)
    slab = ATTN_SLAB_CHUNKS if attn_slab_chunks is None else attn_slab_chunks
    attn_ws = B.attn_workspace(heads, n_q, L, min(slab, n_chunks), device) if slab > 0 else None
    return Streaming(wl, heads, cache, x, init.clone(), q, n_chunks - 1,
                     torch.empty(units, n_tokens, wl.head_dim, dtype=torch.bfloat16, device=device),
                     torch.empty(heads, n_q, wl.head_dim, dtype=torch.bfloat16, device=device),
                     ws, kept, attn_ws)


def step_encode(s: Streaming, iters=None):
    it = s.wl.kmeans_iters_warm if iters is None else iters
    if s.new_index == 0 and iters is None:
        it = s.wl.kmeans_iters_cold
    B.encode_chunk(s.x_new, s.init_new, s.wl.group_size, s.wl.n_stages, it, cache=s.cache,
                   chunk_index=s.new_index, workspace=s.workspace)


def step_decode(s: Streaming):
    B.decode(s.cache, out=s.decoded)


def step_attn(s: Streaming, shared_tiles=True):
    B.attn_decode(s.q, s.k, s.v, out=s.attn_out, workspace=s.attn_ws if shared_tiles else None)


def step(s: Streaming):
    step_encode(s)
    step_decode(s)
    step_attn(s)


def vectors_per_step(s: Streaming) -> dict:
    """Token-vectors (128 bf16 = 256 B each) each part of a step handles."""
    units = 2 * s.heads
    n_tokens = s.cache.ids.shape[1]
    return dict(encode=units * s.x_new.shape[1], decode=units * n_tokens, attn=units * n_tokens)
