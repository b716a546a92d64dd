"""Seeded synthetic K/V, query and start-centroid generators.

The paper measured on the KV cache of real video models; none of them is available
here, so these generators stand in.  They reproduce the shapes (tokens x head_dim
128 per head) and the value structure the paper describes: tokens cluster around a
modest number of modes (Sec. 3.3), and some channels carry much larger magnitudes
than others (Sec. 3.2).  This module holds no arithmetic of the codec itself; its
outputs are plain bf16 tensors handed, byte for byte, to the GPU library and to the
CPU oracle alike.
"""
from __future__ import annotations

import zlib

import torch

from .configs import BASE_SEED, Workload


def _name_id(name: str) -> int:
    return zlib.crc32(name.encode()) % 100003


def _gen(device, *stream) -> torch.Generator:
    """A generator whose seed mixes the base seed with the stream identifiers."""
    s = BASE_SEED
    for v in stream:
        s = (s * 1000003 + int(v) + 12345) % (2**62)
    g = torch.Generator(device=device)
    g.manual_seed(s)
    return g


class MixtureStream:
    """K or V tokens of `units` independent heads, produced chunk by chunk.

    Every unit has its own mixture centres ~ N(0, I) and its own channel scaling;
    a token picks a centre uniformly and adds sigma * N(0, I).  With `drift` > 0 the
    centres take a random-walk step before every chunk after the first.
    """

    def __init__(self, wl: Workload, units: int, kv: int, device="cpu", layer: int = 0):
        self.wl, self.units, self.kv, self.device, self.layer = wl, units, kv, device, layer
        d, M = wl.head_dim, wl.mix_components
        g = _gen(device, _name_id(wl.name), layer, kv, 0)
        self.g = g
        self.centres = torch.randn(units, M, d, generator=g, device=device)
        self.scale = torch.ones(units, 1, d, device=device)
        self.t_channels = None
        if wl.channel_scale == "outlier4x8":
            for u in range(units):
                idx = torch.randperm(d, generator=g, device=device)[:4]
                self.scale[u, 0, idx] = 8.0
        elif wl.channel_scale == "lognormal0.5":
            self.scale = torch.exp(0.5 * torch.randn(units, 1, d, generator=g, device=device))
        elif wl.channel_scale == "student_t3":
            self.t_channels = torch.stack(
                [torch.randperm(d, generator=g, device=device)[:4] for _ in range(units)])
        self.chunk_index = 0

    def next_chunk(self, n_tokens: int) -> torch.Tensor:
        """-> bf16 tensor [units, n_tokens, head_dim]."""
        wl, g, dev = self.wl, self.g, self.device
        d, M = wl.head_dim, wl.mix_components
        if self.chunk_index > 0 and wl.drift > 0:
            self.centres = self.centres + wl.drift * torch.randn(
                self.units, M, d, generator=g, device=dev)
        pick = torch.randint(0, M, (self.units, n_tokens), generator=g, device=dev)
        x = torch.gather(self.centres, 1, pick[:, :, None].expand(-1, -1, d))
        noise = torch.randn(self.units, n_tokens, d, generator=g, device=dev)
        if self.t_channels is not None:
            # heavy tails on four channels: Student-t(3) = N / sqrt(chi2_3 / 3), scaled x8
            z = torch.randn(self.units, n_tokens, 4, 3, generator=g, device=dev)
            t3 = torch.randn(self.units, n_tokens, 4, generator=g, device=dev) / torch.sqrt(
                (z * z).sum(-1) / 3.0)
            idx = self.t_channels[:, None, :].expand(-1, n_tokens, -1)
            noise.scatter_(2, idx, 8.0 * t3)
        x = (x + wl.sigma * noise) * self.scale
        self.chunk_index += 1
        return x.to(torch.bfloat16)


def queries(wl: Workload, units: int, n_q: int, device="cpu", step: int = 0) -> torch.Tensor:
    """bf16 queries ~ N(0, 1), [units, n_q, head_dim]."""
    g = _gen(device, _name_id(wl.name), 7, step)
    return torch.randn(units, n_q, wl.head_dim, generator=g, device=device).to(torch.bfloat16)


def cold_start_centroids(x: torch.Tensor, n_clusters: int, seed: int = 0) -> torch.Tensor:
    """Start centroids for a first chunk: n_clusters tokens of each unit, picked by a
    seeded permutation (the paper's k-means++ start is not specified, Sec. 4.3; a
    seeded pick replaces it and is passed to both implementations).
    x [units, N, d] bf16 -> [units, n_clusters, d] bf16.  If N < n_clusters the picks wrap."""
    units, N, d = x.shape
    g = _gen("cpu", 99, seed)
    out = torch.empty(units, n_clusters, d, dtype=x.dtype, device=x.device)
    for u in range(units):
        perm = torch.randperm(N, generator=g)
        idx = perm[torch.arange(n_clusters) % N].to(x.device)
        out[u] = x[u, idx]
    return out
