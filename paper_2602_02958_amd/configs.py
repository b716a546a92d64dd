"""The five workload configurations this build is measured and tested on.

Shapes follow the paper's models (head_dim 128, 1560 latent tokens per frame and a
21-frame window for the Self-Forcing-Wan-1.3B style cache, Sec. 3.1 and Sec. 5
"Setup"); codec parameters use the paper's names (Sec. 5 "Implementation"):
K centroids, B group size, and T rounds of 2-bit quantization after one smoothing
stage.  Pure data: no arithmetic of the method lives here.
"""
from __future__ import annotations

from dataclasses import dataclass


@dataclass(frozen=True)
class Workload:
    name: str
    layers: int
    heads: int
    head_dim: int
    tokens_per_layer: int     # cached tokens per layer when the cache is full
    chunk: int                # tokens encoded per call
    n_clusters: int           # K
    n_stages: int             # T
    group_size: int           # B
    n_queries: int            # queries per fused-attention step
    mix_components: int       # Gaussians in the synthetic mixture
    sigma: float              # within-component standard deviation
    channel_scale: str        # "none" | "outlier4x8" | "lognormal0.5" | "student_t3"
    drift: float              # per-chunk random-walk sigma of the mixture centres
    kmeans_iters_cold: int
    kmeans_iters_warm: int

    @property
    def n_chunks(self) -> int:
        return -(-self.tokens_per_layer // self.chunk)


CONFIGS = {
    "cfg1_tiny": Workload("cfg1_tiny", 1, 1, 128, 4096, 4096, 16, 2, 64, 64,
                          16, 0.2, "outlier4x8", 0.0, 10, 10),
    "cfg2_window21": Workload("cfg2_window21", 1, 12, 128, 32760 + 4680, 4680, 64, 3, 32, 4680,
                              64, 0.2, "lognormal0.5", 0.0, 10, 3),
    "cfg3_dit_small": Workload("cfg3_dit_small", 30, 12, 128, 126360, 4680, 256, 2, 64, 4680,
                               64, 0.2, "lognormal0.5", 0.0, 10, 3),
    "cfg4_dit_large": Workload("cfg4_dit_large", 40, 40, 128, 108000, 10800, 128, 3, 32, 10800,
                               128, 0.2, "student_t3", 0.0, 10, 3),
    "cfg5_long": Workload("cfg5_long", 30, 12, 128, 748800, 4680, 256, 4, 64, 4680,
                          64, 0.2, "lognormal0.5", 0.05, 10, 3),
}

BASE_SEED = 260202958
