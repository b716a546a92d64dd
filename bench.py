#!/usr/bin/env python3
"""Benchmark of the QVG KV-cache codec hot path on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg5_long]

One step = encode the new chunk + decode the whole cache + fused dequant-attention
(paper_2602_02958_amd/workload.py) on ONE layer of the workload at its full cache length; the
default workload is the largest configuration (cfg5_long: 24 units = 12 heads x K,V, 160 chunks of
4680 tokens = 748800 cached tokens per head, 4680 queries).  Prints ONE JSON line.  `value` is
the bf16-equivalent KV throughput of the whole step: 256 B x (vectors encoded + vectors decoded +
vectors read by the fused attention) / step time, inputs resident in HBM.  Per-phase rates with
their HBM fractions, the roofline of the dominant kernel, batches of all layers' chunks that fill
the chip (the shapes the HBM target of the encoder is stated for), the smaller window
configuration, and the CPU oracle timed on the host cores are in the same line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16

# HBM bytes per launch read off rocprofv3 counters (FETCH_SIZE + WRITE_SIZE, each scaled by what the
# same counter reads for a plain 1 GiB device copy): written by paper_2602_02958_amd/profsum.py
# from a profiling run of `bench.py --only <part>`, one line per (workload, part):
#   <workload> <part> fetch_bytes=<int> write_bytes=<int>
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.txt")


def measured_traffic(workload, part):
    """Counter bytes per launch of one part (attn / decode / encode_I0 ...) on a workload, or None."""
    try:
        for line in open(TRAFFIC_FILE):
            t = line.split()
            if len(t) >= 4 and t[0] == workload and t[1] == part:
                kv = dict(x.split("=") for x in t[2:] if "=" in x)
                return int(kv["fetch_bytes"]) + int(kv["write_bytes"])
    except (OSError, KeyError, ValueError):
        pass
    return None


def _event_ms(fn, reps):
    """Average duration of fn() in ms over reps runs, HIP events on torch's current stream
    (the stream the library launches on)."""
    import torch
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    b.synchronize()
    return a.elapsed_time(b) / reps


def _format_bytes(wl, units, tokens, chunk):
    """Algorithmic bytes of the stored format for `tokens` tokens of `units` units."""
    per_tok = wl.n_stages * (wl.head_dim // 4 + 2 * wl.head_dim // wl.group_size) + 1
    tables = -(-tokens // chunk) * wl.n_clusters * wl.head_dim * 2
    return units * (tokens * per_tok + tables)


def cpu_baseline(wl, budget_s=10.0, max_chunks=16):
    """The oracle as it stands, on the host cores, on a bounded sample of the same step: all units
    encode one chunk; a cache of min(the workload's length, max_chunks chunks) is decoded (the
    encoded chunk repeated: the oracle's decode cost does not depend on the content); a subset of
    the queries attends over that decoded cache.  The number of queries is chosen from an 8-query
    trial to fill budget_s.  `value` is the step's own definition applied to the sample:
    256 B x (vectors encoded + decoded + read by attention, the last scaled by the share of the
    query batch) / time."""
    import numpy as np
    import torch
    from oracle import qvg_oracle as O
    from paper_2602_02958_amd import synth
    cores = O.max_threads()
    heads = wl.heads
    units = 2 * heads
    n_enc = wl.chunk
    n_chunks = min(wl.n_chunks, max_chunks)
    xk = synth.MixtureStream(wl, heads, 0).next_chunk(n_enc)
    xv = synth.MixtureStream(wl, heads, 1).next_chunk(n_enc)
    x = torch.cat([xk, xv], 0)
    init = synth.cold_start_centroids(x, wl.n_clusters)
    xb = x.view(torch.int16).numpy().view(np.uint16)
    ib = init.view(torch.int16).numpy().view(np.uint16)
    t0 = time.perf_counter()
    enc = O.encode_batch(xb, ib, wl.n_clusters, wl.group_size, wl.n_stages, wl.kmeans_iters_warm)
    t_enc = time.perf_counter() - t0
    t0 = time.perf_counter()
    dec = np.concatenate([O.decode_batch(enc["cent"], enc["ids"], enc["codes"], enc["scales"], wl.group_size)
                          for _ in range(n_chunks)], 1)           # chunk by chunk, each with its own table
    t_dec = time.perf_counter() - t0
    n_tok = dec.shape[1]
    qall = synth.queries(wl, heads, wl.n_queries).view(torch.int16).numpy().view(np.uint16)
    t0 = time.perf_counter()
    O.attention_batch(np.ascontiguousarray(qall[:, :8]), dec[:heads], dec[heads:])
    t_trial = time.perf_counter() - t0
    nq = int(min(wl.n_queries, max(8, 8 * budget_s / max(t_trial, 1e-3))))
    t0 = time.perf_counter()
    O.attention_batch(np.ascontiguousarray(qall[:, :nq]), dec[:heads], dec[heads:])
    t_att = time.perf_counter() - t0
    vec_enc, vec_dec = units * n_enc, units * n_tok
    vec_att = units * n_tok * (nq / wl.n_queries)          # share of a full query batch
    total_vec = vec_enc + vec_dec + vec_att
    total_t = t_enc + t_dec + t_att
    return {
        "value": round(total_vec * 256 / total_t / 1e9, 6), "unit": "GB/s", "cores": cores,
        "kind": "oracle",
        "sample": (f"{units} units: encode of one {n_enc}-token chunk (I={wl.kmeans_iters_warm}) {t_enc:.2f}s, "
                   f"decode of {n_tok} of {wl.tokens_per_layer} cached tokens {t_dec:.2f}s, attention of {nq} of "
                   f"{wl.n_queries} queries x {heads} heads over those {n_tok} tokens {t_att:.2f}s (its vectors "
                   f"counted as {nq}/{wl.n_queries} of a pass over them)"),
        "encode_GBps": round(vec_enc * 256 / t_enc / 1e9, 6),
        "decode_GBps": round(vec_dec * 256 / t_dec / 1e9, 6),
        "attn_q_tokens_per_s": round(heads * nq / t_att, 3),
    }


def _large_decode_setup(torch, B, wl, dev):
    """A cache of 3 layers of the workload at full length with random content (ids, levels, scales,
    tables) and the output tensor: the same construction for the benchmark line and for the
    profiling run."""
    units = 2 * 3 * wl.heads
    n = wl.tokens_per_layer
    big = B.alloc_cache(units, n, wl.chunk, wl.n_clusters, wl.group_size, wl.n_stages, wl.head_dim, dev)
    g = torch.Generator(device=dev); g.manual_seed(1)
    big.ids.copy_(torch.randint(0, wl.n_clusters, big.ids.shape, generator=g, device=dev, dtype=torch.uint8))
    # codes: every 2-bit field one of the levels 0, +1, -1 (0b00, 0b01, 0b11)
    f = torch.tensor([0, 1, 3], dtype=torch.uint8, device=dev)[
        torch.randint(0, 3, big.codes.shape + (4,), generator=g, device=dev)]
    big.codes.copy_(f[..., 0] | (f[..., 1] << 2) | (f[..., 2] << 4) | (f[..., 3] << 6)); del f
    big.scales.copy_(torch.rand(big.scales.shape, generator=g, device=dev).to(torch.float16))
    big.centroids.copy_(torch.randn(big.centroids.shape, generator=g, device=dev).to(torch.bfloat16))
    outbuf = torch.empty(units, n, wl.head_dim, dtype=torch.bfloat16, device=dev)
    return big, outbuf, units, n


def _large_encode_setup(torch, B, synth, wl, dev):
    """One chunk of every layer x head x (K, V) of the workload (720 units for the 30 x 12 models):
    the batch that fills the chip several times over and does not fit the Infinity Cache."""
    units = 2 * wl.layers * wl.heads
    x = synth.MixtureStream(wl, units, 0, dev).next_chunk(wl.chunk)
    init = synth.cold_start_centroids(x, wl.n_clusters)
    cache = B.alloc_cache(units, wl.chunk, wl.chunk, wl.n_clusters, wl.group_size, wl.n_stages, wl.head_dim, dev)
    p = B.make_params(units, wl.n_clusters, wl.group_size, wl.n_stages, wl.kmeans_iters_cold)
    ws = torch.empty(B.workspace_bytes(p, B.ENTRY_ENCODE, wl.chunk), dtype=torch.uint8, device=dev)
    B.encode_chunk(x, init, wl.group_size, wl.n_stages, 5, cache=cache, workspace=ws)
    warm = cache.centroids[:, 0].contiguous()
    return units, x, init, warm, cache, ws


def large_encode_supplement(torch, B, synth, wl):
    """Single-pass / warm / cold encode of one chunk of all layers of a workload."""
    dev = "cuda"
    units, x, init, warm, cache, ws = _large_encode_setup(torch, B, synth, wl, dev)
    vec = units * wl.chunk
    alg = vec * 256 + _format_bytes(wl, units, wl.chunk, wl.chunk)
    out = {"workload": wl.name, "units": units, "tokens": wl.chunk, "algorithmic_bytes": int(alg)}
    for name, iters in (("encode_I0", 0), ("encode_I3", 3), ("encode_I10", 10)):
        fn = lambda: B.encode_chunk(x, warm if iters < 10 else init, wl.group_size, wl.n_stages, iters,
                                    cache=cache, workspace=ws)
        fn(); torch.cuda.synchronize()
        ms = _event_ms(fn, 10 if iters == 0 else 4)
        flops = 2.0 * wl.n_clusters * wl.head_dim * (iters + 1) * vec
        out[name] = {"ms": round(ms, 4), "GBps_bf16_equiv": round(vec * 256 / ms / 1e6, 1),
                     "hbm_GBps_algorithmic": round(alg / ms / 1e6, 1),
                     "hbm_frac": round(alg / ms / 1e6 / HBM_PEAK_GBPS, 4),
                     "assign_TFLOPs": round(flops / ms / 1e9, 1),
                     "traffic": measured_traffic(wl.name, "large_" + name)}
    return out


def large_supplement(torch, B, synth, CONFIGS):
    """cfg3-shaped batches that exceed the 256 MB Infinity Cache: decode of 3 layers' full cache,
    encode of one chunk of all 30 layers, attention of one layer."""
    wl = CONFIGS["cfg3_dit_small"]
    dev = "cuda"
    out = large_encode_supplement(torch, B, synth, wl)
    # ---- decode: 3 layers' full cache = 72 units x 126360 tokens
    big, outbuf, units, n = _large_decode_setup(torch, B, wl, dev)
    fn = lambda: B.decode(big, out=outbuf)
    fn(); torch.cuda.synchronize()
    ms = _event_ms(fn, 10)
    vec = units * n
    alg = vec * 256 + _format_bytes(wl, units, n, wl.chunk)
    out["decode"] = {"ms": round(ms, 4), "GBps_bf16_equiv": round(vec * 256 / ms / 1e6, 1),
                     "hbm_GBps_algorithmic": round(alg / ms / 1e6, 1),
                     "hbm_frac": round(alg / ms / 1e6 / HBM_PEAK_GBPS, 4), "units": units, "tokens": n,
                     "traffic": measured_traffic(wl.name, "large_decode")}
    del outbuf
    # ---- fused attention: one layer, 4680 queries of 12 heads over the 126360-token cache
    hd = wl.heads
    k = B.Encoded(big.centroids[:hd], big.ids[:hd], big.codes[:hd], big.scales[:hd], wl.chunk)
    v = B.Encoded(big.centroids[hd:2 * hd], big.ids[hd:2 * hd], big.codes[hd:2 * hd], big.scales[hd:2 * hd], wl.chunk)
    q = synth.queries(wl, hd, wl.n_queries, dev)
    o = torch.empty(hd, wl.n_queries, wl.head_dim, dtype=torch.bfloat16, device=dev)
    fn = lambda: B.attn_decode(q, k, v, out=o)
    fn(); torch.cuda.synchronize()
    ms = _event_ms(fn, 3)
    flops = 4.0 * wl.n_queries * n * wl.head_dim * hd
    out["attn_one_layer"] = {"ms": round(ms, 4), "TFLOPs": round(flops / ms / 1e9, 1),
                             "mfma_frac": round(flops / ms / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4),
                             "q_tokens_per_s": round(wl.n_queries * hd / ms * 1e3, 1),
                             "cache_tokens_per_s": round(n * hd / ms * 1e3, 1)}
    out["attn_one_layer_shared_tiles"] = _attn_shared(torch, B, q, k, v, o, 3, flops)
    return out


def warm_start_supplement(torch, B, synth, wl):
    """Centroid caching (Sec. 4.3): the fit of a chunk started from the previous chunk's centroids
    with few Lloyd iterations, against a cold fit (seeded token picks, more iterations): time of the
    encode call and k-means inertia (sum of squared distances to the assigned centroid, fp32 on
    the GPU with torch: a measurement, not part of the path)."""
    dev = "cuda"
    units, L = 2 * wl.heads, wl.chunk
    sk, sv = synth.MixtureStream(wl, wl.heads, 0, dev), synth.MixtureStream(wl, wl.heads, 1, dev)
    prev = torch.cat([sk.next_chunk(L), sv.next_chunk(L)], 0)
    x = torch.cat([sk.next_chunk(L), sv.next_chunk(L)], 0)
    enc_prev = B.encode_chunk(prev, synth.cold_start_centroids(prev, wl.n_clusters), wl.group_size,
                              wl.n_stages, wl.kmeans_iters_cold)
    warm_init = enc_prev.centroids[:, 0].contiguous()
    cold_init = synth.cold_start_centroids(x, wl.n_clusters, seed=1)
    p = B.make_params(units, wl.n_clusters, wl.group_size, wl.n_stages, wl.kmeans_iters_cold)
    ws = torch.empty(B.workspace_bytes(p, B.ENTRY_ENCODE, L), dtype=torch.uint8, device=dev)
    cache = B.alloc_cache(units, L, L, wl.n_clusters, wl.group_size, wl.n_stages, wl.head_dim, dev)

    def inertia():
        c = cache.centroids[:, 0].float()
        idx = cache.ids.long()[:, :, None].expand(-1, -1, wl.head_dim)
        return float(((x.float() - torch.gather(c, 1, idx)) ** 2).sum())

    out = {}
    for name, init, iters in (("cold", cold_init, wl.kmeans_iters_cold), ("warm", warm_init, wl.kmeans_iters_warm),
                              ("warm_no_iterations", warm_init, 0)):
        fn = lambda: B.encode_chunk(x, init, wl.group_size, wl.n_stages, iters, cache=cache, workspace=ws)
        fn(); torch.cuda.synchronize()
        out[name] = {"iters": iters, "ms": round(_event_ms(fn, 10), 4), "inertia": round(inertia(), 1)}
    out["speedup_warm_vs_cold"] = round(out["cold"]["ms"] / out["warm"]["ms"], 2)
    out["inertia_warm_over_cold"] = round(out["warm"]["inertia"] / out["cold"]["inertia"], 4)
    return out


# The paper's four presets (Sec. 5 "Implementation"): one quantization round, K = 256, FP8 E4M3
# scales; QVG = one smoothing stage with B = 64, QVG-Pro = four with B = 16; INT2 and INT4.
PAPER_PRESETS = {
    "qvg_int2": dict(S=1, group_size=64, bits=2), "qvg_pro_int2": dict(S=4, group_size=16, bits=2),
    "qvg_int4": dict(S=1, group_size=64, bits=4), "qvg_pro_int4": dict(S=4, group_size=16, bits=4),
}
TABLE1_CHUNK_TOKENS = 34800     # the chunk length at which the stored sizes give Table 1's ratios

# What the paper itself reports for this path (Sec. 5; no kernel-level throughput is given there):
# context for a reader of the result line, measured on other hardware with real models, not a target.
PAPER_CONTEXT = {
    "note": "the paper's own figures: end-to-end, NVIDIA H100 (CUDA + Triton kernels), real model KV; context only",
    "qvg_extra_time_in_a_full_run": "0.74 s of 43 s = 1.7 % (H100, Self-Forcing 480p, batch 1; Table 6)",
    "kmeans_and_quantization_share_at_37440_token_chunks": "1.3 % (H100, Self-Forcing; Table 4)",
    "end_to_end_latency_overhead": "2.1 % LongCat-Video-13B, 1.5 % HY-WorldPlay-8B, 4.3 % Self-Forcing (H100; Sec. 5)",
    "centroid_caching": "k-means overhead reduced 3x (Sec. 4.3)",
    "compression_ratio_int2": "6.94x / 7.05x QVG, 4.97x / 5.20x QVG-Pro (Table 1)",
}


def staged_cold_start(torch, B, synth, x, n_clusters, S, group_size, n_stages, iters, bits, scale_format):
    """Start centroids of S smoothing stages for a first chunk: stage s starts from seeded picks
    among the tokens of ITS input, the residual that the library's own fit of the stages before it
    leaves (rebuilt here from that fit's centroids and ids, rounded to bf16 like the library's
    stage input).  Picks among the original tokens would start every later stage far from its
    data: nearly all of its clusters stay empty.  [units, S, K, d] bf16."""
    inits, r = [], x
    for s in range(S):
        inits.append(synth.cold_start_centroids(r, n_clusters, seed=s))
        if s + 1 < S:
            enc = B.encode_chunk(x, torch.stack(inits, 1) if s else inits[0], group_size, n_stages, iters,
                                 bits=bits, scale_format=scale_format)
            cent = enc.centroids[:, 0] if s else enc.centroids[:, 0, None]      # [units, s+1, K, d]
            ids = enc.ids if s else enc.ids[:, :, None]
            idx = ids[:, :, s].long()[:, :, None].expand(-1, -1, x.shape[-1])
            r = (r.float() - torch.gather(cent[:, s], 1, idx).float()).to(torch.bfloat16)
    return torch.stack(inits, 1)


def preset_supplement(torch, B, synth, CONFIGS, S=4, group_size=16, n_stages=1, n_clusters=256, bits=2,
                      scale_format=1):
    """One of the paper's presets on the cfg2 window: 24 units, 8 chunks of 4680 tokens, 4680
    queries."""
    wl = CONFIGS["cfg2_window21"]
    dev = "cuda"
    heads, units, L, n = wl.heads, 2 * wl.heads, wl.chunk, wl.tokens_per_layer
    cache = B.alloc_cache(units, n, L, n_clusters, group_size, n_stages, wl.head_dim, dev, n_smooth=S, bits=bits,
                          scale_format=scale_format)
    sk, sv = synth.MixtureStream(wl, heads, 0, dev), synth.MixtureStream(wl, heads, 1, dev)
    x = init = None
    for c in range(wl.n_chunks):
        x = torch.cat([sk.next_chunk(L), sv.next_chunk(L)], 0)
        if c > 0:
            init = cache.centroids[:, c - 1].contiguous()
        elif S > 1:
            init = staged_cold_start(torch, B, synth, x, n_clusters, S, group_size, n_stages, 10, bits, scale_format)
        else:
            init = synth.cold_start_centroids(x, n_clusters, seed=0)
        B.encode_chunk(x, init, group_size, n_stages, 10 if c == 0 else 3, cache=cache, chunk_index=c)
    out = {"preset": f"S={S} B={group_size} T={n_stages} K={n_clusters} bits={bits} "
                     f"scales={'e4m3' if scale_format else 'f16'}", "units": units, "tokens": n}
    p = B.make_params(units, n_clusters, group_size, n_stages, 3, n_smooth_stages=S, bits=bits,
                      scale_format=scale_format)
    ws = torch.empty(B.workspace_bytes(p, B.ENTRY_ENCODE, L), dtype=torch.uint8, device=dev)
    fn = lambda: B.encode_chunk(x, init, group_size, n_stages, 3, cache=cache, chunk_index=wl.n_chunks - 1, workspace=ws)
    fn(); torch.cuda.synchronize()
    ms = _event_ms(fn, 5)
    out["encode_I3"] = {"ms": round(ms, 4), "GBps_bf16_equiv": round(units * L * 256 / ms / 1e6, 1)}
    dec = torch.empty(units, n, wl.head_dim, dtype=torch.bfloat16, device=dev)
    fn = lambda: B.decode(cache, out=dec)
    fn(); torch.cuda.synchronize()
    ms = _event_ms(fn, 10)
    alg = units * n * 256 + B.compressed_bytes(p, L) * wl.n_chunks
    out["decode"] = {"ms": round(ms, 4), "GBps_bf16_equiv": round(units * n * 256 / ms / 1e6, 1),
                     "hbm_GBps_algorithmic": round(alg / ms / 1e6, 1)}
    q = synth.queries(wl, heads, wl.n_queries, dev)
    k = B.Encoded(cache.centroids[:heads], cache.ids[:heads], cache.codes[:heads], cache.scales[:heads], L, S)
    v = B.Encoded(cache.centroids[heads:], cache.ids[heads:], cache.codes[heads:], cache.scales[heads:], L, S)
    o = torch.empty(heads, wl.n_queries, wl.head_dim, dtype=torch.bfloat16, device=dev)
    fn = lambda: B.attn_decode(q, k, v, out=o)
    fn(); torch.cuda.synchronize()
    ms = _event_ms(fn, 3)
    flops = 4.0 * wl.n_queries * n * wl.head_dim * heads
    out["attn"] = {"ms": round(ms, 4), "TFLOPs": round(flops / ms / 1e9, 1)}
    out["attn_shared_tiles"] = _attn_shared(torch, B, q, k, v, o, 3, flops)
    out["compression_ratio"] = round(units * L * 256 / B.compressed_bytes(p, L), 3)
    out["compression_ratio_at_table1_chunk"] = round(
        units * TABLE1_CHUNK_TOKENS * 256 / B.compressed_bytes(p, TABLE1_CHUNK_TOKENS), 3)
    xhat = dec[:, (wl.n_chunks - 1) * L:].float()
    out["rel_l2_error_last_chunk"] = round(float((xhat - x.float()).norm() / x.float().norm()), 4)
    return out


def presets_supplement(torch, B, synth, CONFIGS):
    return {name: preset_supplement(torch, B, synth, CONFIGS, **kw) for name, kw in PAPER_PRESETS.items()}


def codebook_supplement(torch, B, synth, CONFIGS):
    """The codebook-size study of Sec. 5 (Table 5) on the cfg2 window: QVG INT2 with K = 64 .. 512
    centroids (512: 16-bit ids, the general attention kernel)."""
    return {f"K{K}": preset_supplement(torch, B, synth, CONFIGS, S=1, group_size=64, bits=2, n_clusters=K)
            for K in (64, 128, 256, 512)}


def long_supplement(torch, B, synth, CONFIGS, name="cfg5_long"):
    """One layer of a configuration at full size (default cfg5, the long-horizon one: 12 heads, 160
    chunks of 4680 tokens = 748800 cached tokens per head, K = 256, T = 4, centres drifting from
    chunk to chunk; also run for cfg4: 40 heads, 10 chunks of 10800 tokens, K = 128, T = 3, B = 32):
    the cache is filled chunk by chunk through the rollout object with centroid caching
    (Sec. 4.3), then decoded and attended over as a whole."""
    wl = CONFIGS[name]
    dev = "cuda"
    heads, L, n = wl.heads, wl.chunk, wl.tokens_per_layer
    sc = B.StreamingCache(heads, n, L, wl.n_clusters, wl.group_size, wl.n_stages, wl.head_dim, dev,
                          warm_iters=wl.kmeans_iters_warm, cold_iters=wl.kmeans_iters_cold)
    sk, sv = synth.MixtureStream(wl, heads, 0, dev), synth.MixtureStream(wl, heads, 1, dev)
    ev = []
    x = None
    for c in range(wl.n_chunks):
        x = torch.cat([sk.next_chunk(L), sv.next_chunk(L)], 0)
        init = synth.cold_start_centroids(x, wl.n_clusters) if c == 0 else None
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(); sc.append(x, init=init); e1.record()
        ev.append((e0, e1))
    torch.cuda.synchronize()
    ms = [a.elapsed_time(b) for a, b in ev]
    out = {"workload": wl.name, "units": 2 * heads, "tokens": n, "chunks": wl.n_chunks,
           "fill": {"first_chunk_cold_ms": round(ms[0], 4), "warm_chunk_ms_avg": round(sum(ms[1:]) / (len(ms) - 1), 4),
                    "total_ms": round(sum(ms), 2)}}
    # the last chunk again, cold (seeded token picks, 10 iterations), for the saving of Sec. 4.3
    cold = B.alloc_cache(2 * heads, L, L, wl.n_clusters, wl.group_size, wl.n_stages, wl.head_dim, dev)
    init = synth.cold_start_centroids(x, wl.n_clusters)
    fn = lambda: B.encode_chunk(x, init, wl.group_size, wl.n_stages, wl.kmeans_iters_cold, cache=cold)
    fn(); torch.cuda.synchronize()
    out["fill"]["cold_chunk_ms"] = round(_event_ms(fn, 5), 4)
    out["fill"]["speedup_warm_vs_cold"] = round(out["fill"]["cold_chunk_ms"] / out["fill"]["warm_chunk_ms_avg"], 2)
    stored = sc.stored_bytes()
    out["stored_GB"] = round(stored / 1e9, 3)
    out["compression_ratio"] = round(2 * heads * n * 256 / stored, 3)
    dec = torch.empty(2 * heads, n, wl.head_dim, dtype=torch.bfloat16, device=dev)
    fn = lambda: sc.decode(out=dec)
    fn(); torch.cuda.synchronize()
    ms_d = _event_ms(fn, 3)
    alg = 2 * heads * n * 256 + stored
    out["decode"] = {"ms": round(ms_d, 3), "GBps_bf16_equiv": round(2 * heads * n * 256 / ms_d / 1e6, 1),
                     "hbm_GBps_algorithmic": round(alg / ms_d / 1e6, 1), "hbm_frac": round(alg / ms_d / 1e6 / HBM_PEAK_GBPS, 4)}
    del dec
    q = synth.queries(wl, heads, wl.n_queries, dev)
    o = torch.empty(heads, wl.n_queries, wl.head_dim, dtype=torch.bfloat16, device=dev)
    fn = lambda: sc.attend(q, out=o)
    fn(); torch.cuda.synchronize()
    ms_a = _event_ms(fn, 2)
    flops = 4.0 * wl.n_queries * n * wl.head_dim * heads
    out["attn"] = {"ms": round(ms_a, 3), "TFLOPs": round(flops / ms_a / 1e9, 1),
                   "mfma_frac": round(flops / ms_a / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4),
                   "cache_tokens_per_s": round(n * heads / ms_a * 1e3, 1)}
    out["attn_shared_tiles"] = _attn_shared(torch, B, q, sc.k, sc.v, o, 2, flops, n_kv=sc.n_tokens)
    return out


def integration_supplement(torch, B, s):
    """Attention-side pieces of a generation step on the benchmark's own state: the fused
    attention with the rotary embedding applied to the decoded keys (pre-RoPE key caching, Sec. 5
    "Implementation"), and the merge with the current chunk's own attention result (Sec. 3.1)."""
    wl = s.wl
    n_kv = s.cache.ids.shape[1]
    pos = torch.arange(n_kv, dtype=torch.float64, device="cuda")
    freq = 10000.0 ** (-torch.arange(wl.head_dim // 2, dtype=torch.float64, device="cuda") / (wl.head_dim // 2))
    ang = pos[:, None] * freq[None]
    rope = torch.stack([ang.cos(), ang.sin()], -1).to(torch.float16).contiguous()
    out = {}
    fn = lambda: B.attn_decode(s.q, s.k, s.v, out=s.attn_out, k_rope=rope)
    fn(); torch.cuda.synchronize()
    ms = _event_ms(fn, 5)
    flops = 4.0 * wl.n_queries * n_kv * wl.head_dim * wl.heads
    out["attn_with_rope"] = {"ms": round(ms, 4), "TFLOPs": round(flops / ms / 1e9, 1)}
    out["attn_with_rope_shared_tiles"] = _attn_shared(torch, B, s.q, s.k, s.v, s.attn_out, 5, flops, k_rope=rope)
    oa, la = B.attn_decode(s.q, s.k, s.v, want_lse=True)
    ob, lb = oa.flip(1).contiguous(), la.flip(1).contiguous()
    res = torch.empty_like(oa)
    fn = lambda: B.attn_merge(oa, la, ob, lb, out=res)
    fn(); torch.cuda.synchronize()
    ms = _event_ms(fn, 20)
    nbytes = oa.numel() * 2 * 3 + la.numel() * 4 * 2
    out["merge"] = {"ms": round(ms, 5), "rows": int(la.numel()), "GBps_algorithmic": round(nbytes / ms / 1e6, 1)}
    # chunk-causal order in one call: the queries split into as many groups as the cache has chunks,
    # group c seeing the first c chunks (a prefix length per query)
    n_chunks = -(-n_kv // wl.chunk)
    grp = torch.arange(wl.n_queries, device="cuda") * n_chunks // wl.n_queries + 1
    lens = torch.clamp(grp * wl.chunk, max=n_kv).to(torch.int32)
    full = torch.full_like(lens, n_kv)
    for name, ql in (("causal_chunk_groups", lens), ("causal_all_full_length", full)):
        fn = lambda ql=ql: B.attn_decode(s.q, s.k, s.v, out=s.attn_out, q_kv_len=ql)
        fn(); torch.cuda.synchronize()
        ms = _event_ms(fn, 5)
        fl = 4.0 * float(ql.sum().item()) * wl.head_dim * wl.heads
        out[name] = {"ms": round(ms, 4), "TFLOPs": round(fl / ms / 1e9, 1)}
        out[name + "_shared_tiles"] = _attn_shared(torch, B, s.q, s.k, s.v, s.attn_out, 5, fl, q_kv_len=ql)
    return out


def run_only(args, torch, B, synth, workload, CONFIGS):
    """One part of the path, repeated: what rocprofv3 is pointed at."""
    dev = "cuda"
    wl = CONFIGS[args.workload]
    if args.only == "copy":
        n = 1 << 30
        a = torch.empty(n, dtype=torch.uint8, device=dev).random_(0, 255)
        b = torch.empty_like(a)
        fn = lambda: b.copy_(a)
        nbytes = 2 * n
    elif args.only == "large_decode":
        wl = CONFIGS["cfg3_dit_small"]
        big, outbuf, units, n = _large_decode_setup(torch, B, wl, dev)
        fn = lambda: B.decode(big, out=outbuf)
        nbytes = units * n * 256 + _format_bytes(wl, units, n, wl.chunk)
    elif args.only == "large_encode":
        # one chunk of all layers of --workload (cfg3_dit_small and cfg5_long: 720 units)
        units, x, init, warm, cache, ws = _large_encode_setup(torch, B, synth, wl, dev)
        fn = lambda: B.encode_chunk(x, warm, wl.group_size, wl.n_stages, args.iters, cache=cache, workspace=ws)
        nbytes = units * wl.chunk * 256 + _format_bytes(wl, units, wl.chunk, wl.chunk)
    else:
        s = workload.build_streaming(wl)
        workload.step(s)
        vec = workload.vectors_per_step(s)
        units, n_tok = 2 * wl.heads, s.cache.ids.shape[1]
        if args.only == "decode":
            fn = lambda: workload.step_decode(s)
            nbytes = vec["decode"] * 256 + _format_bytes(wl, units, n_tok, wl.chunk)
        elif args.only == "encode":
            fn = lambda: workload.step_encode(s, iters=args.iters)
            nbytes = vec["encode"] * 256 + _format_bytes(wl, units, s.x_new.shape[1], wl.chunk)
        elif args.only == "step":
            fn = lambda: workload.step(s)
            nbytes = 0
        else:
            fn = lambda: workload.step_attn(s, shared_tiles=args.only == "attn")
            nbytes = _format_bytes(wl, units, n_tok, wl.chunk) + 2 * wl.heads * wl.n_queries * wl.head_dim * 2
    for _ in range(max(args.warmup, 1)):
        fn()
    torch.cuda.synchronize()
    ms = _event_ms(fn, args.steps)
    return {"only": args.only, "workload": wl.name, "ms": round(ms, 5), "algorithmic_bytes": int(nbytes),
            "GBps_algorithmic": round(nbytes / ms / 1e6, 1), "launches": args.steps + max(args.warmup, 1)}


def _attn_shared(torch, B, q, k, v, o, reps, flops, **kw):
    """The same attention with a workspace for the decoded tiles (slabs of workload.ATTN_SLAB_CHUNKS chunks)."""
    H, n_q = q.shape[0], q.shape[1]
    n_kv = kw.get("n_kv") or k.ids.shape[1]
    n_chunks = -(-n_kv // k.chunk_len)
    ws = B.attn_workspace(H, n_q, k.chunk_len, min(n_chunks, workload_slab_chunks()), q.device)
    fn = lambda: B.attn_decode(q, k, v, out=o, workspace=ws, **kw)
    fn(); torch.cuda.synchronize()
    ms = _event_ms(fn, reps)
    return {"ms": round(ms, 4), "TFLOPs": round(flops / ms / 1e9, 1),
            "mfma_frac": round(flops / ms / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4), "workspace_bytes": int(ws.numel())}


def _attn_form(s):
    """How the step's attention runs: with the workspace, the number of slabs of the call."""
    if s.attn_ws is None:
        return {"workspace_bytes": 0, "launches": {"attn_kernel_staged": 1}}
    wl = s.wl
    n_chunks = -(-s.cache.ids.shape[1] // wl.chunk)
    slab = min(n_chunks, workload_slab_chunks())
    slabs = -(-n_chunks // slab)
    return {"workspace_bytes": int(s.attn_ws.numel()), "slab_chunks": slab,
            "launches": {"slab_decode_kernel": slabs, "attn_slab_kernel": slabs}}


def workload_slab_chunks():
    from paper_2602_02958_amd import workload
    return workload.ATTN_SLAB_CHUNKS


def measure_step(torch, B, workload, wl, steps, warmup):
    """Build one layer of `wl` at its full cache length, time `steps` steps after `warmup`, then each
    phase on its own.  -> (streaming state, ms per step, ms of the attention launch inside the
    timed steps, vectors per step, phases dict)."""
    s = workload.build_streaming(wl)
    torch.cuda.synchronize()
    for _ in range(warmup):
        workload.step(s)
    torch.cuda.synchronize()
    # HIP events around the dominant kernel's launch in every timed step, on the stream the library
    # launches on (torch's current stream)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        workload.step_encode(s)
        workload.step_decode(s)
        ev[i][0].record()
        workload.step_attn(s)
        ev[i][1].record()
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / steps
    ms_att_in_step = sum(a.elapsed_time(b) for a, b in ev) / max(steps, 1)
    vec = workload.vectors_per_step(s)

    # ---- per-phase timing (HIP events on the launch stream) -----------------
    reps = max(5, steps)
    ms_dec = _event_ms(lambda: workload.step_decode(s), reps)
    ms_att = _event_ms(lambda: workload.step_attn(s), max(3, steps // 4))
    ms_att_one = _event_ms(lambda: workload.step_attn(s, shared_tiles=False), max(3, steps // 4))
    ms_enc = {i: _event_ms(lambda i=i: workload.step_encode(s, iters=i), reps)
              for i in (0, wl.kmeans_iters_warm, wl.kmeans_iters_cold)}
    units = 2 * wl.heads
    n_tok = s.cache.ids.shape[1]
    n_new = s.x_new.shape[1]
    stored = _format_bytes(wl, units, n_tok, wl.chunk)
    dec_alg = vec["decode"] * 256 + stored
    enc_alg = vec["encode"] * 256 + _format_bytes(wl, units, n_new, wl.chunk)
    att_flops = 4.0 * wl.n_queries * n_tok * wl.head_dim * wl.heads
    note = ""
    if dec_alg < 2.6e8:
        note = "cache-resident size (compressed + bf16 < 256 MB Infinity Cache)"
    elif stored < 2.6e8:
        note = ("the compressed cache (%d MB) fits the 256 MB Infinity Cache and is re-read from it by every "
                "repetition" % (stored >> 20))
    phases = {
        "decode": {"ms": round(ms_dec, 4), "GBps_bf16_equiv": round(vec["decode"] * 256 / ms_dec / 1e6, 1),
                   "algorithmic_bytes": int(dec_alg),
                   "hbm_GBps_algorithmic": round(dec_alg / ms_dec / 1e6, 1),
                   "hbm_frac": round(dec_alg / ms_dec / 1e6 / HBM_PEAK_GBPS, 4),
                   "traffic": measured_traffic(wl.name, "decode"), "note": note},
        "attn": {"ms": round(ms_att, 4), "q_tokens_per_s": round(wl.n_queries * wl.heads / ms_att * 1e3, 1),
                 "cache_tokens_per_s": round(n_tok * wl.heads / ms_att * 1e3, 1),
                 "TFLOPs": round(att_flops / ms_att / 1e9, 2),
                 "mfma_frac": round(att_flops / ms_att / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4),
                 "flops_per_launch": att_flops,
                 "algorithmic_bytes": int(stored + 2 * wl.heads * wl.n_queries * wl.head_dim * 2),
                 "traffic": measured_traffic(wl.name, "attn"),
                 "form": _attn_form(s)},
        # the same attention in one kernel, no workspace: every block of 256 queries decodes for itself
        "attn_one_kernel": {"ms": round(ms_att_one, 4), "TFLOPs": round(att_flops / ms_att_one / 1e9, 2),
                            "mfma_frac": round(att_flops / ms_att_one / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4),
                            "traffic": measured_traffic(wl.name, "attn_one_kernel")},
    }
    for i, ms in ms_enc.items():
        phases[f"encode_I{i}"] = {"ms": round(ms, 4), "GBps_bf16_equiv": round(vec["encode"] * 256 / ms / 1e6, 1),
                                  "algorithmic_bytes": int(enc_alg),
                                  "hbm_GBps_algorithmic": round(enc_alg / ms / 1e6, 1),
                                  "hbm_frac": round(enc_alg / ms / 1e6 / HBM_PEAK_GBPS, 4),
                                  "traffic": measured_traffic(wl.name, f"encode_I{i}")}
    return s, ms_step, ms_att_in_step, vec, phases


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg5_long")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-large", action="store_true")
    ap.add_argument("--only", default=None,
                    choices=["decode", "encode", "attn", "attn_fused", "step", "copy", "large_decode", "large_encode", "presets", "long"],
                    help="profiling aid: run just this part --steps times and print a short JSON "
                         "(copy = a plain device copy of 1 GiB, the reference the HBM counters "
                         "are scaled by; large_encode = one chunk of all layers of --workload)")
    ap.add_argument("--iters", type=int, default=0, help="Lloyd iterations for --only encode / large_encode")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); "
              "--gpus N with N > 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2602_02958_amd import binding as B
    from paper_2602_02958_amd import synth, workload
    from paper_2602_02958_amd.configs import CONFIGS
    B.lib()                                    # fail loudly if the HIP library is missing
    wl = CONFIGS[args.workload]
    torch.cuda.set_device(0)
    if args.only == "long":
        print(json.dumps(long_supplement(torch, B, synth, CONFIGS)))
        torch.cuda.empty_cache()
        print(json.dumps(long_supplement(torch, B, synth, CONFIGS, "cfg4_dit_large")))
        return
    if args.only == "presets":
        w2 = CONFIGS["cfg2_window21"]
        print(json.dumps(presets_supplement(torch, B, synth, CONFIGS)))
        print(json.dumps(codebook_supplement(torch, B, synth, CONFIGS)))
        print(json.dumps(warm_start_supplement(torch, B, synth, w2)))
        return
    if args.only:
        print(json.dumps(run_only(args, torch, B, synth, workload, CONFIGS)))
        return

    s, ms_step, ms_att_in_step, vec, phases = measure_step(torch, B, workload, wl, args.steps, args.warmup)
    total_vec = vec["encode"] + vec["decode"] + vec["attn"]
    value = total_vec * 256 / ms_step / 1e6          # GB/s
    units = 2 * wl.heads
    n_tok = s.cache.ids.shape[1]
    n_new = s.x_new.shape[1]
    # dominant kernel of the step by time: the attention over the decoded tiles (attn_slab_kernel,
    # one launch per slab of chunks).  Its duration is taken, by HIP events over the timed steps
    # above, as that of the WHOLE attention call - its launches and those of the tile decode kernel
    # that feeds them - so `achieved` is a lower bound of the kernel's own rate (the committed
    # rocprofv3 summary has the two kernels apart); flops are those of the call.
    att_flops = phases["attn"]["flops_per_launch"]
    att_tflops = att_flops / ms_att_in_step / 1e9
    form = phases["attn"]["form"]
    roofline = {"bound": "mfma", "kernel": "attn_slab_kernel" if form["workspace_bytes"] else "attn_kernel_staged",
                "achieved": round(att_tflops, 2),
                "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(att_tflops / MFMA_BF16_PEAK_TFLOPS, 4),
                "ms_per_launch": round(ms_att_in_step, 4),
                "flops_per_launch": att_flops,
                "launches_per_step": form["launches"],
                "timed": "the whole attention call (all launches listed), HIP events inside the timed steps",
                "share_of_step_time": round(ms_att_in_step / ms_step, 4),
                "traffic": measured_traffic(wl.name, "attn")}
    result = {
        "metric": "KV encode/decode GB/s (bf16-equiv) + fused dequant-attn tokens/s, % HBM roofline",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "layers_in_step": "1 of %d" % wl.layers, "units": units,
                   "tokens_in_cache": n_tok, "chunk": n_new,
                   "n_queries": wl.n_queries, "K": wl.n_clusters, "T": wl.n_stages, "B": wl.group_size,
                   "kmeans_iters_in_step": wl.kmeans_iters_warm,
                   "step": "encode chunk + decode cache + attention over the compressed cache "
                           "(tiles decoded once per unit into a workspace slab, shared by all query blocks)",
                   "value_definition": "256 B x (vectors encoded + decoded + read by attention) / step time"},
        "roofline": roofline,
        "phases": phases,
    }
    integ_state = s if wl.name == "cfg2_window21" else None
    if not args.no_large:
        if integ_state is None:
            del s
            torch.cuda.empty_cache()
        try:
            # the batches the encoder's HBM target is stated for: one chunk of all layers
            result["large_encode_" + wl.name] = large_encode_supplement(torch, B, synth, wl)
            torch.cuda.empty_cache()
            result["large"] = large_supplement(torch, B, synth, CONFIGS)
        except torch.OutOfMemoryError as e:     # a smaller card than the one this is written for
            result["large"] = {"error": str(e)[:200]}
        torch.cuda.empty_cache()
        w2 = CONFIGS["cfg2_window21"]
        if integ_state is None:
            s2, ms2, ms2_att, vec2, ph2 = measure_step(torch, B, workload, w2, max(5, args.steps // 2), 2)
            result["cfg2_window21"] = {"ms_per_step": round(ms2, 4),
                                       "value": round((vec2["encode"] + vec2["decode"] + vec2["attn"]) * 256 / ms2 / 1e6, 2),
                                       "attn_ms_in_step": round(ms2_att, 4), "phases": ph2}
            integ_state = s2
        result["paper_presets"] = presets_supplement(torch, B, synth, CONFIGS)
        result["codebook_size"] = codebook_supplement(torch, B, synth, CONFIGS)
        result["warm_start"] = warm_start_supplement(torch, B, synth, w2)
        result["attn_integration"] = integration_supplement(torch, B, integ_state)
        del integ_state
        torch.cuda.empty_cache()
        result["long_horizon"] = long_supplement(torch, B, synth, CONFIGS)
        torch.cuda.empty_cache()
        result["cfg4_layer"] = long_supplement(torch, B, synth, CONFIGS, "cfg4_dit_large")
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl)
    result["paper_context"] = PAPER_CONTEXT
    print(json.dumps(result))


if __name__ == "__main__":
    main()
