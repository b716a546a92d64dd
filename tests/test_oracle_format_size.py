"""Pins the storage-size arithmetic against the compression ratios the paper prints
(tests/golden/paper_compression_ratios.txt: Tables 1 and 4; paper_table5_codebook_size.txt:
Table 5)."""
import math
import os

from oracle import qvg_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_compression_ratios.txt")
D = 128


def _rows():
    rows = {}
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        f = line.split()
        rows[f[0]] = dict(bits=int(f[1]), S=int(f[2]), B=int(f[3]), K=int(f[4]), N=int(f[5]),
                          ratio=float(f[6]), tol=float(f[7]))
    return rows


def _ratio(N, r):
    # the paper's own format: FP8 scale (1 byte), uint8 ids, one code set (T = 1)
    stored = O.chunk_bytes(N, D, r["K"], r["B"], r["S"], 1, r["bits"], 1.0, 8.0)
    return (N * D * 2) / stored


def test_table4_ratios():
    rows = _rows()
    for key in ("T4_24frames", "T4_12frames"):
        r = rows[key]
        assert abs(_ratio(r["N"], r) - r["ratio"]) <= r["tol"], key


def _solve_N(r):
    lo, hi = 1000, 10_000_000
    while hi - lo > 1:
        mid = (lo + hi) // 2
        if _ratio(mid, r) < r["ratio"]:
            lo = mid
        else:
            hi = mid
    return hi


def test_table1_qvg_and_pro_rows_are_consistent():
    rows = _rows()
    for base, others in (("T1_longcat_qvg", ["T1_longcat_pro", "T1_longcat_qvg_i4", "T1_longcat_pro_i4"]),
                         ("T1_hy_qvg", ["T1_hy_pro"])):
        N = _solve_N(rows[base])                 # the chunk length the QVG row implies
        assert 20_000 < N < 80_000               # tens of thousands of tokens, as Sec. 5 describes
        for o in others:
            r = rows[o]
            assert abs(_ratio(N, r) - r["ratio"]) <= r["tol"], (o, _ratio(N, r))


def test_codes_dominate_the_footprint():
    """Sec. 5 "Memory usage breakdown": quantized values are >= 65 % of the stored bytes."""
    for S, B in ((1, 64), (4, 16)):
        for bits in (2, 4):
            N = 37440
            total = O.chunk_bytes(N, D, 256, B, S, 1, bits, 1.0, 8.0)
            codes = N * D * bits / 8
            assert codes / total >= (0.65 if S == 1 else 0.60)


def test_this_builds_format_bytes_per_vector():
    # fp16 scales, uint8 ids, T code sets: T*(d/4 + 2*d/B) + 1 bytes per token + table share
    for (K, T, B, N, want) in ((16, 2, 64, 4096, 73), (64, 3, 32, 4680, 121), (256, 2, 64, 4680, 73),
                               (128, 3, 32, 10800, 121), (256, 4, 64, 4680, 145)):
        total = O.chunk_bytes(N, D, K, B, 1, T, 2, 2.0, 8.0)
        assert total == N * want + K * D * 2


def test_table5_codebook_size_sweep():
    """Table 5 (ratio against K = 64 .. 512, 4-bit and 2-bit levels): all eight printed ratios follow
    from ONE chunk length when a token costs its levels plus log2(K) id bits and a chunk its K x d
    bf16 table (scales are not in these figures: with a byte per group no chunk length comes
    within 0.2 of them).  This fixes how the size arithmetic counts ids (bits, not whole bytes)
    and tables (2 bytes per entry), and that 512 centroids cost 9 bits per token."""
    rows = [tuple(float(v) for v in line.split()) for line in
            open(os.path.join(os.path.dirname(__file__), "golden", "paper_table5_codebook_size.txt"))
            if line.strip() and not line.startswith("#")]
    assert [int(r[0]) for r in rows] == [512, 256, 128, 64]

    def ratio(N, K, bits, scale_bytes=0.0):
        return N * D * 2 / O.chunk_bytes(N, D, int(K), 64, 1, 1, bits, scale_bytes, math.log2(K))

    # the chunk length the (K = 256, 2-bit) entry implies
    lo, hi = 1000, 10_000_000
    while hi - lo > 1:
        mid = (lo + hi) // 2
        lo, hi = (mid, hi) if ratio(mid, 256, 2) < 7.539 else (lo, mid)
    N = hi
    assert 20_000 < N < 200_000
    for K, r4, r2 in rows:
        assert abs(ratio(N, K, 4) - r4) <= 0.01, (K, ratio(N, K, 4))
        assert abs(ratio(N, K, 2) - r2) <= 0.01, (K, ratio(N, K, 2))
    # a dropped table term, whole-byte ids at K = 512 or a byte of scale per group would all miss
    assert abs(N * D * 2 / (N * (32 + 9 / 8)) - 7.307) > 0.2
    assert abs(N * D * 2 / O.chunk_bytes(N, D, 512, 64, 1, 1, 2, 0.0, 16.0) - 7.307) > 0.1
    assert min(abs(ratio(n, 256, 2, 1.0) - 7.539) for n in (N // 2, N, 2 * N, 100 * N)) > 0.2
