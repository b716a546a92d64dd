"""Short text summaries of rocprofv3 CSV output for the kernels of libqvg.

    python -m paper_2602_02958_amd.profsum stats   <dir> [--top N]
    python -m paper_2602_02958_amd.profsum counters <dir> [<dir> ...]
    python -m paper_2602_02958_amd.profsum derived <kernel substring> <dir> [<dir> ...]
    python -m paper_2602_02958_amd.profsum traffic <workload> <part> <kernel substring>[*n][,<substring>[*n]..]
                                                   <fetch dir> <write dir> <copy fetch dir> <copy write dir>

`derived` turns the raw counters of the kernels matching the substring into busy fractions of the
chip's 1024 SIMDs (GRBM_GUI_ACTIVE is summed over the 8 XCDs; SQ_ACTIVE_INST_* count issue slots of
4 cycles).  `stats` prints the kernel table of a `--kernel-trace --stats` run; `counters` prints, per library
kernel, the average of every counter a `--pmc` run collected (counters are summed over the
dispatch's workgroups); `traffic` prints one line `<workload> <part> fetch_bytes=.. write_bytes=..`
for profiles/hbm_traffic.txt, scaling FETCH_SIZE / WRITE_SIZE (KiB per dispatch) by what the same
counters read for the plain 1 GiB device copy of `bench.py --only copy`; a part made of several
kernels, each launched n times per call, is given as `a*n,b*n` and its bytes are summed.
Measurement bookkeeping only: nothing of the codec is computed here.
"""
from __future__ import annotations

import collections
import csv
import glob
import os
import sys

COPY_BYTES = 1 << 30


def _one(dir_, suffix):
    files = sorted(glob.glob(os.path.join(dir_, "**", "*" + suffix), recursive=True))
    if not files:
        raise FileNotFoundError(f"no *{suffix} under {dir_}")
    return files[0]


def short(name, width=72):
    return name.replace("void ", "")[:width]


def stats(dir_, top=10):
    rows = list(csv.DictReader(open(_one(dir_, "kernel_stats.csv"))))
    out = [f"{'kernel':<72} {'calls':>6} {'avg_us':>10} {'total_ms':>10} {'pct':>6}"]
    for r in rows[:top]:
        out.append(f"{short(r['Name']):<72} {int(r['Calls']):>6} {float(r['AverageNs']) / 1e3:>10.2f} "
                   f"{float(r['TotalDurationNs']) / 1e6:>10.3f} {float(r['Percentage']):>6.2f}")
    return "\n".join(out)


def counter_means(dir_, only_lib=True):
    """{kernel name: {counter: (mean per dispatch, dispatches)}}"""
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(_one(dir_, "counter_collection.csv"))):
        k = r["Kernel_Name"]
        if only_lib and "qvg::" not in k and "copyBuffer" not in k:
            continue
        acc[k][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return {k: {c: (sum(v) / len(v), len(v)) for c, v in d.items()} for k, d in acc.items()}


def counters(dirs):
    out = []
    for d in dirs:
        for k, cs in sorted(counter_means(d).items()):
            for c, (m, n) in sorted(cs.items()):
                out.append(f"{short(k, 60):<60} {c:<28} {m:>16.1f}  ({n} dispatches)")
    return "\n".join(out)


def derived(needle, dirs):
    out = []
    merged = collections.defaultdict(dict)
    for d in dirs:
        for k, cs in counter_means(d).items():
            if needle in k:
                merged[k].update({c: m for c, (m, n) in cs.items()})
    for k, c in sorted(merged.items()):
        out.append(short(k, 100))
        if "GRBM_GUI_ACTIVE" not in c:
            continue
        cyc = c["GRBM_GUI_ACTIVE"] / 8.0
        simd = cyc * 1024.0
        out.append(f"  cycles per launch {cyc:,.0f}  (x 1024 SIMDs = {simd:,.0f} SIMD-cycles)")
        def pct(name, mul=1.0, label=None):
            if name in c:
                out.append(f"  {label or name:<44} {c[name] * mul / simd * 100:6.1f} % of SIMD-cycles   ({name} = {c[name]:,.0f})")
        pct("SQ_VALU_MFMA_BUSY_CYCLES", 1.0, "matrix pipe busy")
        pct("SQ_ACTIVE_INST_VALU", 4.0, "VALU issue (incl. MFMA issue slots)")
        pct("SQ_ACTIVE_INST_SCA", 4.0, "scalar issue")
        pct("SQ_ACTIVE_INST_LDS", 4.0, "LDS issue")
        pct("SQ_WAVE_CYCLES", 4.0, "resident wavefronts x 100 %")
        for name in ("SQ_INSTS_VALU", "SQ_INSTS_SALU", "SQ_INSTS_LDS", "SQ_INSTS_VALU_MFMA_MOPS_BF16",
                     "SQ_INSTS_VALU_MFMA_MOPS_F16", "SQ_WAIT_INST_ANY", "SQ_WAIT_INST_LDS", "SQ_ACTIVE_INST_ANY"):
            if name in c:
                out.append(f"  {name:<44} {c[name]:,.0f}")
        if "SQ_LDS_BANK_CONFLICT" in c and c.get("SQ_LDS_IDX_ACTIVE"):
            out.append(f"  LDS bank-conflict cycles / LDS active cycles  {c['SQ_LDS_BANK_CONFLICT'] / c['SQ_LDS_IDX_ACTIVE'] * 100:6.1f} %")
    return "\n".join(out)


def _kib(dir_, counter, needle):
    best = None
    for k, cs in counter_means(dir_).items():
        if needle in k and counter in cs:
            # the kernel with the most dispatches wins when the substring matches several instances
            if best is None or cs[counter][1] > best[1]:
                best = cs[counter]
    if best is None:
        raise KeyError(f"{counter} of a kernel matching {needle!r} not found under {dir_}")
    return best[0]


def traffic(workload, part, needle, fetch_dir, write_dir, copy_fetch_dir, copy_write_dir):
    f_scale = COPY_BYTES / (_kib(copy_fetch_dir, "FETCH_SIZE", "copyBuffer") * 1024.0)
    w_scale = COPY_BYTES / (_kib(copy_write_dir, "WRITE_SIZE", "copyBuffer") * 1024.0)
    fb = wb = 0.0
    for item in needle.split(","):
        name, _, times = item.partition("*")
        n = float(times) if times else 1.0
        fb += n * _kib(fetch_dir, "FETCH_SIZE", name) * 1024.0 * f_scale
        wb += n * _kib(write_dir, "WRITE_SIZE", name) * 1024.0 * w_scale
    return (f"{workload} {part} fetch_bytes={int(round(fb))} write_bytes={int(round(wb))} "
            f"kernel={needle} fetch_scale={f_scale:.3f} write_scale={w_scale:.3f}")


def main(argv):
    if len(argv) < 2:
        print(__doc__)
        return 2
    if argv[0] == "stats":
        top = int(argv[argv.index("--top") + 1]) if "--top" in argv else 10
        print(stats(argv[1], top))
    elif argv[0] == "counters":
        print(counters(argv[1:]))
    elif argv[0] == "derived":
        print(derived(argv[1], argv[2:]))
    elif argv[0] == "traffic":
        print(traffic(*argv[1:8]))
    else:
        print(__doc__)
        return 2
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
