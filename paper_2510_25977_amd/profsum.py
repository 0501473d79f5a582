"""Turn rocprofv3 CSV output of a run of ``bench.py`` into the short text summaries kept under ``profiles/``.

    python -m paper_2510_25977_amd.profsum stats   <dir>                 # --kernel-trace run: calls, avg / min / max
    python -m paper_2510_25977_amd.profsum traffic <fetch_dir> <write_dir>   # --pmc FETCH_SIZE and --pmc WRITE_SIZE runs
    python -m paper_2510_25977_amd.profsum counters <dir> [<dir> ...]    # any --pmc run: per-kernel averages
    python -m paper_2510_25977_amd.profsum roofs   <dir>                 # --kernel-trace run of `bench.py --roofs`: the
                                                                         # roof kernels' durations and the rates they mean
    python -m paper_2510_25977_amd.profsum derived <dir> [<dir> ...]     # --pmc runs that together hold the counters
                                                                         # below: per-kernel derived figures

``traffic`` scales both counters by what they read for the plain device copy of known size that
``bench.py --copy-calibration`` adds to the run (torch's copy kernel, 256 MiB read and written per launch).
Kernel names are shortened to the names the library's own per-kernel timing uses (k_gate_up, k_stream_d2, ...).
"""
from __future__ import annotations

import collections
import csv
import glob
import re
import statistics
import sys

COPY_BYTES = 256 << 20
N_CU, N_XCD = 256, 8
STREAM_PHASE = {"0": "d1", "1": "d2", "2": "d4", "3": "d5"}


def short_name(name: str) -> str:
    n = re.sub(r"^void ", "", name).split("(")[0].replace("svdmlp::", "")
    m = re.match(r"k_stream(16)?<(\d)", n)
    if m:
        return "k_stream_" + STREAM_PHASE.get(m.group(2), m.group(2))
    m = re.match(r"(k_roof_(?:mfma|pingpong))<(\d)", n)
    if m:
        return m.group(1) + "_" + {"0": "zero", "1": "constant", "2": "random"}[m.group(2)] + "_operands"
    m = re.match(r"(k_[a-z0-9_]+)", n)
    if m:
        return m.group(1)
    if "copyBuffer" in n:
        return "copy(calibration)"
    return n[:48]


def _csv(d: str, suffix: str):
    fs = glob.glob(d + "/**/*" + suffix, recursive=True)
    if not fs:
        raise SystemExit(f"no *{suffix} under {d}")
    for f in fs:
        with open(f) as fh:
            yield from csv.DictReader(fh)


def kernel_stats(d: str):
    dur = collections.defaultdict(list)
    for r in _csv(d, "kernel_trace.csv"):
        dur[short_name(r["Kernel_Name"])].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    return dur


def counter_means(d: str):
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in _csv(d, "counter_collection.csv"):
        acc[short_name(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return {k: {c: statistics.fmean(v) for c, v in cs.items()} for k, cs in acc.items()}, \
           {k: max(len(v) for v in cs.values()) for k, cs in acc.items()}


def is_ours(k: str) -> bool:
    return k.startswith("k_") and k != "k_repack" and not k.startswith("k_roof")


def cmd_stats(d: str) -> None:
    dur = kernel_stats(d)
    total = sum(sum(v) for k, v in dur.items() if is_ours(k))
    print("per kernel (microseconds; every launch of the run, warm-up included):")
    for k, v in sorted(dur.items(), key=lambda kv: -sum(kv[1])):
        if is_ours(k):
            print(f"  {k:14s} calls {len(v):5d}  avg {statistics.fmean(v):8.1f}  median {statistics.median(v):8.1f}  "
                  f"min {min(v):8.1f}  max {max(v):8.1f}  {100 * sum(v) / total:5.1f} %")


def cmd_roofs(d: str) -> None:
    """Durations of the roof kernels of one `bench.py --roofs` run by the profiler's clock, and the MFMA rates they
    mean (bench.py's iteration counts: 8000 iterations x 4 MFMAs per wave for k_roof_mfma, 4000 steps x 16 MFMAs for
    k_roof_pingpong; eight waves per workgroup, one workgroup per CU, 32768 FLOP per MFMA)."""
    dur = kernel_stats(d)
    flop = {"k_roof_mfma": N_CU * 8 * 4 * 8000 * 32768, "k_roof_pingpong": N_CU * 8 * 16 * 4000 * 32768}
    print("roof kernels (microseconds; every launch of the run):")
    for k, v in sorted(dur.items()):
        if not k.startswith("k_roof"):
            continue
        line = f"  {k:40s} calls {len(v):5d}  median {statistics.median(v):10.1f}  min {min(v):10.1f}"
        for base, fl in flop.items():
            if k.startswith(base + "_"):
                line += f"   {fl / statistics.median(v) / 1e6:7.0f} TFLOP/s (median), {fl / min(v) / 1e6:7.0f} (best)"
        print(line)


def cmd_traffic(fetch_dir: str, write_dir: str) -> None:
    f, _ = counter_means(fetch_dir)
    w, _ = counter_means(write_dir)
    cf = f.get("copy(calibration)", {}).get("FETCH_SIZE")
    cw = w.get("copy(calibration)", {}).get("WRITE_SIZE")
    if not cf or not cw:
        raise SystemExit("no calibration copy in the run (bench.py --copy-calibration)")
    sf, sw = COPY_BYTES / 1024 / cf, COPY_BYTES / 1024 / cw
    print(f"calibration: plain {COPY_BYTES >> 20} MiB device copy: FETCH_SIZE reads {cf:.0f} KiB -> scale {sf:.3f}; "
          f"WRITE_SIZE reads {cw:.0f} KiB -> scale {sw:.3f}")
    print("per launch (averages), HBM-side bytes = counter x scale x 1024:")
    tr = tw = 0.0
    for k in f:
        if is_ours(k) and k in w:
            rmb, wmb = f[k]["FETCH_SIZE"] * sf * 1024 / 1e6, w[k]["WRITE_SIZE"] * sw * 1024 / 1e6
            tr, tw = tr + rmb, tw + wmb
            print(f"  {k:14s} FETCH_SIZE {f[k]['FETCH_SIZE']:9.0f}  WRITE_SIZE {w[k]['WRITE_SIZE']:9.0f}   "
                  f"read {rmb:8.1f} MB  written {wmb:8.1f} MB")
    print(f"  {'whole forward':14s} read {tr:8.1f} MB  written {tw:8.1f} MB  together {tr + tw:8.1f} MB")


def cmd_counters(dirs) -> None:
    for d in dirs:
        means, n = counter_means(d)
        for k, cs in means.items():
            if is_ours(k):
                print(f"  {k:14s} (n={n[k]:3d}) " + "  ".join(f"{c} {v:.4g}" for c, v in sorted(cs.items())))


def cmd_derived(dirs) -> None:
    """Per kernel, from counters spread over several runs (averages per launch):
       cycles        GRBM_GUI_ACTIVE / 8 XCDs: active clocks of the launch
       mfma_busy     SQ_VALU_MFMA_BUSY_CYCLES / (4 SIMDs x 256 CUs) / cycles
       coexec        SQ_VALU_MFMA_COEXEC_CYCLES / SQ_VALU_MFMA_BUSY_CYCLES: share of the matrix-core time with a vector-ALU
                     instruction issued beside it
       lds_conflict  SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE
       l2_miss       TCC_MISS / (TCC_HIT + TCC_MISS), stores included
       fetch         TCP_TCC_READ_REQ x 128 B / (256 CUs x cycles): bytes per clock a CU pulls in from L2
       latency       TCP_TCC_READ_REQ_LATENCY / TCP_TCC_READ_REQ, clocks
       in_flight     fetch x latency / 128 B: 128-byte lines a CU has outstanding at L2 on average (Little's law)"""
    acc = collections.defaultdict(dict)
    for d in dirs:
        means, _ = counter_means(d)
        for k, cs in means.items():
            acc[k].update(cs)
    print("derived per kernel (see `profsum derived --help` text in the module for the formulas):")
    for k, c in acc.items():
        if not is_ours(k) or "GRBM_GUI_ACTIVE" not in c:
            continue
        cyc = c["GRBM_GUI_ACTIVE"] / N_XCD
        out = [f"cycles {cyc:9.0f}"]
        if "SQ_VALU_MFMA_BUSY_CYCLES" in c:
            busy = c["SQ_VALU_MFMA_BUSY_CYCLES"]
            out.append(f"mfma_busy {busy / (4 * N_CU) / cyc:5.3f}")
            if busy and "SQ_VALU_MFMA_COEXEC_CYCLES" in c:
                out.append(f"coexec {c['SQ_VALU_MFMA_COEXEC_CYCLES'] / busy:5.3f}")
        if c.get("SQ_LDS_IDX_ACTIVE"):
            out.append(f"lds_conflict {c.get('SQ_LDS_BANK_CONFLICT', 0.0) / c['SQ_LDS_IDX_ACTIVE']:5.3f}")
        if "TCC_HIT_sum" in c and c["TCC_HIT_sum"] + c["TCC_MISS_sum"] > 0:
            out.append(f"l2_miss {c['TCC_MISS_sum'] / (c['TCC_HIT_sum'] + c['TCC_MISS_sum']):5.3f}")
        if c.get("TCP_TCC_READ_REQ_sum"):
            fetch = c["TCP_TCC_READ_REQ_sum"] * 128.0 / (N_CU * cyc)
            lat = c["TCP_TCC_READ_REQ_LATENCY_sum"] / c["TCP_TCC_READ_REQ_sum"]
            out.append(f"fetch {fetch:5.1f} B/clk/CU  latency {lat:6.0f} clk  in_flight {fetch * lat / 128.0:5.1f} lines/CU")
        print(f"  {k:14s} " + "  ".join(out))


def main(argv) -> None:
    if len(argv) >= 3 and argv[1] == "stats":
        cmd_stats(argv[2])
    elif len(argv) >= 4 and argv[1] == "traffic":
        cmd_traffic(argv[2], argv[3])
    elif len(argv) >= 3 and argv[1] == "counters":
        cmd_counters(argv[2:])
    elif len(argv) >= 3 and argv[1] == "roofs":
        cmd_roofs(argv[2])
    elif len(argv) >= 3 and argv[1] == "derived":
        cmd_derived(argv[2:])
    else:
        raise SystemExit(__doc__)


if __name__ == "__main__":
    main(sys.argv)
