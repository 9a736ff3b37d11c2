"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

    python -m paper_2510_10129_amd.rocprof_summary stats   <kernel_stats.csv> --cmd "<command>"
    python -m paper_2510_10129_amd.rocprof_summary traffic <fetch_counter_collection.csv> \
           <write_counter_collection.csv> --calib-bytes N --cmd "<commands>"

`traffic` reads two counter-collection runs of the same program (FETCH_SIZE in one,
WRITE_SIZE in the other; KiB per dispatch), averages them per kernel, and scales each
counter by the factor that makes it read `calib-bytes` for the library's plain copy
kernel (cc_calib_copy), which the profiled program must have launched once.
"""
from __future__ import annotations

import argparse
import collections
import csv
import re
import sys

KINDS = (
    # the pieces of split launches first: their names also contain an epilogue's or a kernel's name
    ("splitk_finish_kernel", "splitk_finish"), ("EpiPartial", "splitk_share"), ("attn_merge_kernel", "attn_merge"),
    ("EpiGateUp", "gate_up"), ("EpiDown", "down"), ("EpiQKV", "qkv"), ("EpiOProj", "oproj"),
    ("sparse_attn_kernel", "attn"), ("gather_rmsnorm_kernel", "gather_norm"),
    ("rmsnorm_f32_kernel", "post_norm"), ("colsum_kernel", "colsum"), ("select_kernel", "select"),
    ("calib_copy_kernel", "calib_copy"), ("assemble_kernel", "assemble"),
    ("block_scores_kernel", "block_scores"),
)


def kind_of(kernel_name: str):
    for pat, kind in KINDS:
        if pat in kernel_name:
            return kind
    return None


def short(name: str, width: int = 100) -> str:
    name = re.sub(r"\(anonymous namespace\)::", "", name).replace("bool _Accum", "bf16")
    return name if len(name) <= width else name[: width - 3] + "..."


def stats(path: str, cmd: str) -> str:
    rows = list(csv.DictReader(open(path)))
    out = [f"command: {cmd}", "source: rocprofv3 --kernel-trace --stats (kernel_stats.csv); durations in microseconds", "",
           f"{'calls':>6} {'total_us':>12} {'avg_us':>10} {'%':>6}  kind         kernel"]
    for r in rows:
        name = r.get("Name") or r.get("KernelName") or ""
        calls = int(float(r["Calls"]))
        tot = float(r["TotalDurationNs"]) / 1e3
        avg = float(r["AverageNs"]) / 1e3
        pct = float(r["Percentage"])
        kind = kind_of(name)
        if kind is None and pct < 0.5:
            continue
        out.append(f"{calls:6d} {tot:12.1f} {avg:10.2f} {pct:6.2f}  {kind or '-':12s} {short(name)}")
    return "\n".join(out) + "\n"


def _per_kernel(path: str, counter: str):
    acc = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != counter:
            continue
        kind = kind_of(r["Kernel_Name"])
        if kind:
            acc[kind].append(float(r["Counter_Value"]))
    return {k: (sum(v) / len(v), len(v)) for k, v in acc.items()}


def traffic(fetch_csv: str, write_csv: str, calib_bytes: int, cmd: str) -> str:
    f = _per_kernel(fetch_csv, "FETCH_SIZE")
    w = _per_kernel(write_csv, "WRITE_SIZE")
    if "calib_copy" not in f or "calib_copy" not in w:
        raise SystemExit("the profiled run did not launch the calibration copy kernel")
    kf = calib_bytes / (f["calib_copy"][0] * 1024.0)
    kw = calib_bytes / (w["calib_copy"][0] * 1024.0)
    out = [f"command: {cmd}",
           "source: rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE (KiB per dispatch), averaged per kernel",
           f"calibration: cc_calib_copy of {calib_bytes} bytes reads FETCH_SIZE {f['calib_copy'][0]:.0f} KiB, "
           f"WRITE_SIZE {w['calib_copy'][0]:.0f} KiB -> scale factors {kf:.4f} (fetch), {kw:.4f} (write)", "",
           f"{'kind':12s} {'launches':>8} {'fetch_KiB':>12} {'write_KiB':>12} {'scaled_MB_per_launch':>22}"]
    for kind in sorted(set(f) | set(w)):
        fk, n = f.get(kind, (0.0, 0))
        wk, _ = w.get(kind, (0.0, 0))
        total = fk * 1024.0 * kf + wk * 1024.0 * kw
        out.append(f"{kind:12s} {n:8d} {fk:12.0f} {wk:12.0f} {total / 1e6:22.2f}")
        out.append(f"traffic_bytes_per_launch[{kind}]: {total:.0f}")
    return "\n".join(out) + "\n"


def mfma(path: str, cmd: str) -> str:
    """Matrix-pipe utilisation per kernel from SQ counters: SQ_VALU_MFMA_BUSY_CYCLES counts busy
    cycles per SIMD, SQ_BUSY_CU_CYCLES busy cycles per CU (4 SIMDs each)."""
    names = ("SQ_VALU_MFMA_BUSY_CYCLES", "SQ_BUSY_CU_CYCLES", "SQ_INSTS_MFMA", "SQ_ACTIVE_INST_VALU",
             "SQ_ACTIVE_INST_LDS", "SQ_WAVE_CYCLES")
    per = {n: _per_kernel(path, n) for n in names}
    out = [f"command: {cmd}",
           "source: rocprofv3 --pmc (SQ counters, summed over the chip per dispatch), averaged per kernel;",
           "mfma_util = SQ_VALU_MFMA_BUSY_CYCLES / (4 * SQ_BUSY_CU_CYCLES): share of the cycles in which a CU",
           "runs a wave during which a SIMD's matrix pipe is busy (in clocks, at whatever clock the card ran)", "",
           f"{'kind':12s} {'launches':>8} {'mfma_busy_Mcyc':>15} {'cu_busy_Mcyc':>13} {'mfma_insts_M':>13} {'mfma_util':>10}"]
    for kind in sorted(per["SQ_BUSY_CU_CYCLES"]):
        busy, n = per["SQ_VALU_MFMA_BUSY_CYCLES"].get(kind, (0.0, 0))
        cu, _ = per["SQ_BUSY_CU_CYCLES"][kind]
        insts, _ = per["SQ_INSTS_MFMA"].get(kind, (0.0, 0))
        util = busy / (4.0 * cu) if cu else 0.0
        out.append(f"{kind:12s} {n:8d} {busy / 1e6:15.1f} {cu / 1e6:13.1f} {insts / 1e6:13.2f} {util:10.3f}")
    return "\n".join(out) + "\n"


def read_traffic(path: str):
    """Parses the `traffic_bytes_per_launch[kind]: N` lines of a summary written by `traffic`."""
    res = {}
    try:
        for line in open(path):
            m = re.match(r"traffic_bytes_per_launch\[(\w+)\]: (\d+)", line)
            if m:
                res[m.group(1)] = int(m.group(2))
    except OSError:
        pass
    return res


def main():
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="what", required=True)
    a = sub.add_parser("stats")
    a.add_argument("csv")
    a.add_argument("--cmd", required=True)
    b = sub.add_parser("traffic")
    b.add_argument("fetch_csv")
    b.add_argument("write_csv")
    b.add_argument("--calib-bytes", type=int, required=True)
    b.add_argument("--cmd", required=True)
    m = sub.add_parser("mfma")
    m.add_argument("csv")
    m.add_argument("--cmd", required=True)
    args = ap.parse_args()
    if args.what == "stats":
        sys.stdout.write(stats(args.csv, args.cmd))
    elif args.what == "mfma":
        sys.stdout.write(mfma(args.csv, args.cmd))
    else:
        sys.stdout.write(traffic(args.fetch_csv, args.write_csv, args.calib_bytes, args.cmd))


if __name__ == "__main__":
    main()
