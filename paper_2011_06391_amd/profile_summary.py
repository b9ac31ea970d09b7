"""Turn rocprofv3 CSV output into the short summaries kept under profiles/ and into the row of
profiles/hbm_traffic_per_launch.txt that bench.py prices its roofline fraction on.

    python -m paper_2011_06391_amd.profile_summary BASE WORKLOAD

BASE is a directory that holds, for workload W (c2 ... c5), the output of these commands, all run from
the repository root on the MI355X machine (one counter group per run; the program follows `--` directly):

    rocprofv3 --kernel-trace --stats --output-format csv -d BASE/stats_W -o stats -- \
        python3 bench.py --workload W --no-cpu-baseline --no-context        > BASE/stats_W.log
    rocprofv3 --pmc FETCH_SIZE --output-format csv -d BASE/pmc_FETCH_SIZE_W -o pmc -- \
        python3 bench.py --workload W --steps 3 --warmup 1 --no-cpu-baseline --no-context --copy-calibration-mib 1024 \
                                                                            > BASE/pmc_FETCH_SIZE_W.log
    rocprofv3 --pmc WRITE_SIZE ...  (same command)                          > BASE/pmc_WRITE_SIZE_W.log
    rocprofv3 --pmc TCC_HIT_sum TCC_MISS_sum TCC_REQ_sum --output-format csv -d BASE/pmc_tcc_W -o pmc -- \
        python3 bench.py --workload W --steps 3 --warmup 1 --no-cpu-baseline --no-context

FETCH_SIZE and WRITE_SIZE count requests between the L2s and the memory fabric in KiB per dispatch; each is
scaled by what the same counter reads for the plain copy kernel of known size launched by
--copy-calibration-mib.  Host-side text processing only: nothing here touches the GPU or the library.
"""
from __future__ import annotations

import collections
import csv
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
TABLE = os.path.join(ROOT, "profiles", "hbm_traffic_per_launch.txt")
TABLE_HEADER = """# L2 <-> fabric bytes per launch of the main kernel (fusedmm_fast_kernel), read by bench.py.
# A row counts only for the build whose kernel sources hash to its second field and for the plan whose
# statistics it names; otherwise bench.py reports traffic = null and says why.  Written by
# `python -m paper_2011_06391_amd.profile_summary` from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# (commands in profiles/fusedmm_fast_kernel_<workload>.md), each counter scaled by its reading for the copy kernel.
# workload  kernel_sources_sha16  partial_rows  tile_segments  column_classes  fetch_bytes  write_bytes  l2_hit_rate  commit
"""


def _short(name: str) -> str:
    return name.split("(")[0]


def _bench_line(path: str) -> dict:
    lines = [json.loads(l) for l in open(path) if l.startswith("{")]
    if not lines:
        raise SystemExit(f"{path}: no bench.py JSON line")
    return lines[-1]


def _pmc(path: str) -> dict:
    """{counter: {kernel: (launches, average value per launch)}}"""
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(path)):
        if "fmm::" in r["Kernel_Name"]:
            agg[r["Counter_Name"]][_short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    return {c: {k: (len(v), sum(v) / len(v)) for k, v in ks.items()} for c, ks in agg.items()}


def summarise(base: str, w: str) -> str:
    bl = _bench_line(os.path.join(base, f"stats_{w}.log"))
    cfg, roof = bl["config"], bl["roofline"]
    desc = (f"{cfg['description']}; n={cfg['n']}, nnz={cfg['nnz']}, d={cfg['d']}, pattern {cfg['pattern']}; default plan: "
            f"{cfg['plan']['column_classes']} finest column classes, {cfg['plan']['partials']} partial rows")
    out = [f"# fusedmm_fast_kernel on workload {w} ({desc})", "", "## Kernel durations", "",
           "Command (run from the repository root on the MI355X box):", "",
           f"    rocprofv3 --kernel-trace --stats --output-format csv -d {base}/stats_{w} -o stats -- python3 bench.py "
           f"--workload {w} --no-cpu-baseline --no-context", "",
           "| kernel | calls | average ns | min ns | max ns | % of GPU time |", "|---|---|---|---|---|---|"]
    for r in csv.DictReader(open(os.path.join(base, f"stats_{w}", "stats_kernel_stats.csv"))):
        if "fmm::" in r["Name"]:
            out.append(f"| `{_short(r['Name'])}` | {r['Calls']} | {float(r['AverageNs']):.0f} | {r['MinNs']} | {r['MaxNs']} | "
                       f"{float(r['Percentage']):.2f} |")
    steps, warm = bl["steps"], bl["warmup"]
    out += ["", f"bench.py's own figures in the same run ({warm} warm-up, {steps} timed, {steps} event-bracketed executes): "
                f"kernel_ms = {roof['kernel_ms']:.4f} (HIP events around the main kernel, empty bracket subtracted), "
                f"ms_per_step = {bl['ms_per_step']:.4f}, value = {bl['value']:.1f} G(edge*dim)/s.", ""]
    tr = [r for r in csv.DictReader(open(os.path.join(base, f"stats_{w}", "stats_kernel_trace.csv")))
          if "fusedmm_fast_kernel" in r["Kernel_Name"]]
    tr.sort(key=lambda r: int(r["Start_Timestamp"]))
    dur = [int(r["End_Timestamp"]) - int(r["Start_Timestamp"]) for r in tr]
    if len(dur) == 1 + warm + 2 * steps:
        dur = dur[1:]  # the first execute right after plan creation
        seg = lambda a, b: sum(dur[a:b]) / max(1, b - a)
        out += [f"Main kernel, average ns per phase of the run (kernel trace, dispatches in start order, after the first "
                f"execute): warm-up {seg(0, warm):.0f}, timed region {seg(warm, warm + steps):.0f}, event-bracketed pass "
                f"{seg(warm + steps, warm + 2 * steps):.0f} (the pass bench.py's kernel_ms measures).", ""]
    f = _pmc(os.path.join(base, f"pmc_FETCH_SIZE_{w}", "pmc_counter_collection.csv"))["FETCH_SIZE"]
    wr = _pmc(os.path.join(base, f"pmc_WRITE_SIZE_{w}", "pmc_counter_collection.csv"))["WRITE_SIZE"]
    out += ["## L2 <-> fabric traffic (requests of the L2s to the fabric: served by Infinity Cache or HBM)", "",
            "Commands (one counter per run):", "",
            f"    rocprofv3 --pmc FETCH_SIZE --output-format csv -d {base}/pmc_FETCH_SIZE_{w} -o pmc -- python3 bench.py "
            f"--workload {w} --steps 3 --warmup 1 --no-cpu-baseline --no-context --copy-calibration-mib 1024",
            f"    rocprofv3 --pmc WRITE_SIZE --output-format csv -d {base}/pmc_WRITE_SIZE_{w} -o pmc -- python3 bench.py "
            f"--workload {w} --steps 3 --warmup 1 --no-cpu-baseline --no-context --copy-calibration-mib 1024", "",
            "| kernel | launches | FETCH_SIZE KiB/launch | WRITE_SIZE KiB/launch |", "|---|---|---|---|"]
    for k in f:
        out.append(f"| `{k}` | {f[k][0]} | {f[k][1]:.1f} | {wr.get(k, (0, 0.0))[1]:.1f} |")
    cf = [v for k, v in f.items() if "copy" in k][0][1]
    cw = [v for k, v in wr.items() if "copy" in k][0][1]
    pl = _bench_line(os.path.join(base, f"pmc_FETCH_SIZE_{w}.log"))
    copy_kib = pl["config"]["copy_calibration_bytes_each_way"] / 1024.0
    sf, sw = copy_kib / cf, copy_kib / cw
    mf = [v for k, v in f.items() if "fusedmm_fast_kernel" in k][0][1]
    mw = [v for k, v in wr.items() if "fusedmm_fast_kernel" in k][0][1]
    fetch_b, write_b = int(mf * sf * 1024), int(mw * sw * 1024)
    tb = fetch_b + write_b
    out += ["", f"Calibration: `fusedmm_copy_kernel` moves exactly {copy_kib:.0f} KiB each way; the counters read {cf:.1f} "
                f"(fetch) and {cw:.1f} (write) KiB, so the scale factors are {sf:.3f} (FETCH_SIZE) and {sw:.3f} (WRITE_SIZE).",
            f"Main kernel traffic per launch = {mf:.0f}*{sf:.3f} + {mw:.0f}*{sw:.3f} KiB = {tb / 1e9:.3f} GB ({tb} bytes) = "
            f"{tb / (roof['kernel_ms'] * 1e-3) / 1e12:.2f} TB/s over kernel_ms, against {roof['algorithmic_bytes'] / 1e9:.3f} GB "
            f"of algorithmic bytes and {roof['compulsory_bytes'] / 1e9:.3f} GB compulsory.", ""]
    hit = 0.0
    tcc_path = os.path.join(base, f"pmc_tcc_{w}", "pmc_counter_collection.csv")
    if os.path.exists(tcc_path):
        t = _pmc(tcc_path)
        main = [k for k in t.get("TCC_REQ_sum", {}) if "fusedmm_fast_kernel" in k]
        if main:
            k = main[0]
            req, h, mi = t["TCC_REQ_sum"][k][1], t["TCC_HIT_sum"][k][1], t["TCC_MISS_sum"][k][1]
            hit = h / max(1.0, h + mi)
            out += ["## L2 hit rate", "", "Command:", "",
                    f"    rocprofv3 --pmc TCC_HIT_sum TCC_MISS_sum TCC_REQ_sum --output-format csv -d {base}/pmc_tcc_{w} -o pmc -- "
                    f"python3 bench.py --workload {w} --steps 3 --warmup 1 --no-cpu-baseline --no-context", "",
                    f"Main kernel, per launch: TCC_REQ {req:.0f}, TCC_HIT {h:.0f}, TCC_MISS {mi:.0f} (128-byte lines): hit rate "
                    f"{hit:.3f}, miss bytes {mi * 128 / 1e9:.2f} GB.", ""]
    # the table row belongs to the build and plan of the counter run
    for other in (pl, _bench_line(os.path.join(base, f"pmc_WRITE_SIZE_{w}.log"))):
        if other["config"]["plan"] != cfg["plan"] or other["config"]["kernel_sources_sha16"] != cfg["kernel_sources_sha16"]:
            raise SystemExit("the runs under BASE were not made with one build and one plan")
    try:
        commit = subprocess.run(["git", "-C", ROOT, "rev-parse", "--short=12", "HEAD"], capture_output=True, text=True,
                                check=True).stdout.strip()
    except Exception:
        commit = "unknown"
    row = (f"{w} {cfg['kernel_sources_sha16']} {cfg['plan']['partials']} {cfg['plan']['tile_segments']} "
           f"{cfg['plan']['column_classes']} {fetch_b} {write_b} {hit:.3f} {commit}")
    rows = []
    if os.path.exists(TABLE):
        rows = [l.rstrip("\n") for l in open(TABLE) if l.strip() and not l.startswith("#") and l.split()[0] != w]
    rows.append(row)
    with open(TABLE, "w") as fh:
        fh.write(TABLE_HEADER + "\n".join(sorted(rows)) + "\n")
    path = os.path.join(ROOT, "profiles", f"fusedmm_fast_kernel_{w}.md")
    with open(path, "w") as fh:
        fh.write("\n".join(out))
    return row


if __name__ == "__main__":
    if len(sys.argv) != 3:
        raise SystemExit(__doc__)
    print(summarise(sys.argv[1].rstrip("/"), sys.argv[2]))
