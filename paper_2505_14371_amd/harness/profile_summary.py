"""Turn rocprofv3 CSV output of the qoda_probe driver into the short text summaries kept under profiles/.

    python -m paper_2505_14371_amd.harness.profile_summary --name txl --stats DIR --fetch DIR --write DIR \\
        --probe-log FILE --command "..." --out profiles/

Reads <DIR>/**/*_kernel_stats.csv (from --kernel-trace --stats) and <DIR>/**/*_counter_collection.csv (from
--pmc FETCH_SIZE / --pmc WRITE_SIZE, values in KiB per dispatch).  The byte counters are scaled by what the same
counter reads for the plain copy kernel k_copy_f4, whose true size the probe log states.  Writes
<out>/<name>_kernels.txt and merges the per-kernel traffic into <out>/traffic.json (read by bench.py).

    python -m paper_2505_14371_amd.harness.profile_summary --name txl --sq DIR [DIR ...] --probe-log FILE \
        --command "..." --out profiles/

Reads the counter CSVs of one or more --pmc passes over SQ_* / GRBM_* counters, averages every counter per kernel
class over its dispatches (the warm-up round's left out), and writes <out>/<name>_sq_counters.txt: the raw averages
and, from them and the workload size in the probe log, vector / scalar / LDS instructions per node-coordinate, the
share of cycles the vector ALU and the LDS were busy, and LDS bank-conflict cycles.  The vector instructions per
node-coordinate are merged into <out>/sq_counters.json, from which bench.py derives each kernel's model time.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import re


def _one(pattern: str) -> str:
    hits = glob.glob(pattern, recursive=True)
    if not hits:
        raise SystemExit(f"no file matches {pattern}")
    return max(hits, key=os.path.getmtime)   # a directory reused by several runs: the latest one


def _short(name: str) -> str:
    """Kernel symbol -> the library's kernel class name (qoda_kernel_name): qoda::k_decode<4, 1, false>(qoda::Dev) ->
    k_decode<true>; qoda::k_quantize<4>(...) and qoda::k_quantize_b<4>(...) -> k_quantize; k_sumsq<true> stays."""
    m = re.search(r"(k_[a-z0-9_]+)(<[^>]*>)?", name)
    if not m:
        return name[:60]
    base = m.group(1)
    raw = [a.strip() for a in (m.group(2) or "<>")[1:-1].split(",") if a.strip()]
    if base == "k_decode" and len(raw) >= 2:
        return "k_decode<" + {"0": "false", "1": "true", "2": "alt", "3": "extrapolate"}.get(raw[1], raw[1]) + ">"
    if base in ("k_quantize", "k_quantize_b"):   # whatever the code width, with or without a previous message
        return "k_quantize"
    if base == "k_index_hist":
        return base
    args = [a for a in raw if not a.isdigit()]
    return base + ("<" + ", ".join(args) + ">" if args else "")


def _counters(directory: str):
    rows = csv.DictReader(open(_one(os.path.join(directory, "**", "*_counter_collection.csv"))))
    agg = collections.defaultdict(list)
    for r in rows:
        agg[_short(r["Kernel_Name"])].append(float(r["Counter_Value"]) * 1024.0)
    return agg


def _sq_summary(a):
    log = open(a.probe_log).read()
    m = re.search(r"d=(\d+) K=(\d+)", log)
    node_coords = float(m.group(1)) * float(m.group(2))
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for d in a.sq:
        for f in glob.glob(os.path.join(d, "**", "*_counter_collection.csv"), recursive=True):
            for r in csv.DictReader(open(f)):
                name = r["Kernel_Name"]
                if "qoda::" not in name:
                    continue
                label = _short(name)
                if label == "k_quantize" and re.search(r"k_quantize(_b)?<\d+, false", name):
                    label = "k_quantize (no prev)"
                agg[label][r["Counter_Name"]].append(float(r["Counter_Value"]))
    lines = [f"# rocprofv3 --pmc summary (SQ / GRBM counters): {a.name}", "# command:", "#   " + a.command, "#",
             "# probe output:"] + ["#   " + l for l in log.strip().splitlines()]
    lines += ["#", "# Counters are sums over the device (32 shader engines, 256 CUs, 1024 SIMDs); GRBM_GUI_ACTIVE sums the",
              "# 8 XCDs.  One vector instruction occupies its SIMD for 4 cycles (64 lanes over 16).  Derived columns:",
              "#   valu/nc, int64/nc, salu/nc, lds/nc   instructions x 64 lanes / node-coordinates of one launch",
              "#   valu_cycles   4 x SQ_INSTS_VALU / 1024 SIMDs: cycles a SIMD spends issuing vector instructions",
              "#   kernel_cycles GRBM_GUI_ACTIVE / 8: the launch's duration in the counter's clock",
              "#   valu_share    valu_cycles / kernel_cycles: near 1 = the vector ALUs are saturated (the two counters tick in",
              "#                 different clock domains, so the share can pass 1); valu_ms_2.4GHz = valu_cycles / 2.4e9",
              "#   lds_share     SQ_LDS_IDX_ACTIVE / 256 CUs / kernel_cycles;  conflict = SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE", ""]
    big = {"k_sumsq<true>", "k_sumsq<false>", "k_quantize", "k_quantize (no prev)", "k_decode<true>", "k_decode<alt>"}
    valu_per = {}
    for k in sorted(agg):
        c = {n: (sum(v[1:]) / len(v[1:]) if len(v) > 1 else v[0]) for n, v in agg[k].items()}
        if k not in big:
            continue
        lines.append(k)
        for n in sorted(c):
            lines.append(f"    {n:<28}{c[n]:>18.0f}")
        if "SQ_INSTS_VALU" in c:
            per = 64.0 / node_coords
            cyc = c.get("GRBM_GUI_ACTIVE", 0.0) / 8.0
            d = [f"valu/nc={c['SQ_INSTS_VALU'] * per:.2f}"]
            valu_per[k] = c["SQ_INSTS_VALU"] * per
            if "SQ_INSTS_VALU_INT64" in c:
                d.append(f"int64/nc={c['SQ_INSTS_VALU_INT64'] * per:.2f}")
            if "SQ_INSTS_SALU" in c:
                d.append(f"salu/nc={c['SQ_INSTS_SALU'] * per:.2f}")
            if "SQ_INSTS_LDS" in c:
                d.append(f"lds/nc={c['SQ_INSTS_LDS'] * per:.2f}")
            if cyc:
                vc = 4.0 * c["SQ_INSTS_VALU"] / 1024.0
                d.append(f"valu_cycles={vc:.0f}  kernel_cycles={cyc:.0f}  valu_share={vc / cyc:.2f}  valu_ms_2.4GHz={vc / 2.4e6:.3f}")
                if "SQ_LDS_IDX_ACTIVE" in c:
                    d.append(f"lds_share={c['SQ_LDS_IDX_ACTIVE'] / 256.0 / cyc:.2f}")
                    d.append(f"conflict={c.get('SQ_LDS_BANK_CONFLICT', 0.0) / max(c['SQ_LDS_IDX_ACTIVE'], 1.0):.2f}")
            if "TCC_REQ_sum" in c and c["TCC_REQ_sum"]:
                d.append(f"l2_hit_rate={c.get('TCC_HIT_sum', 0.0) / c['TCC_REQ_sum']:.2f}")
            lines.append("    derived: " + "  ".join(d))
        lines.append("")
    os.makedirs(a.out, exist_ok=True)
    with open(os.path.join(a.out, f"{a.name}_sq_counters.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")
    jpath = os.path.join(a.out, "sq_counters.json")
    allc = json.load(open(jpath)) if os.path.exists(jpath) else {}
    allc.setdefault("valu_instructions_per_node_coordinate", {})[a.key or a.name] = {
        k: round(v, 3) for k, v in valu_per.items() if "(" not in k}
    json.dump(allc, open(jpath, "w"), indent=1, sort_keys=True)
    print("\n".join(lines))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--name", required=True)
    ap.add_argument("--key", help="entry of traffic.json to write (default: --name); bench.py looks up "
                                  "<workload>[+alt][+vector|+bucket]")
    ap.add_argument("--stats")
    ap.add_argument("--sq", nargs="+", help="directories of --pmc passes over SQ_* / GRBM_* counters")
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--probe-log", help="stdout of qoda_probe (states the copy kernel's true size); needed with --fetch/--write")
    ap.add_argument("--bench-json", help="the JSON line bench.py printed under the same rocprofv3 run")
    ap.add_argument("--command", required=True)
    ap.add_argument("--out", default="profiles")
    a = ap.parse_args()
    if a.sq:
        return _sq_summary(a)
    if not a.stats:
        raise SystemExit("--stats or --sq is needed")
    lines = [f"# rocprofv3 summary: {a.name}", "# command:", "#   " + a.command, "#"]
    copy_bytes = None
    if a.probe_log:
        log = open(a.probe_log).read()
        copy_bytes = int(re.search(r"k_copy_f4.*bytes_read=(\d+)", log).group(1))
        lines += ["# probe output:"] + ["#   " + l for l in log.strip().splitlines()]
    if a.bench_json:
        b = json.loads(open(a.bench_json).read().strip().splitlines()[-1])
        r = b["roofline"]
        lines += ["# bench.py line of this run (HIP events inside the timed region):",
                  f"#   workload={b['config']['workload']} ms_per_step={b['ms_per_step']:.4f} value={b['value']:.1f} {b['unit']} "
                  f"hbm_peak_fraction_algorithmic={b['hbm_peak_fraction_algorithmic']:.4f}",
                  f"#   roofline: kernel={r['kernel']} avg_ms={r['avg_ms']:.4f} achieved={r['achieved']:.1f} GB/s frac={r['frac']:.4f}"]
    lines += ["", "kernel-trace --stats (ours only):", f"{'kernel':<36}{'calls':>7}{'avg_us':>12}{'min_us':>12}{'max_us':>12}{'pct':>8}"]
    for r in csv.DictReader(open(_one(os.path.join(a.stats, "**", "*_kernel_stats.csv")))):
        if "qoda::" not in r["Name"]:
            continue
        label = _short(r["Name"])
        if label == "k_quantize" and re.search(r"k_quantize(_b)?<\d+, false", r["Name"]):
            label = "k_quantize (no prev)"   # the round-1 variant that reads no previous message
        width = re.search(r"k_(quantize|quantize_b|decode)<(\d+)", r["Name"])
        if width and a.bench_json:             # a run with two workloads: tell their code widths apart
            label += f" [{width.group(2)}-bit codes]"
        lines.append(f"{label:<36}{r['Calls']:>7}{float(r['AverageNs']) / 1e3:>12.1f}"
                     f"{float(r['MinNs']) / 1e3:>12.1f}{float(r['MaxNs']) / 1e3:>12.1f}{float(r['Percentage']):>8.2f}")
    traffic = {}
    if a.fetch and a.write:
        fetch, write = _counters(a.fetch), _counters(a.write)
        f_scale = copy_bytes / (sum(fetch["k_copy_f4"]) / len(fetch["k_copy_f4"]))
        w_scale = copy_bytes / (sum(write["k_copy_f4"]) / len(write["k_copy_f4"]))
        lines += ["", f"--pmc FETCH_SIZE / WRITE_SIZE per dispatch, scaled by the copy kernel ({copy_bytes} B each way):",
                  f"scale factors: FETCH_SIZE x {f_scale:.4f}, WRITE_SIZE x {w_scale:.4f}",
                  f"{'kernel':<22}{'dispatches':>11}{'fetch_MB':>12}{'write_MB':>12}{'total_MB':>12}"]
        for k in sorted(set(fetch) | set(write)):
            if not k.startswith("k_"):
                continue
            # the first dispatch (warm-up round, no previous message) is left out when there are later ones
            fv = fetch.get(k, [0.0])
            wv = write.get(k, [0.0])
            fv = fv[1:] if len(fv) > 1 else fv
            wv = wv[1:] if len(wv) > 1 else wv
            fb, wb = f_scale * sum(fv) / len(fv), w_scale * sum(wv) / len(wv)
            traffic[k] = fb + wb
            lines.append(f"{k:<22}{len(fv):>11}{fb / 1e6:>12.2f}{wb / 1e6:>12.2f}{(fb + wb) / 1e6:>12.2f}")
    os.makedirs(a.out, exist_ok=True)
    with open(os.path.join(a.out, f"{a.name}_kernels.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")
    tpath = os.path.join(a.out, "traffic.json")
    allt = json.load(open(tpath)) if os.path.exists(tpath) else {}
    if traffic:
        allt[a.key or a.name] = traffic
        json.dump(allt, open(tpath, "w"), indent=1, sort_keys=True)
    print("\n".join(lines))


if __name__ == "__main__":
    main()
