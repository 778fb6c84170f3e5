"""Short text summaries of rocprofv3 runs of bench.py, written under profiles/.

The raw profiler output stays outside the repository.  On the GPU machine, with <out> a scratch folder
and <tag> a workload of bench.py (r50, r152, bertl, ...), run (one profiler pass per command;
`cd /tmp && export TMPDIR=/tmp` first):

    rocprofv3 --kernel-trace --stats -d <out> -o kt --output-format csv -- python3 bench.py --config <tag> --steps 20 --warmup 3 --cpu-budget 0 --no-breakdown > <out>/kt.log
    rocprofv3 --pmc FETCH_SIZE -d <out> -o pmc_FETCH_SIZE --output-format csv -- python3 bench.py --config <tag> --steps 3 --warmup 1 --cpu-budget 0 --no-breakdown --copy-calibration
    rocprofv3 --pmc WRITE_SIZE -d <out> -o pmc_WRITE_SIZE --output-format csv -- python3 bench.py --config <tag> --steps 3 --warmup 1 --cpu-budget 0 --no-breakdown --copy-calibration
    grep -h '^{' <out>/kt.log | tail -1 > <out>/bench_line.json

then, from the repository root:  python -m paper_2107_06533_amd.profile_summary <tag> <out>

which writes profiles/<tag>_kernel_trace.md, profiles/<tag>_hbm_traffic.md and the entry of <tag> in
profiles/traffic.json (the HBM bytes per launch of the dominant kernel that bench.py quotes as
`roofline.traffic`).  The byte counters are scaled by what the same counters read for the 1 GiB
device-to-device copies that `--copy-calibration` adds to the run.
"""
import collections
import csv
import json
import os
import sys


def main(tag: str, out_dir: str) -> None:
    O = out_dir.rstrip("/") + "/"
    short = lambda n: n.split("(")[0].replace("kfac::", "").replace("void ", "")[:48]
    CMD_KT = f"cd /tmp && export TMPDIR=/tmp && rocprofv3 --kernel-trace --stats -d <out> -o kt --output-format csv -- python3 bench.py --config {tag} --steps 20 --warmup 3 --cpu-budget 0 --no-breakdown"
    CMD_PMC = f"cd /tmp && export TMPDIR=/tmp && rocprofv3 --pmc {{c}} -d <out> -o pmc_{{c}} --output-format csv -- python3 bench.py --config {tag} --steps 3 --warmup 1 --cpu-budget 0 --no-breakdown --copy-calibration"
    rows = list(csv.DictReader(open(O + "kt_kernel_stats.csv")))
    bench = json.loads(open(O + "bench_line.json").read())
    steps = bench["steps"] + bench["warmup"]
    out = []
    out.append(f"# rocprofv3 kernel-trace summary: K-FAC step on the {tag} workload (one MI355X)\n")
    out.append("Command (committed files only):\n\n    " + CMD_KT + "\n")
    out.append(f"bench.py line of the profiled run: step {bench['value']} ms (profiler attached), roofline kernel avg launch {bench['roofline']['avg_launch_ms']} ms by HIP events.\n")
    out.append(f"{steps} steps were executed (20 timed + 3 warm-up). Durations from `kt_kernel_stats.csv`:\n")
    out.append("| kernel | calls | calls/step | avg us | total ms | ms/step | % |")
    out.append("|---|---|---|---|---|---|---|")
    for r in rows:
        if "kfac" not in r["Name"]: continue
        calls = int(r["Calls"]); tot = float(r["TotalDurationNs"]) / 1e6
        out.append(f"| {short(r['Name'])} | {calls} | {calls/steps:.1f} | {float(r['AverageNs'])/1e3:.1f} | {tot:.2f} | {tot/steps:.3f} | {float(r['Percentage']):.1f} |")
    out.append("")
    out.append("Notes: inside kfac_invert_batch the sweep chain runs on the caller's stream and the off-chain updates on a side stream, so kernels of the two streams overlap and their per-step sums exceed the wall time of the call; tile_gemm_yield_kernel serves the inverse's panel and update products, tile_gemm_kernel and tile_gemm_dl_kernel the two preconditioning products; lag_pairs_kernel and lag_mirror_kernel build the 3x3 activation factors from the lag products that tile_any_kernel wrote.\n")
    open(f"profiles/{tag}_kernel_trace.md", "w").write("\n".join(out))

    # traffic
    res = {}
    lines = [f"# rocprofv3 HBM-traffic counters: K-FAC step on the {tag} workload (one MI355X)\n",
             "Two runs, one counter each (FETCH_SIZE, then WRITE_SIZE; KiB per dispatch):\n",
             "    " + CMD_PMC.format(c="FETCH_SIZE"), "    " + CMD_PMC.format(c="WRITE_SIZE"), "",
             "`--copy-calibration` adds three 1 GiB device-to-device copies (`__amd_rocclr_copyBuffer`, 1 048 576 KiB read and written each); the counter value of those dispatches gives the scale factor applied to every other kernel.\n"]
    scale = {}
    per = {}
    for c in ["FETCH_SIZE", "WRITE_SIZE"]:
        acc = collections.defaultdict(list)
        for r in csv.DictReader(open(O + f"pmc_{c}_counter_collection.csv")):
            acc[short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
        big = [v for v in acc["__amd_rocclr_copyBuffer"] if v > 1e5]
        scale[c] = 1048576.0 / (sum(big) / len(big))
        per[c] = {k: sum(v) / len(v) for k, v in acc.items()}
        lines.append(f"{c}: copy dispatches read {sum(big)/len(big):.0f} KiB for 1 048 576 KiB moved -> scale factor {scale[c]:.3f}")
    lines.append("")
    lines.append("| kernel | FETCH KiB/dispatch (raw) | fetched MB (scaled) | WRITE KiB/dispatch (raw) | written MB (scaled) |")
    lines.append("|---|---|---|---|---|")
    for k in per["FETCH_SIZE"]:
        if not ("tile" in k or "gj_" in k or "lag_" in k): continue
        f = per["FETCH_SIZE"][k]; w = per["WRITE_SIZE"].get(k, 0)
        lines.append(f"| {k} | {f:.0f} | {f*scale['FETCH_SIZE']*1024/1e6:.1f} | {w:.0f} | {w*scale['WRITE_SIZE']*1024/1e6:.1f} |")
        res[k] = {"fetch_bytes": f * scale["FETCH_SIZE"] * 1024, "write_bytes": w * scale["WRITE_SIZE"] * 1024}
    fa = res["tile_any_kernel"]
    alg = json.load(open(O + "bench_line.json"))
    lines.append("")
    lines.append(f"Dominant kernel tile_any_kernel (one launch per step): {fa['fetch_bytes']/1e9:.2f} GB fetched + {fa['write_bytes']/1e9:.2f} GB written per launch.")
    open(f"profiles/{tag}_hbm_traffic.md", "w").write("\n".join(lines) + "\n")
    tpath = "profiles/traffic.json"
    t = json.load(open(tpath)) if os.path.exists(tpath) else {}
    t[tag] = {"factor_tiles_bytes_per_launch": round(fa["fetch_bytes"] + fa["write_bytes"]),
              "factor_tiles_fetch_bytes": round(fa["fetch_bytes"]), "factor_tiles_write_bytes": round(fa["write_bytes"]),
              "fetch_scale": round(scale["FETCH_SIZE"], 4), "write_scale": round(scale["WRITE_SIZE"], 4),
              "source": f"profiles/{tag}_hbm_traffic.md"}
    json.dump(t, open(tpath, "w"), indent=1)


if __name__ == "__main__":
    if len(sys.argv) != 3:
        print(__doc__)
        sys.exit(2)
    main(sys.argv[1], sys.argv[2])
