"""Turns rocprofv3 output of a bench.py run into the summaries kept under profiles/.

bench.py runs its legs one after the other (token loops of both modes, instrumented loops, kernels
launched back to back, ...) and, with --legs-file, writes their order and how many launches of each
kernel a leg makes.  rocprofv3 lists every dispatch in order; this script cuts the list of each kernel at
those counts, so that durations (kernel trace) and HBM byte counters (PMC runs) can be reported per leg
instead of as one average over the whole command.

  kernel trace:  rocprofv3 --kernel-trace --stats --output-format csv -d DIR -o bench -- python3 bench.py --legs-file LEGS
  HBM traffic :  rocprofv3 --pmc FETCH_SIZE --output-format csv -d DIR_F -o bench -- python3 bench.py ... --calibrate-copy --legs-file LEGS_P
                 rocprofv3 --pmc WRITE_SIZE --output-format csv -d DIR_W -o bench -- python3 bench.py ... --calibrate-copy --legs-file LEGS_P

  python -m paper_2603_19289_amd.profile_summary --trace DIR --legs LEGS --bench-json LINE.json \\
         --pmc-fetch DIR_F --pmc-write DIR_W --pmc-legs LEGS_P --pmc-bench-json LINE_P.json --out profiles --tag bench_default

Writes profiles/<tag>_kernel_trace_by_leg.md, profiles/<tag>_pmc_hbm_traffic.md and merges the figures
into profiles/kernel_trace_by_leg.json and profiles/hbm_traffic.json, which bench.py reads.
The byte counters are scaled by what they read for the plain 256 MiB device copy that --calibrate-copy
appends to the run (FETCH_SIZE and WRITE_SIZE count in units that differ between machines).
"""
import argparse
import collections
import csv
import glob
import json
import os
import statistics

CAL_BYTES = 256 << 20


def read_csv(directory, suffix):
    paths = sorted(glob.glob(os.path.join(directory, "**", "*" + suffix), recursive=True))
    if not paths:
        raise SystemExit(f"no *{suffix} under {directory}")
    rows = []
    for p in paths:
        with open(p, newline="") as f:
            rows += list(csv.DictReader(f))
    return rows


def cut_by_legs(sequence, legs, symbol):
    """sequence: the symbol's dispatches in order.  Returns {leg name: slice}.  Legs name a count for the symbol,
    or list it under "uncounted" (at most one run of consecutive such legs can be resolved: it gets the rest)."""
    known = sum(l["counts"].get(symbol, 0) for l in legs)
    open_total = len(sequence) - known
    out, pos, open_used = {}, 0, False
    i = 0
    while i < len(legs):
        leg = legs[i]
        if symbol in leg["counts"]:
            n = leg["counts"][symbol]
            out[leg["leg"]] = sequence[pos:pos + n]
            pos += n
            i += 1
        elif symbol in leg.get("uncounted", []):
            j = i
            names = []
            while j < len(legs) and symbol in legs[j].get("uncounted", []) and symbol not in legs[j]["counts"]:
                names.append(legs[j]["leg"])
                j += 1
            if open_used or open_total < 0:
                raise SystemExit(f"cannot attribute the dispatches of {symbol}: more than one run of uncounted legs")
            out[" + ".join(names)] = sequence[pos:pos + open_total]
            pos += open_total
            open_used = True
            i = j
        else:
            i += 1
    if pos != len(sequence) and not open_used:
        out["(not attributed)"] = sequence[pos:]
    return out


def category(leg_name):
    parts = leg_name.split("/")
    if " + " in leg_name:
        return parts[0], "token_loops_all_modes"
    if len(parts) >= 3 and parts[1] == "isolated":
        return parts[0], "isolated/" + parts[2]
    if len(parts) >= 3 and parts[2].startswith("rep"):
        return parts[0], parts[1] + "_token_loop"
    return parts[0], "/".join(parts[1:]) or "all"


def stats_us(durs):
    return {"launches": len(durs), "mean_us": statistics.mean(durs), "median_us": statistics.median(durs),
            "min_us": min(durs), "max_us": max(durs)}


def merge_json(path, key, value, meta):
    data = {}
    if os.path.exists(path):
        with open(path) as f:
            data = json.load(f)
    data.setdefault("workloads", {})
    for wl, v in value.items():
        data["workloads"][wl] = v
    data[key] = meta
    with open(path, "w") as f:
        json.dump(data, f, indent=1, sort_keys=True)
        f.write("\n")


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--trace")
    ap.add_argument("--legs")
    ap.add_argument("--bench-json")
    ap.add_argument("--trace-command", default="")
    ap.add_argument("--pmc-fetch")
    ap.add_argument("--pmc-write")
    ap.add_argument("--pmc-legs")
    ap.add_argument("--pmc-bench-json")
    ap.add_argument("--pmc-command", default="")
    ap.add_argument("--out", default="profiles")
    ap.add_argument("--tag", required=True)
    a = ap.parse_args()
    symbols = ["route_pair_kernel", "gateup_b1", "down_combine_b1", "stream_read", "expert_mfma_kernel<true",
               "expert_mfma_kernel<false", "advance_kernel"]

    if a.trace:
        legs = json.load(open(a.legs))
        bench = json.load(open(a.bench_json)) if a.bench_json else {}
        rows = read_csv(a.trace, "kernel_trace.csv")
        rows.sort(key=lambda r: int(r["Start_Timestamp"]))
        per_wl = collections.defaultdict(lambda: collections.defaultdict(dict))
        md = [f"# rocprofv3 kernel trace of bench.py, durations per leg ({a.tag})\n",
              "Command (run from /tmp with TMPDIR=/tmp on the MI355X box, repository at $R):\n",
              "    " + (a.trace_command or "rocprofv3 --kernel-trace --stats --output-format csv -d DIR -o bench -- python3 $R/bench.py --legs-file LEGS") + "\n",
              "Every dispatch of the trace is attributed to the leg of bench.py that launched it (the legs run one after the",
              "other; their launch counts come from --legs-file).  Durations are the trace's End - Start per dispatch.\n"]
        if bench:
            md.append(f"bench.py's own line in this profiled run: speculative TPOT {bench['ms_per_step']:.2f} ms ({bench['value']:.2f} tokens/s), "
                      f"on-demand TPOT {bench['on_demand']['tpot_ms']:.2f} ms.\n")
        md += ["| workload | leg | kernel | launches | mean (us) | median (us) | min (us) | max (us) |", "|---|---|---|---|---|---|---|---|"]
        for sym in symbols:
            seq = [(int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3 for r in rows if sym in r["Kernel_Name"]]
            if not seq:
                continue
            for leg_name, durs in cut_by_legs(seq, legs["legs"], sym).items():
                if not durs:
                    continue
                wl, cat = category(leg_name)
                cur = per_wl[wl][cat].get(sym)
                if cur:                                   # several repetitions of one mode: pool them
                    durs = cur["_durs"] + durs
                per_wl[wl][cat][sym] = dict(stats_us(durs), _durs=durs)
        for wl in per_wl:
            for cat in sorted(per_wl[wl]):
                for sym, s in per_wl[wl][cat].items():
                    s.pop("_durs")
                    md.append(f"| {wl} | {cat} | {sym} | {s['launches']} | {s['mean_us']:.2f} | {s['median_us']:.2f} | {s['min_us']:.2f} | {s['max_us']:.2f} |")
        os.makedirs(a.out, exist_ok=True)
        with open(os.path.join(a.out, f"{a.tag}_kernel_trace_by_leg.md"), "w") as f:
            f.write("\n".join(md) + "\n")
        merge_json(os.path.join(a.out, "kernel_trace_by_leg.json"), "source",
                   {wl: {cat: dict(v) for cat, v in cats.items()} for wl, cats in per_wl.items()},
                   {"command": a.trace_command, "summary": f"{a.tag}_kernel_trace_by_leg.md", "unit": "microseconds per dispatch"})

    if a.pmc_fetch and a.pmc_write:
        legs = json.load(open(a.pmc_legs))
        bench = json.load(open(a.pmc_bench_json)) if a.pmc_bench_json else {}
        per = {}
        scale = {}
        for ctr, d in (("FETCH_SIZE", a.pmc_fetch), ("WRITE_SIZE", a.pmc_write)):
            rows = [r for r in read_csv(d, "counter_collection.csv") if r["Counter_Name"] == ctr]
            by_dispatch = collections.OrderedDict()
            for r in sorted(rows, key=lambda r: int(r["Dispatch_Id"])):
                k = int(r["Dispatch_Id"])
                name, val = by_dispatch.get(k, (r["Kernel_Name"], 0.0))
                by_dispatch[k] = (name, val + float(r["Counter_Value"]))
            disp = list(by_dispatch.values())
            cal = [v for n, v in disp if "copyBuffer" in n]
            if not cal:
                raise SystemExit("no calibration copy in the PMC run (bench.py --calibrate-copy)")
            scale[ctr] = CAL_BYTES / cal[-1]              # bytes per count
            for sym in symbols:
                seq = [v for n, v in disp if sym in n]
                if not seq:
                    continue
                for leg_name, vals in cut_by_legs(seq, legs["legs"], sym).items():
                    if vals:
                        per.setdefault((leg_name, sym), {})[ctr] = (len(vals), statistics.median(vals))
        md = [f"# rocprofv3 PMC summary: HBM bytes per launch of bench.py's kernels ({a.tag})\n",
              "Commands (one counter per run, run from /tmp with TMPDIR=/tmp, repository at $R):\n",
              "    " + (a.pmc_command or "rocprofv3 --pmc FETCH_SIZE|WRITE_SIZE --output-format csv -d DIR -o bench -- python3 $R/bench.py ... --calibrate-copy --legs-file LEGS") + "\n",
              f"Scaling: the last dispatch of each run is a plain device-to-device copy of {CAL_BYTES:,} bytes (read once, written once);",
              f"one FETCH_SIZE count is {scale['FETCH_SIZE']:.2f} bytes and one WRITE_SIZE count {scale['WRITE_SIZE']:.2f} bytes on this box.\n",
              "| workload | leg | kernel | launches | FETCH_SIZE median | WRITE_SIZE median | bytes read | bytes written | algorithmic bytes | traffic / algorithmic |",
              "|---|---|---|---|---|---|---|---|---|---|"]
        traffic = collections.defaultdict(dict)
        alg = {}
        for wl_name, res in [(bench.get("config", {}).get("workload", ""), bench)] + list((bench.get("other_workloads") or {}).items()):
            for kname, k in ((res.get("roofline") or {}).get("kernels") or {}).items():
                alg[(wl_name.split(" ")[0], kname)] = k["bytes_per_launch"]
        for (leg_name, sym), c in sorted(per.items()):
            if "FETCH_SIZE" not in c or "WRITE_SIZE" not in c:
                continue
            wl, cat = category(leg_name)
            rb, wb = c["FETCH_SIZE"][1] * scale["FETCH_SIZE"], c["WRITE_SIZE"][1] * scale["WRITE_SIZE"]
            kname = cat.split("/", 1)[1] if cat.startswith("isolated/") else None
            ab = alg.get((wl, kname))
            md.append(f"| {wl} | {cat} | {sym} | {c['FETCH_SIZE'][0]} | {c['FETCH_SIZE'][1]:.1f} | {c['WRITE_SIZE'][1]:.1f} | {rb:,.0f} | {wb:,.0f} | "
                      f"{(format(ab, ',') if ab else '-')} | {((rb + wb) / ab if ab else float('nan')):.3f} |")
            if kname:
                traffic[wl][kname] = {"bytes": round(rb + wb), "fetch_bytes": round(rb), "write_bytes": round(wb),
                                      "algorithmic_bytes": ab, "launches": c["FETCH_SIZE"][0]}
        os.makedirs(a.out, exist_ok=True)
        with open(os.path.join(a.out, f"{a.tag}_pmc_hbm_traffic.md"), "w") as f:
            f.write("\n".join(md) + "\n")
        merge_json(os.path.join(a.out, "hbm_traffic.json"), "source", dict(traffic),
                   {"command": a.pmc_command, "summary": f"{a.tag}_pmc_hbm_traffic.md",
                    "bytes_per_count": scale, "calibration_bytes": CAL_BYTES})


if __name__ == "__main__":
    main()
