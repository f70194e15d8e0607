#!/usr/bin/env python3
"""Writes the rocprofv3 summaries under profiles/ from raw profiler output under gpurun_out/.

The raw output comes from these commands, run on the MI355X machine from the repository root
(`python profile_summary.py --commands` prints them; each counter set is a run of its own):

    stats  rocprofv3 --kernel-trace --stats --output-format csv -d gpurun_out/prof_stats -o bench -- python3 bench.py --no-cfg5
    fetch  rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d gpurun_out/prof_fetch -o bench -- python3 bench.py --no-cpu --no-cfg5 --no-ceiling --no-latency --steps 5 --warmup 1 --copy-calibration
    write  rocprofv3 --pmc WRITE_SIZE --kernel-trace --output-format csv -d gpurun_out/prof_write -o bench -- python3 bench.py --no-cpu --no-cfg5 --no-ceiling --no-latency --steps 5 --warmup 1 --copy-calibration
    mfma   rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_VALU_MFMA_COEXEC_CYCLES SQ_INSTS_VALU SQ_INSTS_MFMA SQ_ACTIVE_INST_VALU SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_WAIT_INST_ANY GRBM_GUI_ACTIVE --kernel-trace --output-format csv -d gpurun_out/prof_mfma -o bench -- python3 bench.py --no-cpu --no-cfg5 --no-ceiling --no-latency --steps 5 --warmup 1
    lds    rocprofv3 --pmc SQ_INSTS_LDS SQ_LDS_BANK_CONFLICT SQ_LDS_ADDR_CONFLICT SQ_ACTIVE_INST_LDS SQ_WAVES SQ_BUSY_CYCLES SQ_INSTS_VMEM_RD --kernel-trace --output-format csv -d gpurun_out/prof_lds -o bench -- python3 bench.py --no-cpu --no-cfg5 --no-ceiling --no-latency --steps 5 --warmup 1
    l2     rocprofv3 --pmc TCC_HIT_sum TCC_MISS_sum TCP_TCC_READ_REQ_sum TCP_TOTAL_CACHE_ACCESSES_sum --kernel-trace --output-format csv -d gpurun_out/prof_l2 -o bench -- python3 bench.py --no-cpu --no-cfg5 --no-ceiling --no-latency --steps 5 --warmup 1

Every run's bench.py line is expected next to its CSV files as gpurun_out/prof_<name>/bench.json
(stdout of the command).  A summary is written for every run whose output is present.  The
byte-counter summary also writes profiles/hbm_traffic.json, which carries a fingerprint of the
kernel sources it was measured on; bench.py reports `traffic_stale` when they have changed since.
"""
from __future__ import annotations

import collections
import csv
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
OUT = os.path.join(ROOT, "profiles")
RAW = os.path.join(ROOT, "gpurun_out")
SUFFIX = "bench_cfg4_reciprocal_cfg3_dense"

COMMANDS = {line.split()[0]: line.split(None, 1)[1] for line in __doc__.splitlines()
            if line.startswith("    ") and " rocprofv3 " in line}


def is_dense_pass1(name):
    """The pass-1 kernel of the dense mode, whichever variant ran."""
    return "dense_staged_kernel<" in name or "dense_kernel<" in name


def short(name: str) -> str:
    name = name.replace("(anonymous namespace)::", "").replace("void fnn::", "").replace("fnn::", "")
    return name.split("(")[0]


def read_csv(run: str, leaf: str):
    path = os.path.join(RAW, f"prof_{run}", leaf)
    if not os.path.exists(path):
        return None
    with open(path) as f:
        return list(csv.DictReader(f))


def bench_line(run: str):
    path = os.path.join(RAW, f"prof_{run}", "bench.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        lines = [ln for ln in f.read().strip().splitlines() if ln.startswith("{")]
    return json.loads(lines[-1]) if lines else None


def write(name: str, lines) -> None:
    os.makedirs(OUT, exist_ok=True)
    path = os.path.join(OUT, name)
    with open(path, "w") as f:
        f.write("\n".join(lines) + "\n")
    print("wrote", os.path.relpath(path, ROOT))


def kernel_stats() -> None:
    stats, bench = read_csv("stats", "bench_kernel_stats.csv"), bench_line("stats")
    if not stats or not bench:
        return
    lines = ["# rocprofv3 kernel statistics: bench.py (cfg 4 batched FastNN reciprocal, cfg 2 single pair, cfg 3 dense mutual NN)", "",
             "Command (on the MI355X box, from the repository root):", "", "    " + COMMANDS["stats"], "",
             "The run holds the warm-up, timed and traced reciprocal steps of 16 pairs, the single-pair calls, the dense calls, the",
             "ceiling loops and the CPU baseline.  Durations in microseconds.", "",
             "| kernel | calls | total | average | % | min | max |", "|---|---|---|---|---|---|---|"]
    for r in stats:
        lines.append(f"| {short(r['Name'])} | {r['Calls']} | {float(r['TotalDurationNs'])/1e3:.1f} | {float(r['AverageNs'])/1e3:.2f} | "
                     f"{float(r['Percentage']):.2f} | {float(r['MinNs'])/1e3:.2f} | {float(r['MaxNs'])/1e3:.2f} |")
    # durations of the batched launches alone, from the kernel trace (grid of 16 pairs), for the agreement check
    trace = read_csv("stats", "bench_kernel_trace.csv") or []
    def avg_us(pred):
        d = [(int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3 for r in trace if pred(r)]
        return (sum(d) / len(d), len(d)) if d else (float("nan"), 0)
    sk_us, sk_n = avg_us(lambda r: ("search_kernel" in r["Kernel_Name"] or "search_first_kernel" in r["Kernel_Name"])
                         and int(r.get("Grid_Size_Y") or 0) == 16)
    dk = [r for r in stats if is_dense_pass1(r["Name"])]
    lines += ["", "## Agreement with bench.py (same run, its own HIP-event timing)", ""]
    if sk_n:
        lines.append(f"* search launches of the 16-pair batch (search_kernel and search_first_kernel together, as in bench.py's `roofline`): "
                     f"kernel-trace average {sk_us:.2f} us over {sk_n} launches; bench.py "
                     f"`roofline.avg_launch_ms` = {bench['roofline']['avg_launch_ms']*1e3:.2f} us over its traced launches (the profiler's "
                     "average also covers the warm-up and untraced timed steps, whose launches are the same mix; the HIP events of bench.py bracket "
                     "each dispatch, so they add a few microseconds per launch, which shows in the 12 launches of a step that find nothing to do: "
                     "the bench line's fraction is the conservative one).")
    if dk and "dense_mutual" in bench:
        lines.append(f"* dense pass-1 kernel: rocprofv3 average {float(dk[0]['AverageNs'])/1e3:.1f} us (minimum {float(dk[0]['MinNs'])/1e3:.1f}; the first calls run on cold clocks); bench.py "
                     f"`dense_mutual.roofline.avg_launch_ms` = {bench['dense_mutual']['roofline']['avg_launch_ms']*1e3:.1f} us.")
    lines += ["", "## bench.py line of this run", "",
              f"Under the profiler every launch takes longer to dispatch, so this line's {bench['ms_per_step']:.2f} ms per step is above an "
              "unprofiled run of the same command; the kernel durations are unaffected.", "", "```json", json.dumps(bench, indent=1), "```"]
    write(f"kernel_stats_{SUFFIX}.md", lines)


def hbm_traffic() -> None:
    per, cal, copies = {}, {}, {}
    for run, counter in (("fetch", "FETCH_SIZE"), ("write", "WRITE_SIZE")):
        rows = read_csv(run, "bench_counter_collection.csv")
        if not rows:
            return
        rows = [r for r in rows if r["Counter_Name"] == counter]
        copy = [float(r["Counter_Value"]) for r in rows if "copyBuffer" in r["Kernel_Name"]]
        if not copy:
            print(f"no calibration copy in the {run} run (bench.py --copy-calibration)", file=sys.stderr)
            return
        copies[run] = max(copy)
        cal[run] = (256 * 1024) / max(copy)            # KiB per counter unit
        table = collections.defaultdict(list)
        for r in rows:
            table[short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
        per[run] = table
    bench = bench_line("fetch")
    times = {}
    for r in read_csv("fetch", "bench_kernel_trace.csv") or []:
        times.setdefault(short(r["Kernel_Name"]), []).append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    lines = ["# HBM traffic per kernel (rocprofv3 byte counters): bench.py workloads", "", "Commands (two runs, one counter each):", "",
             "    " + COMMANDS["fetch"], "    " + COMMANDS["write"], "",
             "`--copy-calibration` adds one plain 256 MiB device-to-device copy (`__amd_rocclr_copyBuffer`, 262144 KiB read and 262144 KiB written).",
             f"It reads FETCH_SIZE = {copies['fetch']:.1f} and WRITE_SIZE = {copies['write']:.1f}, so one FETCH_SIZE unit = {cal['fetch']:.4f} KiB and one "
             f"WRITE_SIZE unit = {cal['write']:.4f} KiB on this part.", "",
             "Scaled values, MiB per launch (average over all launches of the run):", "",
             "| kernel | launches | read MiB/launch | written MiB/launch |", "|---|---|---|---|"]
    names = sorted(set(per["fetch"]) | set(per["write"]), key=lambda k: -sum(per["fetch"].get(k, [0])))
    for k in names:
        f, w = per["fetch"].get(k, [0]), per["write"].get(k, [0])
        lines.append(f"| {k} | {len(f)} | {sum(f)/len(f)*cal['fetch']/1024:.3f} | {sum(w)/len(w)*cal['write']/1024:.3f} |")

    def kernel_bytes(prefix):
        f = [v for k, v in per["fetch"].items() if k.startswith(prefix)]
        w = [v for k, v in per["write"].items() if k.startswith(prefix)]
        if not f or not w:
            return None, None, None
        rd = sum(f[0]) / len(f[0]) * cal["fetch"] * 1024
        wr = sum(w[0]) / len(w[0]) * cal["write"] * 1024
        return rd, wr, f[0]
    s_rd, s_wr, s_list = kernel_bytes("search_kernel")
    d_rd, d_wr, _ = kernel_bytes("dense_staged_kernel")
    if d_rd is None:
        d_rd, d_wr, _ = kernel_bytes("dense_kernel")
    result = {"source": f"profiles/hbm_traffic_{SUFFIX}.md (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by a 256 MiB copy)"}
    if s_rd is not None and bench:
        # bench.py runs its batched reciprocal steps first: one call that builds the outputs, the
        # warm-up, the timed steps and the traced steps, 2 * max_iter search launches each.  The first
        # two of a step are launches of search_first_kernel (the staged kernel that also reads the
        # caller's fp32 maps and writes the prepared copies), the rest of search_kernel.
        per_step = int(round(bench["roofline"]["launches_per_step"]))
        n_steps = 1 + bench["warmup"] + 2 * bench["steps"]
        def mib(run, prefix, count):
            rows = [v for k, v in per[run].items() if k.startswith(prefix)]
            return [x * cal[run] / 1024 for x in rows[0][:count]] if rows else []
        first_rd, first_wr = mib("fetch", "search_first_kernel", 2 * n_steps), mib("write", "search_first_kernel", 2 * n_steps)
        n_first = len(first_rd)
        n_rest = n_steps * per_step - n_first
        rest_rd, rest_wr = mib("fetch", "search_kernel", n_rest), mib("write", "search_kernel", n_rest)
        total = sum(first_rd) + sum(first_wr) + sum(rest_rd) + sum(rest_wr)
        result["search_kernel_bytes_per_launch"] = round(total / (n_steps * per_step) * 1048576)
        live = [x for x in rest_rd if x > 1.0]
        alg = bench["roofline_hbm"]["bytes_per_launch"]
        lines += ["", "## the search launches of the 16-pair reciprocal steps", "",
                  f"search_first_kernel (first forward and first backward search of a step; fp32 maps in, prepared fp16 copy out), last two launches: "
                  + ", ".join(f"{r:.1f} MiB read / {w:.1f} MiB written" for r, w in zip(first_rd[-2:], first_wr[-2:]))
                  + ".  The fp32 maps of 16 pairs are 288 MiB, their fp16 copy 144 MiB.", "",
                  f"search_kernel, read MiB per launch, the {per_step - 2} launches of the last step, in launch order: "
                  + ", ".join(f"{x:.1f}" for x in rest_rd[-(per_step - 2):]), "",
                  f"Average HBM bytes per search launch over these {n_steps * per_step} launches (read + written): "
                  f"{result['search_kernel_bytes_per_launch']/1e6:.1f} MB; algorithmic bytes per launch (bench.py `roofline_hbm.bytes_per_launch`): "
                  f"{alg/1e6:.1f} MB.  A live search of 16 prepared maps must read 16 x 196608 x 48 B = 151 MB = 144 MiB once; the live launches of "
                  f"search_kernel read {sum(live)/max(len(live),1):.1f} MiB on average (the last-level cache keeps part of a map between the searches "
                  "of a step), the launches after the last seed has converged read nothing.", ""]
    if d_rd is not None:
        d_names = [k for k in times if k.startswith("dense_staged_kernel")] or [k for k in times if k.startswith("dense_kernel")]
        d_us = times.get(d_names[0]) if d_names else None
        rate = ""
        if d_us:
            t = sum(d_us) / len(d_us)
            rate = f"  At {t/1e3:.2f} ms per launch (duration under the counter run) that is {(d_rd + d_wr)/t/1e6:.2f} TB/s and does not bound the kernel."
        result["dense_kernel_bytes_per_launch"] = round(d_rd + d_wr)
        lines += ["## dense_kernel (cfg 3)", "",
                  f"Reads {d_rd/1048576:.0f} MiB and writes {d_wr/1048576:.0f} MiB per launch against 19 MB of algorithmic input and 3 MB of keys: the reads are "
                  "query blocks re-fetched by the workgroups through L2 misses, the writes are the 64-bit atomic key merges (each counted as a partial "
                  "cache-line write)." + rate, ""]
    sys.path.insert(0, ROOT)
    from bench import csrc_fingerprint
    result["csrc_fingerprint"] = csrc_fingerprint()
    write(f"hbm_traffic_{SUFFIX}.md", lines)
    with open(os.path.join(OUT, "hbm_traffic.json"), "w") as f:
        json.dump(result, f, indent=1)
    print("wrote profiles/hbm_traffic.json", result)


def mfma_utilisation() -> None:
    rows = read_csv("mfma", "bench_counter_collection.csv")
    trace_rows = read_csv("mfma", "bench_kernel_trace.csv")
    if not rows or not trace_rows:
        return
    disp = collections.defaultdict(dict)
    for r in rows:
        disp[(r["Dispatch_Id"], r["Kernel_Name"])][r["Counter_Name"]] = float(r["Counter_Value"])
    trace = {r["Dispatch_Id"]: (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) for r in trace_rows}
    searches = sorted([(k, v) for k, v in disp.items() if "search_first_kernel" in k[1]], key=lambda kv: -kv[1].get("SQ_INSTS_MFMA", 0))
    first_name = "search_first_kernel"
    if not searches:
        searches = sorted([(k, v) for k, v in disp.items() if "search_kernel" in k[1]], key=lambda kv: -kv[1].get("SQ_INSTS_MFMA", 0))
        first_name = "search_kernel"
    denses = [(k, v) for k, v in disp.items() if is_dense_pass1(k[1])]
    if not searches or not denses:
        return
    sk, dk = searches[min(2, len(searches) - 1)], denses[-1]

    def col(kv, products):
        k, v = kv
        us = trace[k[0]] / 1e3
        cyc = v["GRBM_GUI_ACTIVE"] / 8
        other = v["SQ_INSTS_VALU"] - v["SQ_INSTS_MFMA"]
        return [f"{us:.0f} us under the counter run", f"{cyc/1e6:.2f} M  ({cyc/us/1e3:.2f} GHz)",
                f"{v['SQ_INSTS_MFMA']/1e6:.1f} M ({v['SQ_INSTS_MFMA']/products:.2f} per product)",
                f"{other/1e6:.1f} M ({other/products:.1f} per product)",
                f"{100*v['SQ_VALU_MFMA_BUSY_CYCLES']/(1024*cyc):.1f} % of cycles", f"{100*other*4/(1024*cyc):.1f} % of cycles",
                f"{100*v['SQ_VALU_MFMA_COEXEC_CYCLES']/v['SQ_VALU_MFMA_BUSY_CYCLES']:.0f} %",
                f"{100*v['SQ_WAIT_INST_ANY']/v['SQ_WAVE_CYCLES']:.0f} %"]
    a, b = col(sk, 16 * 96 * 6144), col(dk, 6144 * 6144)
    names = ["duration (kernel trace)", "GPU cycles (per XCD)", "matrix instructions", "other vector instructions", "matrix cores busy",
             "vector instruction issue (4 cycles each)", "matrix busy cycles with a vector instruction co-executing",
             "wave cycles waiting on an instruction (SQ_WAIT_INST_ANY / SQ_WAVE_CYCLES)"]
    lines = ["# Matrix-core and vector-ALU utilisation (rocprofv3 SQ counters): search_kernel and dense_kernel", "", "Command (one counter run):", "",
             "    " + COMMANDS["mfma"], "",
             "Per dispatch.  GRBM_GUI_ACTIVE is summed over the 8 XCDs, SQ_VALU_MFMA_BUSY_CYCLES over the 1024 SIMDs; SQ_INSTS_* count wave instructions",
             "(SQ_INSTS_VALU includes the matrix instructions).  A 32x32 product = one K=16 plus one K=8 matrix instruction.", "",
             f"| quantity | {first_name}, first search of a step (16 x 3072 queries) | dense_kernel (cfg 3) |", "|---|---|---|"]
    lines += [f"| {n} | {x} | {y} |" for n, x, y in zip(names, a, b)]
    lines += ["", "Of the vector instructions per product, 8 (search) and 16 (dense) are the three-input maxima that fold the scores; the rest is location",
              "tracking, address arithmetic, register copies and (dense) the per-super-block column flush."]
    write(f"mfma_utilisation_{SUFFIX}.md", lines)


def lds_l2() -> None:
    def table(run):
        rows = read_csv(run, "bench_counter_collection.csv")
        if not rows:
            return None
        per = collections.defaultdict(lambda: collections.defaultdict(list))
        for r in rows:
            per[short(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
        return per
    lds, l2 = table("lds"), table("l2")
    if not lds or not l2:
        return

    def pick(per, prefix, counter, how):
        for k, v in per.items():
            if k.startswith(prefix) and counter in v:
                return max(v[counter]) if how == "max" else sum(v[counter]) / len(v[counter])
        return float("nan")
    kernels = [("search_first_kernel", "max", "search_first_kernel, first search of a step (fp32 maps in, LDS-staged)"),
               ("search_kernel", "max", "search_kernel, largest launch (third search of a step: 16 x ~1450 queries)"),
               ("resolve_kernel", "max", "resolve_kernel, first resolve of a step"),
               ("dense_staged_kernel<", "mean", "dense_staged_kernel (cfg 3; query blocks staged through LDS)"), ("prep_f32_kernel", "max", "prepare pass, largest launch (the dense legs: both maps of a pair)")]
    lines = ["# LDS and cache counters (rocprofv3 SQ / TCP / TCC counters): bench.py workloads", "", "Commands (two counter runs):", "",
             "    " + COMMANDS["lds"], "    " + COMMANDS["l2"], "",
             "Per dispatch; SQ_BUSY_CYCLES is summed over the shader engines, the cache counters over all channels.", "",
             "| kernel | waves | vector memory reads | LDS instructions | LDS bank-conflict cycles | share of SQ busy cycles | L1 accesses | L1 -> L2 read requests | L1 hit share | L2 hits | L2 misses | L2 hit share |",
             "|---|---|---|---|---|---|---|---|---|---|---|---|"]
    for prefix, how, label in kernels:
        waves, vmem, insts, conf, busy = (pick(lds, prefix, c, how) for c in ("SQ_WAVES", "SQ_INSTS_VMEM_RD", "SQ_INSTS_LDS", "SQ_LDS_BANK_CONFLICT", "SQ_BUSY_CYCLES"))
        acc, req, hit, miss = (pick(l2, prefix, c, how) for c in ("TCP_TOTAL_CACHE_ACCESSES_sum", "TCP_TCC_READ_REQ_sum", "TCC_HIT_sum", "TCC_MISS_sum"))
        lines.append(f"| {label} | {waves:.0f} | {vmem/1e3:.1f} k | {insts/1e3:.1f} k | {conf/1e3:.1f} k | {100*conf/busy:.2f} % | {acc/1e6:.1f} M | {req/1e6:.2f} M | "
                     f"{100*(1-req/acc):.0f} % | {hit/1e6:.2f} M | {miss/1e6:.2f} M | {100*hit/(hit+miss):.0f} % |")
    write(f"lds_l2_counters_{SUFFIX}.md", lines)


def main() -> int:
    if "--commands" in sys.argv:
        for name, cmd in COMMANDS.items():
            print(f"mkdir -p gpurun_out/prof_{name} && {cmd} > gpurun_out/prof_{name}/bench.json")
        return 0
    kernel_stats()
    hbm_traffic()
    mfma_utilisation()
    lds_l2()
    return 0


if __name__ == "__main__":
    sys.exit(main())
