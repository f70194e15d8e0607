#!/usr/bin/env python3
"""Benchmark of the FastNN hot path on one MI355X.

One step = one batched fnn_reciprocal call (seed grid, prepare/cast, up to 2*max_iter fused
searches, reciprocity test, compaction, dedup) over 16 synthetic 512x384, D=24 image pairs
already resident in HBM.  The headline value is image pairs per second.  The same run also
times the dense all-pairs mutual-NN mode on one 512x384 pair (fp16 compute) and, as a baseline
only, the CPU oracle on a sample of the same pairs.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

WIDTH, HEIGHT, D = 512, 384, 24
N_PIX = WIDTH * HEIGHT
BATCH = 16
SUBSAMPLE = 8
MAX_ITER = 10
PEAK_MFMA_16BIT = 2500.0   # TFLOP/s, dense fp16 / bf16
PEAK_FP32 = 157.3          # TFLOP/s
PEAK_HBM = 8000.0          # GB/s


def searches_from_iters(seed_iter, n_seeds, max_iter):
    """Number of active queries in every search of one pair, from the per-seed iterations.

    Search 0 has all seeds; at iteration t the back search and (if it is not the last
    iteration) the following forward search run on the seeds not converged before / at t.
    """
    import numpy as np
    it = np.asarray(seed_iter)
    it = np.where(it < 0, max_iter, it)
    counts = [n_seeds]
    for t in range(max_iter):
        alive = int((it >= t).sum())
        counts.append(alive)                       # U^{t+1} = NN_1(V^t)
        if t < max_iter - 1:
            counts.append(int((it > t).sum()))     # V^{t+1} = NN_2(U^{t+1})
    return counts


def csrc_fingerprint() -> str:
    """Hash of the kernel sources: ties a stored counter measurement to the code it was taken on."""
    import hashlib
    d = os.path.join(ROOT, "paper_2503_10017_amd", "csrc")
    h = hashlib.sha1()
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".hpp")):
            h.update(name.encode())
            with open(os.path.join(d, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()[:16]


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--compute", default="f16", choices=["f16", "bf16", "f32"])
    ap.add_argument("--no-dense", action="store_true", help="skip the dense mutual-NN leg")
    ap.add_argument("--no-cfg5", action="store_true", help="skip the 1024x768 bf16 leg (configs[4]: dense mutual NN + reciprocal)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-latency", action="store_true", help="skip the single-pair latency leg (configs[1])")
    ap.add_argument("--contrast", action="store_true",
                    help="also time the paper's blocked schedules (Algorithms 1 and 2 with a materialised score block)")
    ap.add_argument("--normalize", action="store_true",
                    help="also time the same batch with the L2 normalisation of raw head outputs fused into the prepare pass")
    ap.add_argument("--l2", action="store_true",
                    help="also time the same batch with the squared-distance dist_func (FNN_FLAG_L2)")
    ap.add_argument("--split", action="store_true",
                    help="also time the batch with FNN_FLAG_SPLIT (fp32-grade scores from three fp16 products) and with fp32 products")
    ap.add_argument("--nearest", action="store_true",
                    help="also time fnn_nearest on the same batch: the 3072 seeds of every pair as queries, and every pixel as a query")
    ap.add_argument("--batch-sweep", action="store_true",
                    help="also time the same workload at 1, 2, 4, 8, 32 and 64 pairs per call")
    ap.add_argument("--no-ceiling", action="store_true",
                    help="skip the measurement of what the device sustains on the kernels' bare instruction mix (about a second)")
    ap.add_argument("--f16-maps", action="store_true",
                    help="also time the batch with the maps already stored in the compute format (read in place, no prepare pass)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 256 MiB device copy (reference dispatch for scaling HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build targets ONE MI355X; --gpus must be 1 "
              "(image pairs are independent, so more GPUs would simply take pairs b mod G)", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2503_10017_amd as fnn
    import synth_inputs as synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    fnn.load_library()
    dev = torch.device("cuda:0")
    compute = args.compute

    # ---- inputs: 16 synthetic pairs, resident in HBM before any timing ----------------------
    t_gen = time.time()
    maps = [synth.config_pair(4, p) for p in range(BATCH)]
    seeds_np = np.tile(synth.grid_seeds(WIDTH, HEIGHT, SUBSAMPLE), (BATCH, 1))
    n_seeds = seeds_np.shape[1]
    d1 = torch.from_numpy(np.stack([m[0] for m in maps])).to(dev)
    d2 = torch.from_numpy(np.stack([m[1] for m in maps])).to(dev)
    seeds = torch.from_numpy(seeds_np).to(dev)
    ws = torch.empty(fnn.fnn_workspace_bytes(BATCH, N_PIX, N_PIX, D, n_seeds, compute), dtype=torch.uint8, device=dev)
    out = fnn.fnn_reciprocal(d1, d2, seeds, MAX_ITER, compute, workspace=ws)
    torch.cuda.synchronize()
    gen_s = time.time() - t_gen

    def step():
        fnn.fnn_reciprocal(d1, d2, seeds, MAX_ITER, compute, out=out, workspace=ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    pairs_per_s = BATCH * args.steps / elapsed

    # ---- per-kernel durations of the same steps (HIP events attached to each dispatch) --------
    fnn.fnn_trace_begin(args.steps * 64)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    trace_details = fnn.fnn_trace_end(args.steps * 64, details=True)
    trace = [(name, ms) for name, ms, _ in trace_details]
    trace_details = [row for row in trace_details if row[0] == "search_kernel"]
    by_kernel = {}
    for name, ms in trace:
        by_kernel.setdefault(name, []).append(ms)
    search_ms = by_kernel.get("search_kernel", [])
    launches_per_step = len(search_ms) / args.steps
    avg_search_ms = sum(search_ms) / max(len(search_ms), 1)

    # algorithmic work of the search launches, from the device's own per-seed iterations
    seed_iter = out["seed_iter"].cpu().numpy()
    n_pairs = out["n_pairs"].cpu().numpy()
    per_search = np.zeros(2 * MAX_ITER, dtype=np.int64)
    for b in range(BATCH):
        c = searches_from_iters(seed_iter[b], n_seeds, MAX_ITER)
        per_search[:len(c)] += np.asarray(c)
    esize = 4 if compute == "f32" else 2
    rows_per_step = int(per_search.sum())
    flops_per_step = 2.0 * D * N_PIX * rows_per_step                       # D = 24, no padding counted
    live_launches = int((per_search > 0).sum())
    # bytes: each live search streams every pair's candidate map once, gathers its queries
    # and writes an 8-byte (index, score) result per query
    bytes_per_step = live_launches * BATCH * N_PIX * D * esize + rows_per_step * (D * esize + 8)
    # fp32 maps with a 16-bit compute format: the first forward and the first backward search read the
    # caller's fp32 map (4 bytes per value) and write the prepared copy (esize bytes per value) instead
    # of reading a prepared map -- the cast that a separate prepare pass would have done
    fused_first = compute != "f32" and any(d >= 100 for _, _, d in trace_details[:2 * int(round(launches_per_step))])
    if fused_first:
        bytes_per_step += 2 * BATCH * N_PIX * D * 4
    flops_per_launch = flops_per_step / max(launches_per_step, 1)
    bytes_per_launch = bytes_per_step / max(launches_per_step, 1)
    achieved_tflops = flops_per_launch / (avg_search_ms * 1e-3) / 1e12 if avg_search_ms > 0 else 0.0
    achieved_gbs = bytes_per_launch / (avg_search_ms * 1e-3) / 1e9 if avg_search_ms > 0 else 0.0
    peak = PEAK_FP32 if compute == "f32" else PEAK_MFMA_16BIT
    kernel_ms_per_step = {k: sum(v) / args.steps for k, v in sorted(by_kernel.items())}

    # per-search view: launch i of every step has the same live query count, so average the
    # i-th search launch over the steps and set it against the roofline that bounds it
    per_search_rows = []
    lps = int(round(launches_per_step))
    for i in range(lps):
        k_act = int(per_search[i]) if i < len(per_search) else 0
        if k_act == 0:
            continue
        us = sum(search_ms[i::lps]) / max(len(search_ms[i::lps]), 1) * 1e3
        fl = 2.0 * D * N_PIX * k_act
        by = BATCH * N_PIX * D * esize + k_act * (D * esize + 8)
        if fused_first and i < 2:
            by += BATCH * N_PIX * D * 4   # fp32 map read and prepared copy written instead of a prepared map read
        t_mfma = fl / (peak * 1e12) * 1e6
        t_hbm = by / (PEAK_HBM * 1e9) * 1e6
        per_search_rows.append({
            "queries": k_act, "us": round(us, 1), "bytes": by, "TFLOP/s": round(fl / us / 1e6, 1), "GB/s": round(by / us / 1e3, 1),
            "bound": "mfma" if t_mfma >= t_hbm else "hbm", "frac_of_bound": round(max(t_mfma, t_hbm) / us, 3)})

    hbm_rows = [r for r in per_search_rows if r["bound"] == "hbm"]
    hbm_bytes = sum(r["bytes"] for r in hbm_rows)
    hbm_us = sum(r["us"] for r in hbm_rows)
    hbm_gbs = hbm_bytes / hbm_us / 1e3 if hbm_us > 0 else 0.0

    result = {
        "metric": "FastNN image pairs/sec at 512x384 D=24",
        "value": round(pairs_per_s, 2),
        "unit": "pairs/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": compute,
        "dtype_detail": {"f16": "descriptors rounded to f16, products exact in f32, f32 accumulation and selection",
                         "bf16": "descriptors rounded to bf16, products exact in f32, f32 accumulation and selection",
                         "f32": "f32 throughout"}[compute],
        "data": "synthetic",
        "config": {"workload": "configs[3]: 16 pairs 512x384 D=24 fp32 maps, FastNN reciprocal, subsample 8 "
                               "(3072 seeds/pair), max_iter 10, batched in one call", "batch": BATCH,
                   "pixels": N_PIX, "d": D, "seeds_per_pair": n_seeds, "max_iter": MAX_ITER, "compute": compute},
        "matches_per_pair": round(float(n_pairs.mean()), 1),
        "active_queries_per_search": (per_search / BATCH).round(1).tolist(),
        "kernel_ms_per_step": {k: round(v, 4) for k, v in kernel_ms_per_step.items()},
        "live_searches": per_search_rows,
        "roofline": {
            "kernel": "search_kernel", "bound": "mfma",
            "achieved": round(achieved_tflops, 2), "peak": peak, "unit": "TFLOP/s",
            "frac": round(achieved_tflops / peak, 4), "traffic": None,
            "launches_per_step": launches_per_step, "avg_launch_ms": round(avg_search_ms, 5),
            "flops_per_launch": flops_per_launch,
            "note": "algorithmic flops = 2*24*M*(active queries), averaged over all search launches of a step "
                    "(launches after every seed has converged do no work but count)",
        },
        "roofline_hbm": {
            "kernel": "search_kernel", "bound": "hbm", "achieved": round(achieved_gbs, 1), "peak": PEAK_HBM,
            "unit": "GB/s", "frac": round(achieved_gbs / PEAK_HBM, 4), "bytes_per_launch": bytes_per_launch,
        },
        "roofline_hbm_bound": {
            "kernel": "search_kernel", "bound": "hbm", "achieved": round(hbm_gbs, 1), "peak": PEAK_HBM, "unit": "GB/s",
            "frac": round(hbm_gbs / PEAK_HBM, 4), "launches_per_step": len(hbm_rows), "bytes_per_step": hbm_bytes,
            "us_per_step": round(hbm_us, 1),
            "note": "sum of algorithmic bytes / sum of durations over the search launches of a step whose bound is HBM "
                    "(few live queries: streaming the candidate maps takes longer than the matrix work at peak)",
        },
        "input_generation_s": round(gen_s, 1),
    }

    # HBM traffic of the search kernel, measured offline with rocprofv3 byte counters (the
    # command and the scaling are in profiles/); bench.py itself cannot read those counters
    traffic_file = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(traffic_file) and compute == "f16":
        with open(traffic_file) as f:
            traffic = json.load(f)
        result["roofline"]["traffic"] = traffic.get("search_kernel_bytes_per_launch")
        result["roofline_hbm"]["traffic"] = traffic.get("search_kernel_bytes_per_launch")
        result["roofline"]["traffic_source"] = traffic.get("source")
        # the counters were read on one revision of the kernels; say so when the sources have changed since
        result["roofline"]["traffic_stale"] = traffic.get("csrc_fingerprint") != csrc_fingerprint()
    else:
        traffic = {}

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- optional: the same batch as raw head outputs (normalisation fused into the prepare pass) --
    if args.normalize:
        nout = fnn.fnn_reciprocal(d1, d2, seeds, MAX_ITER, compute, normalize=True, workspace=ws)
        for _ in range(args.warmup):
            fnn.fnn_reciprocal(d1, d2, seeds, MAX_ITER, compute, out=nout, normalize=True, workspace=ws)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fnn.fnn_reciprocal(d1, d2, seeds, MAX_ITER, compute, out=nout, normalize=True, workspace=ws)
        torch.cuda.synchronize()
        n_s = (time.perf_counter() - t0) / args.steps
        fnn.fnn_trace_begin(64)  # one more step with per-kernel events, for the prepare kernel's own duration
        fnn.fnn_reciprocal(d1, d2, seeds, MAX_ITER, compute, out=nout, normalize=True, workspace=ws)
        torch.cuda.synchronize()
        prep = [ms for name, ms in fnn.fnn_trace_end(64) if name == "prep_kernel"]
        result["normalize_variant"] = {
            "ms_per_step": round(n_s * 1e3, 4), "pairs_per_s": round(BATCH / n_s, 2),
            "prep_kernel_ms": round(sum(prep) / max(len(prep), 1), 4),
            "note": "same 16 pairs with FNN_FLAG_NORMALIZE: norm, division and cast in one pass over the fp32 maps",
        }

    # ---- optional: maps the caller already holds in the compute format are read where they are ------
    if args.f16_maps and compute != "f32":
        tdt = torch.float16 if compute == "f16" else torch.bfloat16
        h1, h2 = d1.to(tdt), d2.to(tdt)
        hout = fnn.fnn_reciprocal(h1, h2, seeds, MAX_ITER, compute, workspace=ws)
        for _ in range(args.warmup):
            fnn.fnn_reciprocal(h1, h2, seeds, MAX_ITER, compute, out=hout, workspace=ws)
        torch.cuda.synchronize()
        same = all(torch.equal(hout[k], out[k]) for k in ("pairs", "n_pairs", "seed_i", "seed_j", "seed_iter"))
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fnn.fnn_reciprocal(h1, h2, seeds, MAX_ITER, compute, out=hout, workspace=ws)
        torch.cuda.synchronize()
        h_s = (time.perf_counter() - t0) / args.steps
        result["stored_in_compute_format_variant"] = {
            "ms_per_step": round(h_s * 1e3, 4), "pairs_per_s": round(BATCH / h_s, 2), "same_result": bool(same),
            "note": "same 16 pairs handed over as %s arrays: used in place, the prepare pass only clears state" % compute,
        }
        del h1, h2

    # ---- optional: the same batch with dist_func = squared distance ------------------------------
    if args.l2:
        need = fnn.fnn_workspace_bytes_opts(BATCH, N_PIX, N_PIX, D, n_seeds, compute, l2=True)
        lws = torch.empty(need, dtype=torch.uint8, device=dev)
        lout = fnn.fnn_reciprocal(d1, d2, seeds, MAX_ITER, compute, l2=True, workspace=lws)
        for _ in range(args.warmup):
            fnn.fnn_reciprocal(d1, d2, seeds, MAX_ITER, compute, out=lout, l2=True, workspace=lws)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fnn.fnn_reciprocal(d1, d2, seeds, MAX_ITER, compute, out=lout, l2=True, workspace=lws)
        torch.cuda.synchronize()
        l2_s = (time.perf_counter() - t0) / args.steps
        result["l2_variant"] = {
            "ms_per_step": round(l2_s * 1e3, 4), "pairs_per_s": round(BATCH / l2_s, 2),
            "matches_per_pair": round(float(lout["n_pairs"].float().mean().item()), 1),
            "note": "same 16 pairs, score = -|a-b|^2/2 through 4 extra channels (rows of 32 instead of 24 channels)",
        }
        del lws

    # ---- optional: one-directional search (fnn_nearest) on the same batch ------------------------------
    if args.nearest:
        nws = torch.empty(fnn.fnn_workspace_bytes(BATCH, N_PIX, N_PIX, D, N_PIX, compute), dtype=torch.uint8, device=dev)
        legs = {}
        for name, kw, reps in (("seeds_as_queries", {"q_idx": seeds}, args.steps), ("every_pixel_a_query", {}, max(args.steps // 10, 2))):
            for _ in range(2):
                fnn.fnn_nearest(d1, d2, compute=compute, workspace=nws, **kw)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                fnn.fnn_nearest(d1, d2, compute=compute, workspace=nws, **kw)
            torch.cuda.synchronize()
            n_s = (time.perf_counter() - t0) / reps
            nq = n_seeds if kw else N_PIX
            legs[name] = {"ms_per_call": round(n_s * 1e3, 4), "queries_per_pair": nq,
                          "tflops": round(2.0 * D * N_PIX * nq * BATCH / n_s / 1e12, 1)}
        legs["note"] = "fnn_nearest on the 16 pairs, fp32 maps in: image-1 queries against every pixel of image 2"
        result["nearest_batch"] = legs
        del nws

    # ---- optional: the same workload at other batch sizes ---------------------------------------------
    if args.batch_sweep:
        sweep = {}
        for nb in (1, 2, 4, 8, 32, 64):
            pick = [p % BATCH for p in range(nb)]
            b1, b2, bseeds = d1[pick].contiguous(), d2[pick].contiguous(), seeds[pick].contiguous()
            bws = torch.empty(fnn.fnn_workspace_bytes(nb, N_PIX, N_PIX, D, n_seeds, compute), dtype=torch.uint8, device=dev)
            bout = fnn.fnn_reciprocal(b1, b2, bseeds, MAX_ITER, compute, workspace=bws)
            for _ in range(3):
                fnn.fnn_reciprocal(b1, b2, bseeds, MAX_ITER, compute, out=bout, workspace=bws)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                fnn.fnn_reciprocal(b1, b2, bseeds, MAX_ITER, compute, out=bout, workspace=bws)
            torch.cuda.synchronize()
            b_s = (time.perf_counter() - t0) / args.steps
            sweep[str(nb)] = {"ms_per_call": round(b_s * 1e3, 4), "pairs_per_s": round(nb / b_s, 1)}
            del b1, b2, bseeds, bws, bout
        sweep[str(BATCH)] = {"ms_per_call": round(ms_per_step, 4), "pairs_per_s": round(pairs_per_s, 1)}
        result["batch_sweep"] = sweep

    # ---- optional: the same batch at fp32-grade precision, two ways ---------------------------------
    if args.split:
        variants = {}
        for name, comp, kw in (("split_fp16", "f16", {"split": True}), ("fp32_products", "f32", {})):
            need = fnn.fnn_workspace_bytes_opts(BATCH, N_PIX, N_PIX, D, n_seeds, comp, **kw)
            sws = torch.empty(need, dtype=torch.uint8, device=dev)
            sout = fnn.fnn_reciprocal(d1, d2, seeds, MAX_ITER, comp, workspace=sws, **kw)
            fnn.fnn_reciprocal(d1, d2, seeds, MAX_ITER, comp, out=sout, workspace=sws, **kw)
            torch.cuda.synchronize()
            reps = max(args.steps // 4, 3)
            t0 = time.perf_counter()
            for _ in range(reps):
                fnn.fnn_reciprocal(d1, d2, seeds, MAX_ITER, comp, out=sout, workspace=sws, **kw)
            torch.cuda.synchronize()
            v_s = (time.perf_counter() - t0) / reps
            variants[name] = {"ms_per_step": round(v_s * 1e3, 4), "pairs_per_s": round(BATCH / v_s, 2),
                              "matches_per_pair": round(float(sout["n_pairs"].float().mean().item()), 1)}
            if name == "split_fp16":
                split_out = {k: v.clone() for k, v in sout.items()}
            else:
                same = (sout["seed_j"] == split_out["seed_j"]) & (sout["seed_i"] == split_out["seed_i"])
                variants["seeds_with_the_same_match_in_both"] = round(float(same.float().mean().item()), 5)
            del sws, sout
        variants["note"] = ("same 16 pairs; split_fp16 = FNN_FLAG_SPLIT (rows of 80 fp16 channels, 5 K=16 matrix instructions per block), "
                            "fp32_products = compute f32 (12 K=2 fp32 matrix instructions per block)")
        result["fp32_grade_variants"] = variants

    # ---- optional: the device's own ceiling for the kernels' instruction mix ------------------------
    if not args.no_ceiling and compute != "f32":   # the loops use the 16-bit matrix instructions
        names = {0: "k16", 1: "k16_k8", 2: "k16_k16", 3: "k16_k8_fold8", 4: "k16_k8_max16", 5: "quad_16x16x32",
                 6: "bf16_k16_k8", 7: "bf16_k16_k8_fold8", 8: "bf16_k16_k8_max16"}
        ns = {names[mix]: round(fnn.fnn_measure_ceiling(mix, 65536, scratch=ws), 2) for mix in names}
        n_simd = torch.cuda.get_device_properties(dev).multi_processor_count * 4
        def tflops(ns_per_block, channels):                    # algorithmic flops of a 32x32 block with that many channels
            return round(2.0 * 32 * 32 * channels * n_simd / ns_per_block / 1e3, 1)
        result["measured_ceilings"] = {
            "ns_per_32x32_block_per_simd": ns,
            "tflops": {"k16 (16 channels)": tflops(ns["k16"], 16), "k16_k8 (24 channels)": tflops(ns["k16_k8"], 24),
                       "k16_k16 (32 channels)": tflops(ns["k16_k16"], 32),
                       "k16_k8_fold8 (search arithmetic, 24 channels)": tflops(ns["k16_k8_fold8"], 24),
                       "k16_k8_max16 (dense arithmetic, 24 channels)": tflops(ns["k16_k8_max16"], 24),
                       "quad_16x16x32 (24 channels padded to 32, four 16x16x32 instructions)": tflops(ns["quad_16x16x32"], 24),
                       "bf16_k16_k8 (24 channels)": tflops(ns["bf16_k16_k8"], 24),
                       "bf16_k16_k8_fold8 (search arithmetic, bf16)": tflops(ns["bf16_k16_k8_fold8"], 24),
                       "bf16_k16_k8_max16 (dense arithmetic, bf16)": tflops(ns["bf16_k16_k8_max16"], 24)},
            "matrix_only_ceiling_fraction_of_published_peak_d24": round(
                max(tflops(ns["k16_k8"], 24), tflops(ns["quad_16x16x32"], 24)) / PEAK_MFMA_16BIT, 4),
            "note": "register-only loops of the matrix instructions (and the 3-input maxima) of one score block, two waves per SIMD, "
                    "all %d SIMDs; the published fp16 peak is 2500 TFLOP/s" % n_simd,
        }

    # ---- optional: single-pair latency (configs[1]) ----------------------------------------------
    if not args.no_latency:
        a, b = synth.config_pair(2)
        ta, tb = torch.from_numpy(a).to(dev), torch.from_numpy(b).to(dev)
        ts = seeds[:1].contiguous()
        o1 = fnn.fnn_reciprocal(ta, tb, ts, MAX_ITER, compute, workspace=ws)
        # untimed calls first: the host thread has just slept through the long ceiling kernels, and on
        # some boxes its core takes tens of milliseconds to clock up again -- until then the 52 launches
        # of a call take the host longer to enqueue than the device needs to run them
        for _ in range(200):
            fnn.fnn_reciprocal(ta, tb, ts, MAX_ITER, compute, out=o1, workspace=ws)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(50):
            fnn.fnn_reciprocal(ta, tb, ts, MAX_ITER, compute, out=o1, workspace=ws)
        torch.cuda.synchronize()
        result["single_pair_ms"] = round((time.perf_counter() - t0) / 50 * 1e3, 4)
        # the same call recorded once into a HIP graph and replayed: the 52 launches of a call cost the
        # host more than the device needs for one pair, and a replay hands them over in one piece
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            fnn.fnn_reciprocal(ta, tb, ts, MAX_ITER, compute, out=o1, workspace=ws)
        eager = {k: v.clone() for k, v in o1.items()}
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        same = all(torch.equal(o1[k], eager[k]) for k in eager)
        t0 = time.perf_counter()
        for _ in range(50):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = round((time.perf_counter() - t0) / 50 * 1e3, 4)
        result["single_pair"] = {"workload": "configs[1]: one 512x384 D=24 pair, FastNN reciprocal, 3072 seeds, max_iter 10",
                                 "ms_per_call": result["single_pair_ms"], "ms_per_call_graph_replay": graph_ms,
                                 "graph_replay_same_result": bool(same), "matches": int(o1["n_pairs"][0]), "calls_timed": 50}
        del graph

    # ---- optional: the paper's schedules against the fused search, first search of one pair --------
    if args.contrast:
        a, b = synth.config_pair(2)
        ta, tb = torch.from_numpy(a).to(dev), torch.from_numpy(b).to(dev)
        q = seeds[0].contiguous()
        rows = 1024

        def timed(fn, reps):
            fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / reps * 1e3

        lib = fnn.load_library()
        need1 = int(lib.fnn_blocked_workspace_bytes(N_PIX, N_PIX, D, rows, 0, 1))
        need2 = int(lib.fnn_blocked_workspace_bytes(N_PIX, N_PIX, D, rows, rows, 1))
        cws = torch.empty(max(need1, need2), dtype=torch.uint8, device=dev)
        fused_ms = timed(lambda: fnn.fnn_nearest(ta, tb, q_idx=q[None], compute="f16", workspace=ws), 20)
        single_ms = timed(lambda: fnn.fnn_nearest_blocked(ta, tb, rows, 0, q_idx=q, compute="f16", workspace=cws), 5)
        double_ms = timed(lambda: fnn.fnn_nearest_blocked(ta, tb, rows, rows, q_idx=q, compute="f16", workspace=cws), 2)
        score_bytes = float(n_seeds) * N_PIX * 4
        result["schedule_contrast"] = {
            "workload": "one search of configs[1]: 3072 grid queries of image 1 against the 196608 pixels of image 2, "
                        "f16 products; every variant includes the prepare pass",
            "fused_ms": round(fused_ms, 4),
            "single_loop_ms": round(single_ms, 4), "double_loop_ms": round(double_ms, 4), "block_size": rows,
            "score_block_bytes_written_and_read": 2 * score_bytes,
            "fused_bytes": float(N_PIX) * D * 2 + n_seeds * (D * 2 + 8),
            "note": "single loop = Algorithm 2 (FastNN-Lite), double loop = Algorithm 1; both materialise the scores in HBM "
                    "and launch two kernels per block; the fused search keeps them in registers",
        }
        del cws

    # ---- dense all-pairs mutual NN on one 512x384 pair (configs[2]), fp16 ------------------------
    if not args.no_dense:
        a, b = synth.config_pair(3)
        ta, tb = torch.from_numpy(a).to(dev), torch.from_numpy(b).to(dev)
        dws = torch.empty(fnn.fnn_workspace_bytes(1, N_PIX, N_PIX, D, 0, "f16"), dtype=torch.uint8, device=dev)
        dout = fnn.fnn_mutual_dense(ta, tb, "f16", workspace=dws)
        for _ in range(3):  # warm-up, like the reciprocal leg
            fnn.fnn_mutual_dense(ta, tb, "f16", out=dout, workspace=dws)
        torch.cuda.synchronize()
        reps = 10
        t0 = time.perf_counter()
        for _ in range(reps):
            fnn.fnn_mutual_dense(ta, tb, "f16", out=dout, workspace=dws)
        torch.cuda.synchronize()
        call_ms = (time.perf_counter() - t0) / reps * 1e3
        fnn.fnn_trace_begin(reps * 16)
        for _ in range(reps):
            fnn.fnn_mutual_dense(ta, tb, "f16", out=dout, workspace=dws)
        torch.cuda.synchronize()
        dk = [ms for name, ms in fnn.fnn_trace_end(reps * 16) if name == "dense_kernel"]
        dense_ms = sum(dk) / max(len(dk), 1)
        dflops = 2.0 * D * N_PIX * N_PIX
        dtf = dflops / (dense_ms * 1e-3) / 1e12 if dense_ms > 0 else 0.0
        result["dense_mutual"] = {
            "workload": "configs[2]: one 512x384 D=24 pair, all 196608 x 196608 scores, fp16 products / fp32 accumulate",
            "call_ms": round(call_ms, 4), "tflops_call": round(dflops / (call_ms * 1e-3) / 1e12, 2),
            "mutual_pairs": int(dout["n_pairs"][0]),
            "roofline": {"kernel": "dense_kernel", "bound": "mfma", "achieved": round(dtf, 2), "peak": PEAK_MFMA_16BIT,
                         "unit": "TFLOP/s", "frac": round(dtf / PEAK_MFMA_16BIT, 4),
                         "traffic": traffic.get("dense_kernel_bytes_per_launch"),
                         "avg_launch_ms": round(dense_ms, 4), "flops_per_launch": dflops,
                         "note": "algorithmic flops 2*24*N*M (a K=16 plus a K=8 matrix instruction per 32x32 block, no padding)"},
        }

    # ---- the large pair (configs[4]): 1024x768, dense mutual NN in bf16, then FastNN reciprocal ------
    if not args.no_dense and not args.no_cfg5:
        a5, b5 = synth.config_pair(5)
        n5 = a5.shape[0]
        t5a, t5b = torch.from_numpy(a5).to(dev), torch.from_numpy(b5).to(dev)
        s5 = torch.from_numpy(synth.grid_seeds(1024, 768, SUBSAMPLE)).to(dev)[None]
        ws5 = torch.empty(fnn.fnn_workspace_bytes(1, n5, n5, D, s5.shape[1], "bf16"), dtype=torch.uint8, device=dev)
        d5 = fnn.fnn_mutual_dense(t5a, t5b, "bf16", workspace=ws5)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(3):
            fnn.fnn_mutual_dense(t5a, t5b, "bf16", out=d5, workspace=ws5)
        torch.cuda.synchronize()
        call5 = (time.perf_counter() - t0) / 3
        fnn.fnn_trace_begin(32)
        fnn.fnn_mutual_dense(t5a, t5b, "bf16", out=d5, workspace=ws5)
        torch.cuda.synchronize()
        k5 = [ms for name, ms in fnn.fnn_trace_end(32) if name == "dense_kernel"]
        r5 = fnn.fnn_reciprocal(t5a, t5b, s5, MAX_ITER, "bf16", workspace=ws5)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(10):
            fnn.fnn_reciprocal(t5a, t5b, s5, MAX_ITER, "bf16", out=r5, workspace=ws5)
        torch.cuda.synchronize()
        flops5 = 2.0 * D * n5 * n5
        result["large_pair"] = {
            "workload": "configs[4]: one 1024x768 D=24 pair, bf16 products / fp32 accumulate: all 786432 x 786432 scores, "
                        "then FastNN reciprocal from 12288 seeds",
            "dense_call_ms": round(call5 * 1e3, 3), "dense_tflops_call": round(flops5 / call5 / 1e12, 2),
            "dense_kernel_ms": round(k5[0], 3) if k5 else None,
            "dense_kernel_frac_of_mfma_peak": round(flops5 / (k5[0] * 1e-3) / 1e12 / PEAK_MFMA_16BIT, 4) if k5 else None,
            "mutual_pairs": int(d5["n_pairs"][0]),
            "reciprocal_ms": round((time.perf_counter() - t0) / 10 * 1e3, 4), "matches": int(r5["n_pairs"][0]),
        }
        del t5a, t5b, ws5, d5

    # ---- CPU oracle on a bounded sample of the same workload (baseline only) ----------------------
    if not args.no_cpu:
        import oracle
        sample = 4
        t0 = time.perf_counter()
        for p in range(sample):
            ref = oracle.reciprocal(maps[p][0], maps[p][1], seeds_np[p], MAX_ITER)
        cpu_s = time.perf_counter() - t0
        if cpu_s < 5.0:                              # many cores: take the rest of the batch too
            t0 = time.perf_counter()
            for p in range(BATCH):
                ref = oracle.reciprocal(maps[p][0], maps[p][1], seeds_np[p], MAX_ITER)
            cpu_s = time.perf_counter() - t0
            sample = BATCH
        result["cpu_baseline"] = {
            "value": round(sample / cpu_s, 4), "unit": "pairs/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": f"{sample} of the {BATCH} pairs of the same workload, full FastNN reciprocal each "
                      f"(fp32 brute-force searches), {cpu_s:.1f} s",
        }
        del ref

    # the kernels against the device's own ceiling for their arithmetic (measured above, same process)
    if "measured_ceilings" in result:
        ceil_tf = result["measured_ceilings"]["tflops"]
        first = [row for row in result.get("live_searches", []) if row.get("bound") == "mfma"]
        if first:
            result["measured_ceilings"]["first_search_fraction_of_search_arithmetic_ceiling"] = round(
                first[0]["TFLOP/s"] / ceil_tf["k16_k8_fold8 (search arithmetic, 24 channels)"], 3)
        if "dense_mutual" in result:
            result["measured_ceilings"]["dense_kernel_fraction_of_dense_arithmetic_ceiling"] = round(
                result["dense_mutual"]["roofline"]["achieved"] / ceil_tf["k16_k8_max16 (dense arithmetic, 24 channels)"], 3)
        lp = result.get("large_pair", {})
        if lp.get("dense_kernel_frac_of_mfma_peak"):
            result["measured_ceilings"]["large_pair_dense_kernel_fraction_of_bf16_dense_arithmetic_ceiling"] = round(
                lp["dense_kernel_frac_of_mfma_peak"] * PEAK_MFMA_16BIT / ceil_tf["bf16_k16_k8_max16 (dense arithmetic, bf16)"], 3)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
