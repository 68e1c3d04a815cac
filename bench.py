"""Benchmark of the TransE completion join on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2_mid_l2] [--prune on|off]

A step is one whole kgc_join (operand staging, pruning, join kernel, compaction, count read-back) on
synthetic inputs already resident in HBM.  Prints ONE JSON line: effective triple-scores/s
(N*N*R / time), the roofline of the dominant kernel (the join kernel, timed with HIP events on the
library's stream), and the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0          # MI355X dense bf16 MFMA
PEAK_VALU_TLANEOPS = 39.3          # 256 CU x 4 SIMD x 16 lanes x 2.4 GHz, plain (unpacked) float32 lane-ops
PEAK_HBM_GBS = 8000.0



def measured_traffic(workload, kernel, tile_cfg, mode):
    """HBM-side bytes per launch of a join kernel from profiles/traffic.json: separate rocprofv3 --pmc runs of this
    script (FETCH_SIZE and WRITE_SIZE, scaled by what the same counters read for a plain copy of known size).
    Counters cannot be read inside the timed run, so the figure is attached to the configuration it was taken on;
    None when the file has no entry for this workload, kernel, tile variant and mode."""
    try:
        with open(os.path.join(ROOT, "profiles", "traffic.json")) as f:
            entries = json.load(f)["entries"]
    except (OSError, ValueError, KeyError):
        return None
    for e in entries:
        if (e.get("workload"), e.get("kernel"), e.get("tile_cfg"), e.get("mode")) == (workload, kernel, tile_cfg, mode):
            return e.get("bytes_per_launch")
    return None


def calibrate(ms_target):
    """The in-library calibration loops (kgc_calibrate_mfma): what bf16 32x32x16 MFMAs sustain on this machine, alone and
    when fed as the join kernel is."""
    import paper_2307_12059_amd as kgc
    out = {"unit": "TFLOP/s", "ms_target": ms_target, "wave_tile": "4x2 blocks (128 x 64), two waves per SIMD"}
    for feed, key in ((0, "mfma_only"), (1, "head_fragments_from_lds"), (2, "lds_and_tail_fragments_from_cache")):
        rc, tf, ms = kgc.kgc_calibrate_mfma(0, feed, ms_target)
        if rc != 0:
            raise RuntimeError(f"kgc_calibrate_mfma failed with code {rc}")
        out[key] = tf
    rc, tf, ms = kgc.kgc_calibrate_mfma(1, 0, ms_target)
    out["mfma_only_4x4_tile"] = tf
    return out


def cpu_baseline(wl, target_seconds=20.0):
    """The oracle as it stands (brute-force mode, all host threads) on a bounded sample of the workload."""
    import numpy as np

    import oracle
    spec = wl.spec
    d = wl.E.shape[1]
    threads = oracle.num_threads()
    n0 = min(wl.E.shape[0], 1500)
    r0 = min(wl.Rv.shape[0], 4)
    t0 = time.perf_counter()
    oracle.join(wl.E[:n0], wl.Rv[:r0], spec.p, wl.delta, mode="brute")
    rate0 = n0 * n0 * r0 / max(time.perf_counter() - t0, 1e-6)
    ns = min(wl.E.shape[0], 4000)
    rs = int(max(1, min(wl.Rv.shape[0], round(rate0 * target_seconds / (ns * ns)))))
    t0 = time.perf_counter()
    res = oracle.join(wl.E[:ns], wl.Rv[:rs], spec.p, wl.delta, mode="brute")
    dt = time.perf_counter() - t0
    return {"value": ns * ns * rs / dt, "unit": "triple-scores/s", "cores": threads, "kind": "oracle",
            "sample": f"first {ns} entities x first {rs} relations of {spec.name} (d={d}, p={spec.p}), "
                      f"brute-force fp64, {dt:.1f} s, {res['count']} hits"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="c2_mid_l2")
    ap.add_argument("--prune", choices=["on", "off"], default="on")
    ap.add_argument("--tile", type=int, default=0)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--also-dense", type=int, default=3, help="extra dense (prune off) steps reported beside a pruned run")
    ap.add_argument("--also-factorised", type=int, default=3,
                    help="extra dense steps through the optional relation-factorised kernel (L2, d <= 282), reported beside")
    ap.add_argument("--general-form", type=int, default=0, metavar="STEPS",
                    help="also time kgc_join_ab (connector outputs supplied by the caller, pruned and dense) on the TransE connectors "
                         "A[r][h] = E[h] + Rv[r], B = E of the workload; needs R * N * d elements of extra memory")
    ap.add_argument("--se-form", type=int, default=0, metavar="STEPS",
                    help="also time kgc_join_se (structured embedding: connectors W_r e formed on the device) on the "
                         "workload's entities with seeded near-identity maps, L1, pruned and dense; R is cut to --se-relations")
    ap.add_argument("--se-relations", type=int, default=64)
    ap.add_argument("--blocks", type=int, default=0, metavar="STEPS",
                    help="also time kgc_join_blocks: the workload drained through a buffer of a quarter of its result, "
                         "4 x 4 entity blocks and 4 relation ranges")
    ap.add_argument("--topk", type=int, default=0, metavar="STEPS",
                    help="also time kgc_top1 and kgc_topk (k = 1000 over all relations, k = 100 for one relation) on the workload")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MiB",
                    help="only run a plain device copy of this many MiB (reference for the FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--calibrate-mfma", type=int, default=0, metavar="MS",
                    help="only run the MFMA calibration loops, about this many milliseconds each, and print them as one JSON line")
    ap.add_argument("--calibration-ms", type=int, default=250,
                    help="length of each in-run calibration loop behind roofline.frac_calibrated (0: skip)")
    ap.add_argument("--dense-c4", type=int, default=3, metavar="STEPS",
                    help="extra dense (prune off) steps on c4_large_l2 (N=100000, d=200), the configuration the MFMA target "
                         "is stated on, reported as dense_c4 with a roofline of its own (0: skip)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2307_12059_amd as kgc
    import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    if args.calibrate_copy > 0:
        n = args.calibrate_copy * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_MiB": args.calibrate_copy, "bytes_read": n * 4, "bytes_written": n * 4, "copies": 3}))
        return
    if args.calibrate_mfma > 0:
        print(json.dumps({"calibrate_mfma": calibrate(args.calibrate_mfma), "peak_datasheet": PEAK_BF16_TFLOPS}))
        return

    def resident(wl):
        spec = wl.spec
        if spec.storage == "bf16":
            E = torch.from_numpy(wl.E_bits.view(np.int16)).cuda().view(torch.bfloat16)
            Rv = torch.from_numpy(wl.Rv_bits.view(np.int16)).cuda().view(torch.bfloat16)
        else:
            E = torch.from_numpy(wl.E).cuda()
            Rv = torch.from_numpy(wl.Rv).cuda()
        cap = int(4 * spec.selectivity * spec.n_triples) + 4096
        return E, Rv, cap, torch.empty((cap, 4), dtype=torch.int32, device="cuda")

    wl = workloads.generate(args.workload)
    spec = wl.spec
    N, R, d, p = spec.N, spec.R, spec.d, spec.p
    E, Rv, cap, out = resident(wl)

    def run(prune, steps, warmup, factorised=False, wl=wl, E=E, Rv=Rv, cap=cap, out=out):
        spec = wl.spec
        N, R, d, p = spec.N, spec.R, spec.d, spec.p
        j = kgc.Join(dtype=spec.storage, prune=kgc.KGC_PRUNE_ON if prune else kgc.KGC_PRUNE_OFF, tile_cfg=args.tile,
                     factorised=factorised)
        res = None
        for _ in range(warmup):
            res = j.join(E, Rv, p, wl.delta, cap, out=out, fetch=False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        acc = {"ms_join": 0.0, "ms_precompute": 0.0, "ms_prune": 0.0, "ms_total": 0.0}
        for _ in range(steps):
            res = j.join(E, Rv, p, wl.delta, cap, out=out, fetch=False)
            for k in acc:
                acc[k] += res["stats"][k]
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        j.close()
        st = res["stats"]
        launches = max(1, st["join_launches"])
        ms_join = acc["ms_join"] / steps
        work = 2.0 * d * st["pairs_evaluated"]                 # flop (L2) or lane-ops (L1) of the join kernel per step
        if st["join_variant"] == 100:
            # relation-factorised kernel: the matrix work is 1/R of the per-relation form and the time goes into
            # vector arithmetic, 1.5 lane-ops per evaluated triple (one addition, half a three-way minimum)
            work = 1.5 * st["pairs_evaluated"]
            roof = {"bound": "alu", "achieved": work / (ms_join * 1e-3) / 1e12 if ms_join > 0 else 0.0,
                    "peak": PEAK_VALU_TLANEOPS, "unit": "Tlane-op/s"}
        elif p == 2:
            roof = {"bound": "mfma", "achieved": work / (ms_join * 1e-3) / 1e12 if ms_join > 0 else 0.0,
                    "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s"}
        else:
            roof = {"bound": "alu", "achieved": work / (ms_join * 1e-3) / 1e12 if ms_join > 0 else 0.0,
                    "peak": PEAK_VALU_TLANEOPS, "unit": "Tlane-op/s"}
        roof["frac"] = roof["achieved"] / roof["peak"]
        roof["traffic"] = None      # filled below for configurations with a committed counter measurement
        v = st["join_variant"]
        roof["kernel"] = ("k_join_l1" if p == 1 else "k_join_l2_fact" if v == 100 else "k_join_l2_dense" if v == 18
                          else "k_join_l2_direct" if v >= 15 else "k_join_l2_ares" if v >= 11
                          else "k_join_l2_stream" if v >= 6 else "k_join_l2")
        if prune and p == 2 and 6 <= v <= 14:
            # the pruned join: the tile kernel (128 x 128 tiles: tile by tile or row by row, chosen per batch on the
            # device) lists the accumulator blocks with candidates, a second kernel scores them in double precision;
            # ms_join spans both
            roof["kernel"] = ("k_join_l2_pairs|k_join_l2_ares" if v == 14 else roof["kernel"]) + " + k_exact_blocks"
        roof["tile_cfg"] = v
        roof["launches_per_step"] = launches
        roof["avg_launch_ms"] = ms_join / launches
        return {"ms_per_step": dt * 1e3 / steps, "count": res["count"], "code": res["code"], "stats": st,
                "phase_ms": {k: v / steps for k, v in acc.items()}, "roofline": roof}

    main_run = run(args.prune == "on", args.steps, args.warmup)
    # The join kernel's roofline is measured where every tile goes through it: the dense (prune off) mode, the
    # analogue of the paper's naive GPU approach.  When the timed run is the pruned one, a few dense steps are
    # run in the same invocation for it.
    # (a dense pass over the 1e15-triple workload would take minutes per step: the extra legs are only run when
    # their estimated cost is a few seconds)
    est_dense_s = 2.0 * d * N * N * R / (1.0e15 if p == 2 else 3.5e13)
    est_fact_s = 1.5 * N * N * R / 3.0e13
    want_dense = args.also_dense > 0 and est_dense_s * (args.also_dense + 1) <= 20.0
    dense = main_run if args.prune == "off" else (run(False, args.also_dense, 1) if want_dense else None)
    calib = calibrate(args.calibration_ms) if (p == 2 and args.calibration_ms > 0) else None

    def finish_roofline(r, wl_name, n_rows, n_rel, stats, mode):
        """traffic, algorithmic bytes and the calibrated fraction of a join kernel's roofline block"""
        r = dict(r)
        r["traffic"] = measured_traffic(wl_name, r["kernel"], r["tile_cfg"], mode)
        r["traffic_unit"] = "bytes per launch (rocprofv3 FETCH_SIZE / WRITE_SIZE of separate runs, profiles/traffic.json)"
        if r["bound"] == "mfma":
            # every staged operand row once: R * N head rows and N tail rows, each in whole 32-wide K slices of bf16
            k_read = (stats["k_padded"] + 31) // 32 * 32
            r["algorithmic_bytes"] = 2.0 * k_read * n_rows * (n_rel + 1) if mode == "dense" else None
            if calib is not None:
                r["peak_calibrated"] = calib["mfma_only"]
                r["frac_calibrated"] = r["achieved"] / calib["mfma_only"]
        return r

    roof = finish_roofline((dense or main_run)["roofline"], spec.name, N, R, (dense or main_run)["stats"],
                           "dense" if dense is not None else "pruned")
    roof["measured_in"] = "dense (prune off) steps of this invocation" if dense is not None else "the timed (pruned) steps"
    line = {
        "metric": "triple-scores/sec (effective N\u00b2R) + MFMA util %",
        "value": N * N * R / (main_run["ms_per_step"] * 1e-3),
        "unit": "triple-scores/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_run["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if p == 2 else "f32", "data": "synthetic",
        "config": {"workload": f"{spec.name}: N={N} R={R} d={d} L{p} {spec.storage} storage, delta={wl.delta:.6g}, "
                               f"selectivity {spec.selectivity:g}",
                   "prune": args.prune, "tile": [main_run["stats"]["tile_m"], main_run["stats"]["tile_n"]]},
        "hits": main_run["count"],
        "evaluated_triple_scores_per_sec": main_run["stats"]["pairs_evaluated"] / (main_run["ms_per_step"] * 1e-3),
        "tiles": {"total": main_run["stats"]["tiles_total"], "pruned": main_run["stats"]["tiles_pruned"],
                  "pruned_frac": main_run["stats"]["tiles_pruned"] / max(1, main_run["stats"]["tiles_total"])},
        "groups": main_run["stats"]["groups"],
        "candidates": main_run["stats"]["candidates"],
        "exact_blocks": main_run["stats"]["exact_blocks"],
        "phase_ms": main_run["phase_ms"],
        "roofline": roof,
        # MFMA utilisation of the dense join tiles: algorithmic flop rate over the bf16 MFMA peak (the counter
        # view, MFMA-busy cycles and the sustained clock, is in profiles/counters_*.txt)
        "mfma_util_pct": 100.0 * roof["frac"] if p == 2 else None,
    }
    if calib is not None:
        line["calibration"] = calib
    if args.prune == "on":
        # the timed (pruned) steps' own join kernel: same accounting, on the pairs of the surviving tiles
        line["roofline_pruned"] = finish_roofline(main_run["roofline"], spec.name, N, R, main_run["stats"], "pruned")
    if dense is not None and dense is not main_run:
        line["dense"] = {"ms_per_step": dense["ms_per_step"], "value": N * N * R / (dense["ms_per_step"] * 1e-3),
                         "hits": dense["count"], "phase_ms": dense["phase_ms"],
                         "speedup_prune_on_vs_off": dense["ms_per_step"] / main_run["ms_per_step"]}
        assert dense["count"] == main_run["count"], "pruned and dense runs disagree on the number of hits"
    if p == 2 and d <= 282 and args.also_factorised > 0 and est_fact_s * (args.also_factorised + 1) <= 20.0:
        fr = run(False, args.also_factorised, 1, factorised=True)
        assert fr["count"] == main_run["count"], "factorised and main runs disagree on the number of hits"
        line["dense_factorised"] = {"ms_per_step": fr["ms_per_step"], "value": N * N * R / (fr["ms_per_step"] * 1e-3),
                                    "hits": fr["count"], "phase_ms": fr["phase_ms"], "roofline": fr["roofline"]}
    if args.dense_c4 > 0 and spec.name != "c4_large_l2" and p == 2:
        # the MFMA target (>= 50 % of the bf16 peak on dense tiles) is stated at N = 100,000, d = 200: a few dense steps there
        wl4 = workloads.generate("c4_large_l2")
        E4, Rv4, cap4, out4 = resident(wl4)
        r4 = run(False, args.dense_c4, 1, wl=wl4, E=E4, Rv=Rv4, cap=cap4, out=out4)
        s4 = wl4.spec
        roof4 = finish_roofline(r4["roofline"], s4.name, s4.N, s4.R, r4["stats"], "dense")
        line["dense_c4"] = {"workload": f"{s4.name}: N={s4.N} R={s4.R} d={s4.d} L2 {s4.storage} storage, delta={wl4.delta:.6g}, prune off",
                            "steps": args.dense_c4, "ms_per_step": r4["ms_per_step"],
                            "value": s4.N * s4.N * s4.R / (r4["ms_per_step"] * 1e-3), "hits": r4["count"],
                            "phase_ms": r4["phase_ms"], "roofline": roof4, "mfma_util_pct": 100.0 * roof4["frac"]}
        del E4, Rv4, out4
    if args.general_form > 0:
        # the general form of Section 4.3 on the TransE connectors: same kernels, connector outputs supplied here
        A = (E.unsqueeze(0) + Rv.unsqueeze(1)).contiguous()
        line["general_form"] = {"note": "hits differ from the main run only by the float rounding of A = E + Rv"}
        for label, mode in (("pruned", kgc.KGC_PRUNE_ON), ("dense", kgc.KGC_PRUNE_OFF)):
            j = kgc.Join(dtype=spec.storage, prune=mode)
            res = j.join_ab(A, E, p, wl.delta, cap)                     # warm-up
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.general_form):
                res = j.join_ab(A, E, p, wl.delta, cap)
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / args.general_form
            j.close()
            st = res["stats"]
            line["general_form"][label] = {
                "ms_per_step": ms, "value": N * N * R / (ms * 1e-3), "hits": res["count"], "launches": st["join_launches"],
                "tiles_pruned_frac": st["tiles_pruned"] / max(1, st["tiles_total"]),
                "achieved": 2.0 * d * st["pairs_evaluated"] / (st["ms_join"] * 1e-3) / 1e12,
                "unit": "TFLOP/s" if p == 2 else "Tlane-op/s (join, staging and bound test together)"}
    if args.se_form > 0:
        # the structured-embedding instance of Section 4.3: a = W1_r h, b = W2_r t under the L1 norm; the maps are
        # seeded perturbations of the identity, so that the clusters of the workload survive and hits exist
        Rs = min(R, args.se_relations)
        gen = torch.Generator(device="cpu").manual_seed(4242)
        eye = torch.eye(d).unsqueeze(0)
        W1 = (eye + 0.03 / d ** 0.5 * torch.randn((Rs, d, d), generator=gen)).to(E.dtype).cuda().contiguous()
        W2 = (eye + 0.03 / d ** 0.5 * torch.randn((Rs, d, d), generator=gen)).to(E.dtype).cuda().contiguous()
        # threshold: 2.5 standard deviations below the mean L1 distance of two members of a cluster of the workload
        # (per-coordinate difference N(0, 2 sigma^2): mean |x| = 0.798 sqrt(2) sigma, standard deviation 0.603 sqrt(2) sigma)
        sig = {"c1_tiny_l2": 0.1, "c2_mid_l2": 0.15, "c3_l1": 0.1, "c4_large_l2": 0.1, "c5_scale_l2": 0.05}.get(spec.name, 0.1)
        delta_se = 1.4142 * sig * (0.798 * d - 2.5 * 0.603 * d ** 0.5)
        cap_se = 1 << 24
        line["se_form"] = {"relations": Rs, "p": 1, "delta": delta_se,
                           "connector_flop": 2.0 * 2.0 * Rs * N * d * d}
        for label, mode in (("pruned", kgc.KGC_PRUNE_ON), ("dense", kgc.KGC_PRUNE_OFF)):
            j = kgc.Join(dtype=spec.storage, prune=mode)
            res = j.join_se(E, W1, W2, 1, delta_se, cap_se, fetch=False)   # warm-up
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.se_form):
                res = j.join_se(E, W1, W2, 1, delta_se, cap_se, fetch=False)
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / args.se_form
            j.close()
            line["se_form"][label] = {"ms_per_step": ms, "value": N * N * Rs / (ms * 1e-3), "hits": res["count"],
                                      "code": res["code"], "relation_batches": res["stats"]["relation_batches"],
                                      "ms_join_ab_total": res["stats"]["ms_total"]}
    if args.blocks > 0:
        # the join unit by unit (Section 4.7): 4 x 4 blocks of the row order, 4 relation ranges, a buffer of a quarter of
        # the result; every call's records are fetched to the host as a caller draining the buffer would
        hits = main_run["count"]
        cap_b = max(1024, hits // 4)
        block_rows = (N // 4 + 255) // 256 * 256
        rel_block = (R + 3) // 4
        line["blocks"] = {"cap": cap_b, "block_rows": block_rows, "rel_block": rel_block}
        for label, mode in (("pruned", kgc.KGC_PRUNE_ON), ("dense", kgc.KGC_PRUNE_OFF)):
            if mode == kgc.KGC_PRUNE_OFF and est_dense_s * 16 > 30.0:
                continue          # (every unit of a dense join stages and joins its window: only for small workloads)
            j = kgc.Join(dtype=spec.storage, prune=mode)
            ms_all, calls, total, units = 0.0, 0, 0, 0
            for it in range(args.blocks + 1):
                cursor, calls, total, cap_now = None, 0, 0, cap_b
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                while True:
                    got = j.join_blocks(E, Rv, p, wl.delta, cap_now, block_rows, rel_block, cursor)
                    cursor = got["cursor"]
                    calls += 1
                    total += got["count"]
                    if got["code"] == kgc.KGC_OVERFLOW and got["count"] == 0:
                        cap_now = int(cursor.need)
                    if got["code"] == 0:
                        break
                if it > 0:
                    ms_all += (time.perf_counter() - t0) * 1e3
                units = int(cursor.units)
            j.close()
            assert total == hits, "the drained join and the main run disagree on the number of hits"
            line["blocks"][label] = {"ms_per_join": ms_all / args.blocks, "calls": calls, "units": units, "hits": total}
    if args.topk > 0:
        # the smallest distances instead of a threshold (the Top-1 score of Section 3.3 and its k-best form)
        j = kgc.Join(dtype=spec.storage, prune=kgc.KGC_PRUNE_ON)
        line["topk"] = {}
        for label, fn in (("top1", lambda: j.top1(E, Rv, p)),
                          ("top1000", lambda: j.topk(E, Rv, p, 1000)),
                          ("top100_of_relation_0", lambda: j.topk(E, Rv, p, 100, r_range=(0, 1)))):
            res = fn()                                                 # warm-up
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.topk):
                res = fn()
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / args.topk
            line["topk"][label] = {"ms_per_call": ms, "smallest_dist": float(res["dist"] if label == "top1" else res["dist"][0]),
                                   "found": 1 if label == "top1" else int(res["count"])}
        j.close()
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
