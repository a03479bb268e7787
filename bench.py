#!/usr/bin/env python3
"""Benchmark of the decode-time MoE layer step with speculative expert prefetch on one MI355X.

A "step" is one decode token: all L layer steps of the hot path (route, predict, prefetch,
expert GEMVs, combine) for one batch of synthetic input, with expert weights already resident
in the pinned host pool and everything else in HBM.  The headline value is tokens/s in
speculative mode; on-demand loading is measured beside it on the same tokens, interleaved.

Prints one JSON line (see README for the fields).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
# HBM bytes per launch of the dominant kernel measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a
# plain copy of known size (profiles/bench_c2_qwen3_pmc_hbm_traffic.md, profiles/bench_c5_qwen3_b32_kernel_trace_and_pmc.md);
# only for the workloads it was measured on
PMC_TRAFFIC_BYTES = {"c2_qwen3_30b_a3b": 50487521, "c5_qwen3_b32": 304003275}
LINK_PEAK_GBS = 64.0           # PCIe Gen5 x16, one direction, nominal


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=48, help="timed decode tokens per mode per repetition")
    p.add_argument("--warmup", type=int, default=4, help="untimed decode tokens before each timed run")
    p.add_argument("--reps", type=int, default=3, help="interleaved A/B repetitions")
    p.add_argument("--workload", default="c2_qwen3_30b_a3b")
    p.add_argument("--layers", type=int, default=0, help="development only: fewer layers than the workload names")
    p.add_argument("--cpu-tokens", type=int, default=4, help="tokens the CPU checker is timed on (0 = skip)")
    p.add_argument("--with-hint", action="store_true",
                   help="also time the prefetch-as-hint policy (prefetch the prediction, execute the true experts, re-fetch misses)")
    p.add_argument("--diagnostics", action="store_true",
                   help="also collect per-layer recall@k, rank agreement and cosine similarity for the quasi-hidden "
                        "state and for the baseline signal s_l (the statistics of the paper's per-layer figures)")
    p.add_argument("--calibrate-copy", action="store_true",
                   help="also run one plain 256 MiB device-to-device copy (reference dispatch for scaling PMC byte counters)")
    p.add_argument("--prefill", type=int, default=512, metavar="P",
                   help="also time the prefill step on a prompt of P tokens (every expert of every layer streamed); 0 = skip")
    p.add_argument("--kernel-reps", type=int, default=480)
    p.add_argument("--copy-engine", choices=["auto", "kernel", "dma", "dma2"], default="auto",
                   help="auto: each mode gets the engine that is fastest for it (speculative: two DMA queues, "
                        "on-demand: gather-copy kernel)")
    return p.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run with --gpus 1.  How the path would shard is described in DESIGN.md.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2603_19289_amd import moe_spec as M
    from paper_2603_19289_amd import workload as W
    from paper_2603_19289_amd.engine import engine_for

    M.lib()          # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")

    wl = W.CONFIGS[args.workload]
    reduced = bool(args.layers) and args.layers != wl.n_layers
    if args.layers:
        wl = wl.with_(n_layers=args.layers)
    K, Wm, B, L, H = args.steps, args.warmup, wl.batch, wl.n_layers, wl.hidden
    T = K + Wm

    t_setup = time.time()
    res = W.make_resident(wl)
    pool = W.alloc_pinned_pool(wl)
    W.fill_experts_gpu(wl, pool)
    x0_np, eps_np = W.make_inputs(wl, tokens=T)
    x0 = torch.from_numpy(x0_np).to(dev)
    eps = torch.from_numpy(eps_np).to(dev)
    log(f"[bench] {wl.name}: pool {L * wl.n_experts * wl.expert_bytes / 1e9:.1f} GB pinned, setup {time.time() - t_setup:.1f} s")

    codes = {"kernel": M.COPY_KERNEL, "dma": M.COPY_DMA, "dma2": M.COPY_DMA2}
    # the second DMA queue pays off from a few MB per expert on; below that their set-up latency dominates
    spec_auto = "dma2" if wl.expert_bytes >= (4 << 20) else "kernel"
    engine_names = {"speculative": spec_auto if args.copy_engine == "auto" else args.copy_engine,
                    "on_demand": "kernel" if args.copy_engine == "auto" else args.copy_engine}
    mode_codes = {"speculative": M.MODE_SPECULATIVE, "on_demand": M.MODE_ON_DEMAND,
                  "prefetch_hint": M.MODE_PREFETCH_HINT}
    if args.with_hint:
        engine_names["prefetch_hint"] = "kernel" if args.copy_engine == "auto" else args.copy_engine

    def make(mode, profile, predict=0):
        return engine_for(wl, mode_codes[mode], res, pool, predict_in_on_demand=predict, profile=profile,
                          copy_engine=codes[engine_names[mode]])

    modes = ["speculative", "on_demand"] + (["prefetch_hint"] if args.with_hint else [])

    def run_tokens(eng, t_first, n):
        out = torch.empty((B, H), dtype=torch.float32, device=dev)
        rbuf = [torch.empty((B, H), dtype=torch.float32, device=dev) for _ in range(2)]
        with torch.cuda.stream(eng.compute):
            for t in range(t_first, t_first + n):
                eng.begin_token()
                r = x0[t]
                for l in range(L):
                    eng.layer_step(l, r, out, sync_input=False)
                    if l + 1 < L:
                        r = eng.advance(r, out, eps[t, l], wl.res_a, wl.res_b, rbuf[l & 1])

    def timed(eng):
        # one context alive at a time: every context owns streams, and idle ones would share the
        # process's few hardware queues with the one being timed
        eng.reset()
        run_tokens(eng, 0, Wm)
        torch.cuda.synchronize()
        before = eng.stats()
        t0 = time.perf_counter()
        run_tokens(eng, Wm, K)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        after = eng.stats()
        d = {k: after[k] - before[k] for k in after}
        return dt, d

    results = {m: [] for m in modes}
    for rep in range(args.reps):
        for mode in modes:
            eng = make(mode, 0)
            dt, d = timed(eng)
            eng.close()
            results[mode].append((dt, d))
            log(f"[bench] rep {rep} {mode}: TPOT {dt / K * 1e3:.3f} ms, H2D {d['h2d_bytes'] / dt / 1e9:.2f} GB/s "
                f"({d['cache_misses']} misses, {d['cache_hits']} hits)")

    def summary(mode):
        tp = np.array([dt / K * 1e3 for dt, _ in results[mode]])
        d = results[mode][-1][1]
        dt = results[mode][-1][0]
        return {"tpot_ms": float(tp.mean()), "tpot_ms_std": float(tp.std()), "tokens_per_s": float(B / (tp.mean() / 1e3)),
                "h2d_gb_per_token": d["h2d_bytes"] / K / 1e9, "h2d_gbs_wall": d["h2d_bytes"] / dt / 1e9,
                "link_frac_wall_nominal": d["h2d_bytes"] / dt / 1e9 / LINK_PEAK_GBS,
                "cache_hit_rate": d["cache_hits"] / max(1, d["cache_hits"] + d["cache_misses"]),
                "hbm_gb_algorithmic_per_token": d["hbm_bytes_algorithmic"] / K / 1e9}

    spec, ond = summary("speculative"), summary("on_demand")
    hint = summary("prefetch_hint") if args.with_hint else None

    # ---- instrumented legs (separate contexts with timing events): compute / copy / stall breakdown,
    #      hit statistics, and the duration of every gate/up kernel launch inside the token loop
    breakdown = {}
    gu_ms, gu_n = 0.0, 0
    gemv_bytes = wl.top_k * 2 * wl.inter * H * wl.elem_bytes * 1.0
    prof_eng = None
    for mode in ("speculative", "on_demand"):
        eng = make(mode, 1, predict=1)
        dt, d = timed(eng)
        busy = d["copy_ms"]
        gu_ms += d["gateup_ms"]
        gu_n += d["gateup_launches"]
        breakdown[mode] = {
            "wall_ms_per_token": dt / K * 1e3, "copy_ms_per_token": d["copy_ms"] / K,
            "compute_ms_per_token": d["compute_ms"] / K, "stall_ms_per_token": d["stall_ms"] / K,
            "idle_ms_per_token": max(0.0, (dt * 1e3 - d["copy_ms"] - d["compute_ms"]) / K) if mode == "on_demand" else None,
            "h2d_gbs_while_copying": d["h2d_bytes"] / (busy / 1e3) / 1e9 if busy > 0 else None,
            "link_frac_while_copying_nominal": d["h2d_bytes"] / (busy / 1e3) / 1e9 / LINK_PEAK_GBS if busy > 0 else None,
            "overlap_fraction": ((d["copy_ms"] + d["compute_ms"] - dt * 1e3) / min(d["copy_ms"], d["compute_ms"]))
            if min(d["copy_ms"], d["compute_ms"]) > 0 else None,
            "hit_rate_recall_at_k": d["hits"] / max(1, d["predictions"]),
            "gateup_us_per_launch_in_flow": d["gateup_ms"] / max(1, d["gateup_launches"]) * 1e3,
            "gateup_gbs_in_flow": gemv_bytes / (d["gateup_ms"] / max(1, d["gateup_launches"]) / 1e3) / 1e9
            if d["gateup_ms"] > 0 else None}
        if mode == "on_demand":
            prof_eng = eng
        else:
            eng.close()

    # ---- roofline of the dominant kernel (gate/up GEMV).  achieved = algorithmic bytes per launch over the
    #      mean launch duration inside the two instrumented token loops (event pairs on the compute stream);
    #      the same kernels timed back to back on cold slots, without the token loop, are listed beside it
    kern = {}
    mfma = wl.dtype == "bf16" and B >= 2          # the kernels a batch of this size runs on
    which_list = [(0, "expert_gateup_gemv"), (3, "pure_read_of_the_same_bytes"), (1, "expert_down_combine_gemv"),
                  (2, "router")] + ([(4, "expert_gateup_mfma"), (5, "expert_down_mfma")] if mfma else [])
    for which, name in which_list:
        ms, nbytes = prof_eng.time_kernel(which, args.kernel_reps)
        kern[name] = {"us_per_launch": ms * 1e3, "bytes_per_launch": nbytes, "gbs": nbytes / (ms / 1e3) / 1e9}
    prof_eng.close()
    dom_name = "expert_gateup_mfma" if mfma else "expert_gateup_gemv"
    dom = kern[dom_name]
    roofline = {"bound": "hbm",
                "kernel": ("expert_mfma_kernel<gate/up> (W_gate/W_up tiles + SwiGLU on the matrix cores, batch %d over %d resident experts)"
                           % (B, dom["bytes_per_launch"] // (2 * wl.inter * H * wl.elem_bytes))) if mfma else
                          ("gateup_b1 kernels (expert W_gate/W_up GEMV + SwiGLU, batch 1)" if B == 1 else "gate/up expert kernel (batch 1 shape)"),
                "achieved": dom["gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": dom["gbs"] / HBM_PEAK_GBS,
                "traffic": PMC_TRAFFIC_BYTES.get(wl.name) if not reduced else None, "launches_timed": args.kernel_reps, "bytes_per_launch": dom["bytes_per_launch"],
                "us_per_launch": dom["us_per_launch"],
                "how": "two HIP events on the compute stream around back-to-back launches, each on the slots of the next layer",
                "other_kernels": {k: v for k, v in kern.items() if k != dom_name},
                "in_token_loop_event_pairs": {m: {"us_per_launch": breakdown[m]["gateup_us_per_launch_in_flow"],
                                                   "gbs": breakdown[m]["gateup_gbs_in_flow"]} for m in breakdown},
                "in_token_loop_launches": gu_n}

    # ---- the paper's analytic model (Sec. 5.1): prefetching can hide min(copy, compute) per layer.  Compute per
    #      token two ways: the kernels of one layer step timed back to back (two routing launches, gate/up,
    #      down+combine) times L, and the event-bracketed spans of the instrumented on-demand leg (which also
    #      hold the event records and the residual driver); layers taken as alike.  Against the reduction
    #      measured between the two un-instrumented modes.
    od = breakdown["on_demand"]
    kernel_ms = L * (2 * kern["router"]["us_per_launch"] + kern["expert_gateup_gemv"]["us_per_launch"] +
                     kern["expert_down_combine_gemv"]["us_per_launch"]) / 1e3 if B == 1 else None
    tpot_model = {"copy_ms_per_token": od["copy_ms_per_token"],
                  "compute_ms_per_token_kernels_back_to_back": kernel_ms,
                  "compute_ms_per_token_event_spans": od["compute_ms_per_token"],
                  "predicted_improvement_ms": min(od["copy_ms_per_token"], kernel_ms) if kernel_ms else None,
                  "predicted_improvement_ms_from_event_spans": min(od["copy_ms_per_token"], od["compute_ms_per_token"]),
                  "measured_improvement_ms": ond["tpot_ms"] - spec["tpot_ms"],
                  "predicted_reduction": min(od["copy_ms_per_token"], kernel_ms) / ond["tpot_ms"] if kernel_ms else None,
                  "measured_reduction": 1.0 - spec["tpot_ms"] / ond["tpot_ms"]}

    diagnostics = None
    if args.diagnostics:
        diagnostics = {}
        for signal, name in ((0, "quasi_hidden_state"), (1, "baseline_s_l")):
            eng = engine_for(wl, M.MODE_ON_DEMAND, res, pool, predict_in_on_demand=1, copy_engine=codes[engine_names["on_demand"]],
                             predict_signal=signal, diagnostics=1)
            run_tokens(eng, 0, min(T, 16))
            per = [eng.layer_diagnostics(l) for l in range(L)]
            eng.close()
            diagnostics[name] = {
                "tokens": min(T, 16), "execution": "true experts (on-demand), so both signals see the same trajectory",
                "recall_at_k_per_layer": [round(d["hits"] / d["predictions"], 4) if d["predictions"] else None for d in per],
                "cosine_to_next_router_input_per_layer": [round(d["cos_sum"] / d["cos_count"], 4) if d["cos_count"] else None for d in per],
                "top_rank_agreement_per_layer": [round(d["rank_match"][0] / d["cos_count"], 4) if d["cos_count"] else None for d in per]}

    # ---- prefill (Sec. 5.2, prefill phase): all prompt tokens per layer, every expert streamed layer-ahead
    prefill = None
    if args.prefill > 0:
        import dataclasses
        P = args.prefill
        px0, peps = W.make_inputs(dataclasses.replace(wl, batch=P), tokens=1)
        pr0 = torch.from_numpy(px0[0]).to(dev)
        pe = torch.from_numpy(peps[0]).to(dev)
        name = spec_auto if args.copy_engine == "auto" else args.copy_engine
        eng = engine_for(wl, M.MODE_SPECULATIVE, res, pool, copy_engine=codes[name], max_batch=min(64, P),
                         max_prefill_tokens=P)
        pout = torch.empty((P, H), dtype=torch.float32, device=dev)
        pbuf = [torch.empty((P, H), dtype=torch.float32, device=dev) for _ in range(2)]

        def prompt_pass():
            with torch.cuda.stream(eng.compute):
                r = pr0
                for l in range(L):
                    eng.prefill_layer_step(l, r, pout, sync_input=False)
                    if l + 1 < L:
                        r = eng.advance(r, pout, pe[l], wl.res_a, wl.res_b, pbuf[l & 1])
        prompt_pass()
        torch.cuda.synchronize()
        before = eng.stats()
        t0 = time.perf_counter()
        for _ in range(2):
            prompt_pass()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / 2
        after = eng.stats()
        eng.close()
        nbytes = (after["h2d_bytes"] - before["h2d_bytes"]) / 2
        prefill = {"prompt_tokens": P, "micro_batch": min(64, P), "copy_engine": name, "ms_per_prompt": dt * 1e3,
                   "ms_per_layer": dt * 1e3 / L, "prompt_tokens_per_s": P / dt, "h2d_gb_per_prompt": nbytes / 1e9,
                   "h2d_gbs_wall": nbytes / dt / 1e9, "link_frac_wall_nominal": nbytes / dt / 1e9 / LINK_PEAK_GBS}
        log(f"[bench] prefill P={P}: {dt * 1e3:.1f} ms per prompt, {dt * 1e3 / L:.2f} ms per layer, H2D {nbytes / dt / 1e9:.2f} GB/s")

    if args.calibrate_copy:
        a = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
        log("[bench] calibration copy: 268435456 bytes read + 268435456 bytes written in one dispatch")

    # ---- the CPU checker timed on this host, on a bounded prefix of the same workload
    cpu = None
    if args.cpu_tokens > 0:
        from oracle import moe_oracle as O
        n_tok = min(args.cpu_tokens, T)
        pool_np = W.PoolView(pool)
        model = O.OracleModel(n_layers=L, hidden=H, n_experts=wl.n_experts, top_k=wl.top_k, inter=wl.inter,
                              dtype=O.DTYPE_BF16 if wl.dtype == "bf16" else O.DTYPE_F32, router_w=res["router_w"],
                              rms_gain=res["rms_gain"], dvecs=res["dvecs"], experts=pool_np)
        orc = O.MoEOracle(model, O.MODE_SPECULATIVE, wl.slots)
        t0 = time.perf_counter()
        O.run_tokens(orc, x0_np[:n_tok], lambda t, l, r, o: W.advance_residual(wl, r, o, eps_np[t, l]))
        dt = time.perf_counter() - t0
        try:
            from threadpoolctl import threadpool_info
            threads = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
        except Exception:
            threads = os.cpu_count()
        cpu = {"value": B * n_tok / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
               "sample": f"first {n_tok} decode tokens of the same workload (all {L} layers, speculative mode), "
                         f"{dt:.1f} s of numpy float64 on the host"}

    line = {
        "metric": "decode tokens/s with speculative expert prefetch (TPOT in ms_per_step); on-demand loading beside it",
        "value": spec["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": spec["tpot_ms"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name + (" (REDUCED LAYERS, development run)" if reduced else ""),
                   "layers": L, "hidden": H, "experts": wl.n_experts, "top_k": wl.top_k, "inter": wl.inter,
                   "batch": B, "slots_per_layer": wl.slots, "reps": args.reps, "copy_engine": engine_names,
                   "expert_bytes": wl.expert_bytes, "host_pool_gb": L * wl.n_experts * wl.expert_bytes / 1e9},
        "speculative": spec, "on_demand": ond, "prefetch_hint": hint,
        "tpot_reduction_vs_on_demand": 1.0 - spec["tpot_ms"] / ond["tpot_ms"],
        "breakdown_instrumented": breakdown, "tpot_model_sec_5_1": tpot_model,
        "link": {"peak_nominal_gbs": LINK_PEAK_GBS, "achieved_gbs_speculative_wall": spec["h2d_gbs_wall"],
                 "achieved_gbs_on_demand_wall": ond["h2d_gbs_wall"]},
        "roofline": roofline, "cpu_baseline": cpu, "signal_diagnostics": diagnostics,
        "prefill": prefill,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
