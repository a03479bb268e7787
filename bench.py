#!/usr/bin/env python3
"""Benchmark of the decode-time MoE layer step with speculative expert prefetch on one MI355X.

A "step" is one decode token: all L layer steps of the hot path (route + predict, prefetch, expert
GEMVs, combine) for one batch of synthetic input, with expert weights already resident in the pinned
host pool and everything else in HBM.  The headline value is tokens/s in speculative mode on the
Qwen3-30B-A3B-shaped workload; on-demand loading is measured beside it on the same tokens, interleaved.
After the headline workload two more are timed in the same run, shorter: the batch-32 workload (the
matrix-core expert path) and the tiny float32 one.

Prints one JSON line: metric, value (tokens/s), ms_per_step (TPOT), both modes' figures, the instrumented
compute / copy / stall breakdown, `roofline` (dominant kernel, every hot kernel, the layer step), the paper's
analytic model against the measurement, `cpu_baseline`, and the same for the other workloads of the run.
"""
import argparse
import json
import os
import platform
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
LINK_PEAK_GBS = 64.0           # PCIe Gen5 x16, one direction, nominal
# HBM bytes per launch (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a plain copy of known size) and
# per-leg kernel durations (rocprofv3 --kernel-trace) of this same command, as last written by
# `python -m paper_2603_19289_amd.profile_summary` next to the .md summaries
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")
TRACE_FILE = os.path.join(ROOT, "profiles", "kernel_trace_by_leg.json")

# time_kernel modes (include/moe_spec.h) -> name in the output, and the kernel's name in a profile
K_GATEUP, K_DOWN, K_ROUTE_OLD, K_READ_GU, K_MFMA_GU, K_MFMA_DOWN, K_ROUTE_TRUE, K_ROUTE_PAIR, K_READ_DOWN = 0, 1, 2, 3, 4, 5, 6, 7, 9
KERNEL_NAMES = {K_GATEUP: ("expert_gateup_gemv", "gateup_b1"), K_DOWN: ("expert_down_combine_gemv", "down_combine_b1"),
                K_READ_GU: ("pure_read_of_the_gateup_bytes", "stream_read"), K_READ_DOWN: ("pure_read_of_the_down_bytes", "stream_read"),
                K_MFMA_GU: ("expert_gateup_mfma", "expert_mfma_kernel<true"), K_MFMA_DOWN: ("expert_down_mfma", "expert_mfma_kernel<false"),
                K_ROUTE_TRUE: ("route_true_only", "route_pair_kernel"), K_ROUTE_PAIR: ("route_true_and_prediction", "route_pair_kernel")}


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
    p.add_argument("--extra", default="auto",
                   help="comma-separated workloads timed after the headline one, shorter (auto: c5_qwen3_b32, c1_tiny, "
                        "c3_gpt_oss_20b, c3_gpt_oss_20b_b8 and c4_mixtral_8x7b after the default workload, none otherwise; 'none' to skip)")
    p.add_argument("--cpu-tokens", type=int, default=3, help="tokens the CPU checker is timed on with all cores (0 = skip); "
                                                           "one more token is timed on a single thread")
    p.add_argument("--with-hint", action="store_true",
                   help="also time the prefetch-as-hint policy (prefetch the prediction, execute the true experts, re-fetch misses)")
    p.add_argument("--with-lookahead", action="store_true",
                   help="also time speculative mode with the two-layer lookahead (lookahead = 2: experts predicted for layer "
                        "l+2 are requested as a cache hint one layer before the regular prefetch), on every workload of the run")
    p.add_argument("--diagnostics", action="store_true",
                   help="also collect per-layer recall@k, rank agreement and cosine similarity for the quasi-hidden "
                        "state and for the baseline signal s_l (the statistics of the paper's per-layer figures)")
    p.add_argument("--calibrate-copy", action="store_true",
                   help="also run one plain 256 MiB device-to-device copy (reference dispatch for scaling PMC byte counters)")
    p.add_argument("--prefill", type=int, default=512, metavar="P",
                   help="also time the prefill step on a prompt of P tokens (every expert of every layer streamed); 0 = skip")
    p.add_argument("--kernel-reps", type=int, default=480)
    p.add_argument("--legs-file", default="", help="write the order of the run's legs and their kernel launch counts here "
                                                 "(read by paper_2603_19289_amd.profile_summary to split a kernel trace)")
    p.add_argument("--per-layer-misses", action="store_true", help="also report cache misses per layer for both modes")
    p.add_argument("--copy-engine", choices=["auto", "kernel", "dma", "dma2"], default="auto",
                   help="auto: each mode gets the engine that is fastest for it (speculative: two DMA queues, "
                        "on-demand: gather-copy kernel)")
    return p.parse_args()


def load_json(path):
    try:
        with open(path) as f:
            return json.load(f)
    except (OSError, ValueError):
        return None


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return platform.processor() or "unknown"


class Bench:
    """One run of bench.py: shared device state, the list of legs, and the per-workload measurements."""

    def __init__(self, args):
        import torch
        from paper_2603_19289_amd import moe_spec as M
        from paper_2603_19289_amd import workload as W
        self.args, self.torch, self.M, self.W = args, torch, M, W
        M.lib()          # fail loudly if the HIP library is missing
        assert torch.cuda.is_available(), "bench.py needs a GPU"
        self.dev = torch.device("cuda:0")
        self.legs = []
        self.traffic = load_json(TRAFFIC_FILE) or {}
        self.trace = load_json(TRACE_FILE) or {}
        self.codes = {"kernel": M.COPY_KERNEL, "dma": M.COPY_DMA, "dma2": M.COPY_DMA2}
        self.mode_codes = {"speculative": M.MODE_SPECULATIVE, "on_demand": M.MODE_ON_DEMAND,
                           "prefetch_hint": M.MODE_PREFETCH_HINT, "speculative_lookahead2": M.MODE_SPECULATIVE}

    def leg(self, name, counts=None, uncounted=()):
        """counts: launches of each kernel (by a substring of its name) in this leg; uncounted: kernels the leg
        launches a data-dependent number of times (see leg_waves)."""
        self.legs.append({"leg": name, "counts": dict(counts or {}), "uncounted": list(uncounted)})

    def leg_waves(self, eng):
        """The leg just run launched its expert kernels once per cache wave: now that the count is known, record it."""
        leg = self.legs[-1]
        waves = eng.stats()["cache_waves"]
        for sym in leg["uncounted"]:
            leg["counts"][sym] = waves
        leg["uncounted"] = []

    # ------------------------------------------------------------------ one workload
    def run(self, wl, K, Wm, reps, pool=None, headline=False):
        """TPOT of both modes (interleaved repetitions), the instrumented breakdown, the kernels timed back to
        back, and (headline only) prefill, hint mode, diagnostics and the CPU checker.  Returns (result, pool)."""
        import numpy as np
        from paper_2603_19289_amd.engine import engine_for
        args, torch, M, W, dev = self.args, self.torch, self.M, self.W, self.dev
        B, L, H = wl.batch, wl.n_layers, wl.hidden
        T = K + Wm
        t_setup = time.time()
        res = W.make_resident(wl)
        if pool is None:
            pool = W.alloc_pinned_pool(wl)
        W.fill_experts_gpu(wl, pool)
        x0_np, eps_np = W.make_inputs(wl, tokens=T)
        x0 = torch.from_numpy(x0_np).to(dev)
        eps = torch.from_numpy(eps_np).to(dev)
        log(f"[bench] {wl.name}: pool {wl.pool_bytes / 1e9:.1f} GB pinned ({wl.distinct_pool_layers} of {L} layers' expert blocks held), "
            f"setup {time.time() - t_setup:.1f} s")

        # the second DMA queue pays off from a few MB per expert on; below that their set-up latency dominates
        spec_auto = "dma2" if wl.expert_bytes >= (4 << 20) else "kernel"
        engine_names = {"speculative": spec_auto if args.copy_engine == "auto" else args.copy_engine,
                        "on_demand": "kernel" if args.copy_engine == "auto" else args.copy_engine}
        modes = ["speculative", "on_demand"]
        if headline and args.with_hint:
            engine_names["prefetch_hint"] = "kernel" if args.copy_engine == "auto" else args.copy_engine
            modes.append("prefetch_hint")
        if args.with_lookahead:
            engine_names["speculative_lookahead2"] = engine_names["speculative"]
            modes.append("speculative_lookahead2")

        def make(mode, profile, predict=0):
            return engine_for(wl, self.mode_codes[mode], res, pool, predict_in_on_demand=predict, profile=profile,
                              copy_engine=self.codes[engine_names[mode]], lookahead=2 if mode.endswith("lookahead2") else 0)

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

        fast_b1 = B == 1
        MFMA = ("expert_mfma_kernel<true", "expert_mfma_kernel<false")

        def token_loop_counts(n_tokens, fused_route=True):
            steps = n_tokens * L
            c = {"advance_kernel": n_tokens * (L - 1)}
            if fused_route:
                c["route_pair_kernel"] = steps
            if fast_b1:
                c.update({"gateup_b1": steps, "down_combine_b1": steps})
            return c
        uncounted = () if fast_b1 else MFMA

        def timed(eng, name):
            # one context alive at a time: every context owns streams, and idle ones would share the
            # process's few hardware queues with the one being timed
            eng.reset()
            self.leg(f"{wl.name}/{name}", token_loop_counts(T), uncounted)
            run_tokens(eng, 0, Wm)
            torch.cuda.synchronize()
            before = eng.stats()
            t0 = time.perf_counter()
            run_tokens(eng, Wm, K)
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            after = eng.stats()
            self.leg_waves(eng)
            return dt, {k: after[k] - before[k] for k in after}

        results = {m: [] for m in modes}
        for rep in range(reps):
            for mode in modes:
                eng = make(mode, 0)
                dt, d = timed(eng, f"{mode}/rep{rep}")
                eng.close()
                results[mode].append((dt, d))
                log(f"[bench] {wl.name} rep {rep} {mode}: TPOT {dt / K * 1e3:.3f} ms, H2D {d['h2d_bytes'] / dt / 1e9:.2f} GB/s "
                    f"({d['cache_misses']} misses, {d['cache_hits']} hits)")

        def summary(mode):
            tp = np.array([dt / K * 1e3 for dt, _ in results[mode]])
            dt, d = results[mode][-1]
            return {"recall_at_k_two_layers_ahead": d["hits2"] / d["predictions2"] if d["predictions2"] else None,
                    "tpot_ms": float(tp.mean()), "tpot_ms_std": float(tp.std()), "tokens_per_s": float(B / (tp.mean() / 1e3)),
                    "h2d_gb_per_token": d["h2d_bytes"] / K / 1e9, "h2d_gbs_wall": d["h2d_bytes"] / dt / 1e9,
                    "link_frac_wall_nominal": d["h2d_bytes"] / dt / 1e9 / LINK_PEAK_GBS,
                    "expert_transfers_per_token": d["cache_misses"] / K,
                    "cache_hit_rate": d["cache_hits"] / max(1, d["cache_hits"] + d["cache_misses"]),
                    "hbm_gb_algorithmic_per_token": d["hbm_bytes_algorithmic"] / K / 1e9}

        spec, ond = summary("speculative"), summary("on_demand")
        out = {"config": {"workload": wl.name, "layers": L, "hidden": H, "experts": wl.n_experts, "top_k": wl.top_k,
                          "inter": wl.inter, "batch": B, "slots_per_layer": wl.slots, "reps": reps, "steps": K, "warmup": Wm,
                          "copy_engine": engine_names, "expert_bytes": wl.expert_bytes,
                          "host_pool_gb": wl.pool_bytes / 1e9, "host_pool_layers": wl.distinct_pool_layers, "dtype": wl.dtype},
               "speculative": spec, "on_demand": ond,
               "prefetch_hint": summary("prefetch_hint") if "prefetch_hint" in modes else None,
               "speculative_lookahead2": summary("speculative_lookahead2") if "speculative_lookahead2" in modes else None,
               "tpot_reduction_vs_on_demand": 1.0 - spec["tpot_ms"] / ond["tpot_ms"]}

        # ---- instrumented legs (separate contexts with timing events): compute / copy / stall breakdown, hit
        #      statistics, and the duration of the expert launches of every cache wave inside the token loop
        breakdown = {}
        prof_eng = None
        for mode in ("speculative", "on_demand"):
            eng = make(mode, 1, predict=1)
            dt, d = timed(eng, f"{mode}/instrumented")
            busy, waves = d["copy_ms"], max(1, d["expert_launches"])
            breakdown[mode] = {
                "wall_ms_per_token": dt / K * 1e3, "copy_ms_per_token": d["copy_ms"] / K,
                "compute_ms_per_token": d["compute_ms"] / K, "stall_ms_per_token": d["stall_ms"] / K,
                "idle_ms_per_token": max(0.0, (dt * 1e3 - d["copy_ms"] - d["compute_ms"]) / K) if mode == "on_demand" else None,
                "h2d_gbs_while_copying": d["h2d_bytes"] / (busy / 1e3) / 1e9 if busy > 0 else None,
                "link_frac_while_copying_nominal": d["h2d_bytes"] / (busy / 1e3) / 1e9 / LINK_PEAK_GBS if busy > 0 else None,
                # copies and kernels never run side by side when every load blocks: the figure exists for prefetching only
                "overlap_fraction": ((d["copy_ms"] + d["compute_ms"] - dt * 1e3) / min(d["copy_ms"], d["compute_ms"]))
                if mode == "speculative" and min(d["copy_ms"], d["compute_ms"]) > 0 else None,
                "hit_rate_recall_at_k": d["hits"] / max(1, d["predictions"]),
                "expert_launches_us_per_cache_wave_event_pairs": d["expert_ms"] / waves * 1e3,
                "note": "event pairs around every cache wave's expert launches; each pair adds 2-8 us"}
            if mode == "on_demand":
                prof_eng = eng
            else:
                eng.close()
        out["breakdown_instrumented"] = breakdown

        # ---- the kernels of one layer step, each launched back to back between two HIP events on the compute
        #      stream, every launch on the slots / tables of the next layer in turn so that nothing is found in a cache
        mfma = wl.dtype == "bf16" and B >= 2
        which_list = ([K_MFMA_GU, K_MFMA_DOWN] if mfma else [K_GATEUP, K_READ_GU, K_DOWN, K_READ_DOWN]) + [K_ROUTE_TRUE, K_ROUTE_PAIR]
        kern = {}
        for which in which_list:
            name, sym = KERNEL_NAMES[which]
            self.leg(f"{wl.name}/isolated/{name}", {sym: args.kernel_reps + min(args.kernel_reps, 4)})
            ms, nbytes = prof_eng.time_kernel(which, args.kernel_reps)
            kern[name] = {"us_per_launch": ms * 1e3, "bytes_per_launch": nbytes, "gbs": nbytes / (ms / 1e3) / 1e9,
                          "frac_of_hbm_peak": nbytes / (ms / 1e3) / 1e9 / HBM_PEAK_GBS}
        prof_eng.close()
        traffic = (self.traffic.get("workloads") or {}).get(wl.name, {})
        for name, entry in kern.items():
            t = traffic.get(name)
            entry["hbm_traffic_bytes_pmc"] = t["bytes"] if t else None
        if not mfma:
            kern["expert_gateup_gemv"]["frac_of_pure_read"] = kern["pure_read_of_the_gateup_bytes"]["us_per_launch"] / kern["expert_gateup_gemv"]["us_per_launch"]
            kern["expert_down_combine_gemv"]["frac_of_pure_read"] = kern["pure_read_of_the_down_bytes"]["us_per_launch"] / kern["expert_down_combine_gemv"]["us_per_launch"]
        dom_name = "expert_gateup_mfma" if mfma else "expert_gateup_gemv"
        dom = kern[dom_name]
        experts_per_launch = dom["bytes_per_launch"] // (2 * wl.inter * H * wl.elem_bytes)
        step_names = ["route_true_and_prediction", dom_name, "expert_down_mfma" if mfma else "expert_down_combine_gemv"]
        step_us = sum(kern[n]["us_per_launch"] for n in step_names)
        step_bytes = sum(kern[n]["bytes_per_launch"] for n in step_names)
        roofline = {
            "bound": "hbm",
            "kernel": (f"expert_mfma_kernel<gate/up> (W_gate/W_up tiles + SwiGLU on the matrix cores, batch {B} over {experts_per_launch} resident experts)"
                       if mfma else "gateup_b1 kernels (expert W_gate/W_up GEMV + SwiGLU, batch 1)"),
            "achieved": dom["gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": dom["gbs"] / HBM_PEAK_GBS,
            "traffic": dom["hbm_traffic_bytes_pmc"], "traffic_source": os.path.relpath(TRAFFIC_FILE, ROOT) if dom["hbm_traffic_bytes_pmc"] else None,
            "launches_timed": args.kernel_reps, "bytes_per_launch": dom["bytes_per_launch"], "us_per_launch": dom["us_per_launch"],
            "how": "two HIP events on the compute stream around back-to-back launches, each launch on the slots of the next layer in turn",
            "kernels": kern,
            "layer_step": {"kernels": step_names, "algorithmic_bytes": step_bytes, "us_back_to_back": step_us,
                           "gbs": step_bytes / step_us / 1e3, "frac_of_hbm_peak": step_bytes / step_us / 1e3 / HBM_PEAK_GBS,
                           "routing_share_of_kernel_time": kern["route_true_and_prediction"]["us_per_launch"] / step_us,
                           "note": "one routing launch (true routing + prediction) and the expert launches of one cache wave"},
            "in_token_loop_event_pairs": {m: breakdown[m]["expert_launches_us_per_cache_wave_event_pairs"] for m in breakdown},
            "in_token_loop_rocprof": (self.trace.get("workloads") or {}).get(wl.name),
            "in_token_loop_rocprof_source": os.path.relpath(TRACE_FILE, ROOT) if (self.trace.get("workloads") or {}).get(wl.name) else None}
        out["roofline"] = roofline

        # ---- the paper's analytic model (Sec. 5.1): prefetching can hide min(copy, compute) per layer.  Compute per
        #      token: the kernels of one layer step timed back to back, times L (layers taken as alike); copy per token:
        #      the copy stream's busy time in the instrumented on-demand leg.  Against the measured difference of the two
        #      un-instrumented modes.
        od = breakdown["on_demand"]
        kernel_ms = L * step_us / 1e3 if B == 1 else None
        out["tpot_model_sec_5_1"] = {
            "copy_ms_per_token": od["copy_ms_per_token"], "compute_ms_per_token_kernels_back_to_back": kernel_ms,
            "compute_ms_per_token_event_spans": od["compute_ms_per_token"],
            "predicted_improvement_ms": min(od["copy_ms_per_token"], kernel_ms) if kernel_ms else None,
            "predicted_improvement_ms_from_event_spans": min(od["copy_ms_per_token"], od["compute_ms_per_token"]),
            "measured_improvement_ms": ond["tpot_ms"] - spec["tpot_ms"],
            "predicted_reduction": min(od["copy_ms_per_token"], kernel_ms) / ond["tpot_ms"] if kernel_ms else None,
            "measured_reduction": 1.0 - spec["tpot_ms"] / ond["tpot_ms"]}
        out["link"] = {"peak_nominal_gbs": LINK_PEAK_GBS, "achieved_gbs_speculative_wall": spec["h2d_gbs_wall"],
                       "achieved_gbs_on_demand_wall": ond["h2d_gbs_wall"]}

        if args.per_layer_misses:
            out["cache_misses_per_layer"] = self.per_layer_misses(wl, make, x0, eps, min(T, 32))

        if headline and args.diagnostics:
            diagnostics = {}
            for signal, name in ((0, "quasi_hidden_state"), (1, "baseline_s_l")):
                eng = engine_for(wl, M.MODE_ON_DEMAND, res, pool, predict_in_on_demand=1, copy_engine=self.codes[engine_names["on_demand"]],
                                 predict_signal=signal, diagnostics=1)
                self.leg(f"{wl.name}/diagnostics/{name}", token_loop_counts(min(T, 16), fused_route=False), uncounted)
                run_tokens(eng, 0, min(T, 16))
                per = [eng.layer_diagnostics(l) for l in range(L)]
                self.leg_waves(eng)
                eng.close()
                diagnostics[name] = {
                    "tokens": min(T, 16), "execution": "true experts (on-demand), so both signals see the same trajectory",
                    "recall_at_k_per_layer": [round(d["hits"] / d["predictions"], 4) if d["predictions"] else None for d in per],
                    "cosine_to_next_router_input_per_layer": [round(d["cos_sum"] / d["cos_count"], 4) if d["cos_count"] else None for d in per],
                    "top_rank_agreement_per_layer": [round(d["rank_match"][0] / d["cos_count"], 4) if d["cos_count"] else None for d in per]}
            out["signal_diagnostics"] = diagnostics

        # ---- prefill (Sec. 5.2, prefill phase): all prompt tokens per layer, every expert streamed layer-ahead
        if headline and args.prefill > 0:
            import dataclasses
            P = args.prefill
            px0, peps = W.make_inputs(dataclasses.replace(wl, batch=P), tokens=1)
            pr0 = torch.from_numpy(px0[0]).to(dev)
            pe = torch.from_numpy(peps[0]).to(dev)
            name = spec_auto if args.copy_engine == "auto" else args.copy_engine
            eng = engine_for(wl, M.MODE_SPECULATIVE, res, pool, copy_engine=self.codes[name], max_batch=min(64, P),
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
            group = min(max(wl.slots // 2, 1), wl.n_experts)          # experts per launch pair of the prefill step
            n_pairs = 3 * L * ((wl.n_experts + group - 1) // group)
            micro = min(64, P)                                        # tokens per routing launch
            self.leg(f"{wl.name}/prefill", dict({"advance_kernel": 3 * (L - 1),
                                                 "route_pair_kernel": 3 * L * ((P + micro - 1) // micro)},
                                                **({m: n_pairs for m in MFMA} if wl.dtype == "bf16" else {})))
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
            out["prefill"] = {"prompt_tokens": P, "micro_batch": min(64, P), "copy_engine": name, "ms_per_prompt": dt * 1e3,
                              "ms_per_layer": dt * 1e3 / L, "prompt_tokens_per_s": P / dt, "h2d_gb_per_prompt": nbytes / 1e9,
                              "h2d_gbs_wall": nbytes / dt / 1e9, "link_frac_wall_nominal": nbytes / dt / 1e9 / LINK_PEAK_GBS}
            log(f"[bench] prefill P={P}: {dt * 1e3:.1f} ms per prompt, {dt * 1e3 / L:.2f} ms per layer, H2D {nbytes / dt / 1e9:.2f} GB/s")

        # ---- the CPU checker timed on this host, on a bounded prefix of the same workload
        if headline and args.cpu_tokens > 0:
            out["cpu_baseline"] = self.cpu_baseline(wl, res, pool, x0_np, eps_np, min(args.cpu_tokens, T))
        return out, pool

    def per_layer_misses(self, wl, make, x0, eps, n_tokens):
        """Expert transfers per layer, per mode: the per-layer difference of the transfer counter over n_tokens."""
        torch = self.torch
        B, L, H = wl.batch, wl.n_layers, wl.hidden
        res = {}
        for mode in ("speculative", "on_demand"):
            eng = make(mode, 0)
            self.leg(f"{wl.name}/{mode}/per_layer_misses",
                     dict({"route_pair_kernel": n_tokens * L, "advance_kernel": n_tokens * (L - 1)},
                          **({"gateup_b1": n_tokens * L, "down_combine_b1": n_tokens * L} if B == 1 else {})),
                     () if B == 1 else ("expert_mfma_kernel<true", "expert_mfma_kernel<false"))
            out = torch.empty((B, H), dtype=torch.float32, device=self.dev)
            rbuf = [torch.empty((B, H), dtype=torch.float32, device=self.dev) for _ in range(2)]
            per_layer = [0] * L           # transfers issued during the call for layer l (speculative: the prefetch for l+1)
            prev = 0
            with torch.cuda.stream(eng.compute):
                for t in range(n_tokens):
                    eng.begin_token()
                    r = x0[t]
                    for l in range(L):
                        eng.layer_step(l, r, out, sync_input=False)
                        now = eng.stats()["cache_misses"]
                        per_layer[l] += now - prev
                        prev = now
                        if l + 1 < L:
                            r = eng.advance(r, out, eps[t, l], wl.res_a, wl.res_b, rbuf[l & 1])
            st = eng.stats()
            self.leg_waves(eng)
            eng.close()
            res[mode] = {"tokens": n_tokens, "transfers_issued_during_layer_call": per_layer,
                         "transfers_per_token": st["cache_misses"] / n_tokens,
                         "cache_hit_rate": st["cache_hits"] / max(1, st["cache_hits"] + st["cache_misses"]),
                         "recall_at_k": st["hits"] / max(1, st["predictions"])}
        return res

    def cpu_baseline(self, wl, res, pool, x0_np, eps_np, n_tok):
        from oracle import moe_oracle as O
        W = self.W
        L, B = wl.n_layers, wl.batch
        pool_np = W.PoolView(pool)
        model = O.OracleModel(n_layers=L, hidden=wl.hidden, n_experts=wl.n_experts, top_k=wl.top_k, inter=wl.inter,
                              dtype=O.DTYPE_BF16 if wl.dtype == "bf16" else O.DTYPE_F32, router_w=res["router_w"],
                              rms_gain=res["rms_gain"], dvecs=res["dvecs"], experts=pool_np)

        def run(n):
            orc = O.MoEOracle(model, O.MODE_SPECULATIVE, wl.slots)
            t0 = time.perf_counter()
            O.run_tokens(orc, x0_np[:n], lambda t, l, r, o: W.advance_residual(wl, r, o, eps_np[t, l]))
            return time.perf_counter() - t0
        try:
            from threadpoolctl import threadpool_info, threadpool_limits
            threads = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
        except Exception:
            threadpool_limits, threads = None, os.cpu_count()
        dt_all = run(n_tok)
        single = None
        if threadpool_limits is not None:
            with threadpool_limits(limits=1):
                dt_one = run(1)
            single = {"value": B / dt_one, "unit": "tokens/s", "cores": 1, "sample": f"first decode token, {dt_one:.1f} s"}
        return {"value": B * n_tok / dt_all, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
                "cpu_model": cpu_model(), "host_logical_cpus": os.cpu_count(), "single_thread": single,
                "sample": f"first {n_tok} decode tokens of the same workload (all {L} layers, speculative mode), "
                          f"{dt_all:.1f} s of numpy float64 on the host with {threads} BLAS threads; one more pass over "
                          f"the first token with the BLAS limited to one thread"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    b = Bench(args)
    W = b.W
    wl = W.CONFIGS[args.workload]
    if not wl.pinnable:
        print(f"bench.py: the pinned pool of {wl.name} ({wl.pool_bytes / 1e9:.0f} GB) exceeds what this box can "
              f"page-lock (about 72 GB); give the workload fewer pool_layers (layers then share expert blocks).", file=sys.stderr)
        sys.exit(2)
    reduced = bool(args.layers) and args.layers != wl.n_layers
    if args.layers:
        wl = wl.with_(n_layers=args.layers)
    K, Wm = args.steps, args.warmup

    head, pool = b.run(wl, K, Wm, args.reps, headline=True)
    if reduced:
        head["config"]["workload"] += " (REDUCED LAYERS, development run)"

    extra = args.extra
    if extra == "auto":
        extra = ("c5_qwen3_b32,c1_tiny,c3_gpt_oss_20b,c3_gpt_oss_20b_b8,c4_mixtral_8x7b"
                 if args.workload == "c2_qwen3_30b_a3b" and not reduced else "none")
    legs = {}

    def pool_shape(w):
        return (w.n_layers, w.n_experts, w.expert_elems, w.dtype)
    held = wl                                     # the workload whose pinned pool is held at the moment
    for name in [n for n in extra.split(",") if n and n != "none"]:
        try:                                      # a further workload that fails must not cost the headline result
            xw = W.CONFIGS[name]
            xk = max(4, K // 2) if xw.batch > 1 else max(K, 32)
            small = xw.pool_bytes < (1 << 30)
            xreps = 1 if xw.expert_bytes > (100 << 20) else min(args.reps, 2)  # a quarter of a second per token: once
            if pool is not None and pool_shape(xw) == pool_shape(held):
                res, pool = b.run(xw, xk, min(Wm, 2), xreps, pool=pool)
            elif small:                           # a pool this small is pinned beside the one that is held
                res, xpool = b.run(xw, xk, min(Wm, 2), xreps)
                W.free_pinned_pool(xpool)
            else:                                 # the box cannot page-lock two large pools at once
                if pool is not None:
                    W.free_pinned_pool(pool)
                pool, held = None, None
                res, pool = b.run(xw, xk, min(Wm, 2), xreps)
                held = xw
        except Exception as exc:                  # noqa: BLE001 - reported in the line, the run goes on
            log(f"[bench] {name} failed: {type(exc).__name__}: {exc}")
            res = {"error": f"{type(exc).__name__}: {exc}"}
            try:                                  # whatever the failed run still holds page-locked
                b.torch.cuda.synchronize()
                W.free_all_pinned()
            except Exception:                     # noqa: BLE001
                pass
            pool, held = None, None
        legs[name] = res

    if args.calibrate_copy:
        import torch
        a = torch.empty(256 << 20, dtype=torch.uint8, device=b.dev)
        c = torch.empty_like(a)
        b.leg("calibration_copy", {})
        c.copy_(a)
        torch.cuda.synchronize()
        log("[bench] calibration copy: 268435456 bytes read + 268435456 bytes written in one dispatch")
    if pool is not None:
        W.free_pinned_pool(pool)       # tens of GB of page-locked memory: unpin now, not while the process exits
    if args.legs_file:
        with open(args.legs_file, "w") as f:
            json.dump({"legs": b.legs, "argv": sys.argv[1:]}, f)

    spec = head["speculative"]
    line = {
        "metric": "decode tokens/s with speculative expert prefetch (TPOT in ms_per_step); on-demand loading beside it",
        "value": spec["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": spec["tpot_ms"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic"}
    line.update(head)
    for key in ("cpu_baseline", "prefill", "signal_diagnostics"):
        line.setdefault(key, None)
    line["other_workloads"] = legs
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
