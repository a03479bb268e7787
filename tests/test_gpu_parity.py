"""GPU parity: the HIP path, called through the C ABI, against the CPU checker on the same
seeded inputs.  Expert ids, hit counts and cache traffic must be equal; layer outputs within
1e-5 (float32 weights) or 2e-2 (bf16 weights) relative L2 error per token row."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2603_19289_amd import workload as W
from tests.helpers import build, check_output, make_advance, small_workload

pytestmark = pytest.mark.gpu

MODES = {"on_demand": O.MODE_ON_DEMAND, "speculative": O.MODE_SPECULATIVE, "prefetch_hint": O.MODE_PREFETCH_HINT}


def run_teacher_forced(wl, mode, gains="random", q_from_normalized=0, label="", prebuilt=None, oracle_kw=None,
                       **engine_kw):
    """The checker runs free; the GPU step is fed the checker's r_l at every layer.
    prebuilt = (resident tables, checker model, pinned torch pool) for pools drawn on the GPU."""
    from paper_2603_19289_amd.engine import engine_for
    print(f"[case] {label or wl.name} mode={mode} L={wl.n_layers} H={wl.hidden} E={wl.n_experts} k={wl.top_k} "
          f"I={wl.inter} B={wl.batch} S={wl.slots} {wl.dtype}", flush=True)
    if prebuilt is None:
        res, ex, model = build(wl, gains)
    else:
        res, model, ex = prebuilt
    x0, eps = W.make_inputs(wl)
    orc = O.MoEOracle(model, mode, wl.slots, q_from_normalized=bool(q_from_normalized), **(oracle_kw or {}))
    trace = O.run_tokens(orc, x0, make_advance(wl, eps))
    eng = engine_for(wl, mode, res, ex, q_from_normalized=q_from_normalized, **engine_kw)
    worst = worst_elem = 0.0
    try:
        for t in range(wl.tokens):
            eng.begin_token()
            for l in range(wl.n_layers):
                r_np, want = trace[t][l]
                r = torch.from_numpy(r_np.astype(np.float32)).to("cuda")
                out, ids = eng.layer_step(l, r, want_ids=True)
                torch.cuda.synchronize()
                where = f"token {t} layer {l}"
                np.testing.assert_array_equal(ids["true_ids"].cpu().numpy(), want.true_ids, err_msg=where)
                np.testing.assert_allclose(ids["true_gates"].cpu().numpy(), want.true_gates, atol=2e-7, rtol=1e-6, err_msg=where)
                np.testing.assert_array_equal(ids["exec_ids"].cpu().numpy(), want.exec_ids, err_msg=where)
                np.testing.assert_allclose(ids["exec_gates"].cpu().numpy(), want.exec_gates, atol=2e-7, rtol=1e-6, err_msg=where)
                if want.next_ids is not None:
                    np.testing.assert_array_equal(ids["next_ids"].cpu().numpy(), want.next_ids, err_msg=where)
                    np.testing.assert_allclose(ids["next_gates"].cpu().numpy(), want.next_gates, atol=2e-7, rtol=1e-6, err_msg=where)
                else:
                    assert (ids["next_ids"].cpu().numpy() == -1).all(), where
                l2, elem = check_output(out.cpu().numpy(), want.out, wl.dtype, where, terms=wl.top_k * wl.inter)
                worst, worst_elem = max(worst, l2), max(worst_elem, elem)
        st = eng.stats()
        for name in ("tokens", "layer_steps", "predictions", "hits", "cache_hits", "cache_misses", "h2d_bytes",
                     "predictions2", "hits2", "cache_waves"):
            assert st[name] == getattr(orc.stats, name), (name, st[name], getattr(orc.stats, name))
    finally:
        eng.close()
    print(f"[ok] worst relative L2 error {worst:.3e}, worst element error {worst_elem:.3e} of the row RMS; hits {orc.stats.hits}/{orc.stats.predictions}; "
          f"cache {orc.stats.cache_hits} hits {orc.stats.cache_misses} misses", flush=True)
    return worst


@pytest.mark.parametrize("mode", list(MODES))
def test_c1_tiny_fp32(mode):
    wl = W.CONFIGS["c1_tiny"]
    run_teacher_forced(wl, MODES[mode], gains="ones")


@pytest.mark.parametrize("mode", list(MODES))
def test_c1_tiny_fp32_per_layer_default_vector(mode):
    # the literal reading of the workload text: one default vector per layer, shared by all experts
    run_teacher_forced(W.CONFIGS["c1_tiny"].with_(per_layer_dvec=True, tokens=8), MODES[mode], gains="ones")


@pytest.mark.parametrize("mode", list(MODES))
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ragged_shapes_single_token(mode, dtype):
    # H, I not multiples of the 512/256-element wave strides, E not a multiple of rows per block
    wl = small_workload(name="ragged", n_layers=4, hidden=328, n_experts=21, top_k=3, inter=136,
                        dtype=dtype, batch=1, tokens=6, slots=5, seed=11)
    run_teacher_forced(wl, MODES[mode])


@pytest.mark.parametrize("mode", list(MODES))
@pytest.mark.parametrize("B,S", [(3, 6), (5, 4), (8, 3)])
def test_batches_and_cache_waves(mode, B, S):
    # S smaller than the union of routed experts forces several cache waves per layer
    wl = small_workload(name="waves", n_layers=3, hidden=264, n_experts=12, top_k=3, inter=200,
                        dtype="bf16", batch=B, tokens=4, slots=S, seed=5)
    run_teacher_forced(wl, MODES[mode])


@pytest.mark.parametrize("mode", list(MODES))
@pytest.mark.parametrize("B,S", [(16, 12), (23, 5), (40, 4), (64, 7)])
def test_matrix_core_path_batches_of_16_and_more(mode, B, S):
    # bf16 and B >= 16 runs the MFMA expert kernels: ragged K tail (264 = 4*64 + 8), ragged row
    # tiles (200 = 12*16 + 8), more than 16 tokens per expert, several cache waves
    wl = small_workload(name="mfma", n_layers=3, hidden=264, n_experts=12, top_k=3, inter=200,
                        dtype="bf16", batch=B, tokens=2, slots=S, seed=13)
    run_teacher_forced(wl, MODES[mode])


@pytest.mark.parametrize("mode", list(MODES))
def test_edge_shapes(mode):
    # every expert selected; pool exactly k; one expert; one layer (no prediction at all)
    run_teacher_forced(small_workload(name="all_experts", n_experts=4, top_k=4, slots=4, tokens=3, dtype="f32"), MODES[mode])
    run_teacher_forced(small_workload(name="one_expert", n_experts=1, top_k=1, slots=1, tokens=3), MODES[mode])
    run_teacher_forced(small_workload(name="one_layer", n_layers=1, tokens=3), MODES[mode])
    run_teacher_forced(small_workload(name="wide_router", n_experts=200, top_k=16, slots=16, tokens=2, hidden=128), MODES[mode])
    run_teacher_forced(small_workload(name="max_inter", n_layers=2, hidden=64, inter=32768, n_experts=2, top_k=1, slots=1,
                                      batch=2, tokens=1), MODES[mode])       # 128 KB of LDS in the down kernel
    run_teacher_forced(small_workload(name="max_batch", batch=64, n_experts=16, top_k=2, slots=8, tokens=2, dtype="f32"), MODES[mode])
    # a batch large enough for sixteen router rows per workgroup, with a ragged last workgroup (50 = 3 * 16 + 2)
    run_teacher_forced(small_workload(name="many_rows_per_workgroup", batch=48, n_experts=50, top_k=5, slots=50, tokens=2,
                                      hidden=136, inter=40), MODES[mode])


@pytest.mark.parametrize("dtype,H", [("bf16", 4608), ("f32", 4352), ("bf16", 8192), ("f32", 8192)])
def test_wide_hidden_sizes_take_the_streaming_fallbacks(dtype, H):
    # beyond 64*8 register chunks per lane the routing kernel streams its row in a loop; float32 rows
    # beyond 4096 columns leave the register-resident batch-1 expert kernel for the LDS-staged one;
    # 8192 is the largest hidden size the library accepts (64 KB of float64 LDS per token)
    wl = small_workload(name="wide", n_layers=3, hidden=H, n_experts=6, top_k=2, inter=72, dtype=dtype,
                        batch=1, tokens=2, slots=3, seed=71)
    run_teacher_forced(wl, O.MODE_SPECULATIVE)


@pytest.mark.parametrize("dtype,H,I,k,what", [
    ("bf16", 256, 768, 4, "down: 384 chunks per row, one wavefront, six loads per lane"),
    ("bf16", 256, 1024, 4, "down: 512 chunks, two wavefronts of four loads"),
    ("bf16", 256, 776, 4, "down: a chunk count that is no multiple of 64, four wavefronts with a ragged end"),
    ("f32", 128, 520, 3, "down: float32 rows with a ragged end; gate/up: pair kernel with few rows"),
    ("bf16", 512, 2048, 4, "gate/up: 8192 rows, the largest launch of the two-rows-per-wavefront kernel"),
    ("bf16", 512, 2056, 4, "gate/up: 8224 rows, the smallest launch of the pipelined kernel"),
    ("bf16", 2560, 72, 2, "gate/up: five register chunks per lane, pipelined kernel whatever the row count"),
])
def test_batch_one_kernel_variants(dtype, H, I, k, what):
    # the launchers of the batch-1 expert kernels pick a kernel and its shape from I, k and H
    wl = small_workload(name="b1_variant", n_layers=2, hidden=H, n_experts=6, top_k=k, inter=I, dtype=dtype,
                        batch=1, tokens=2, slots=k + 1, seed=83)
    run_teacher_forced(wl, O.MODE_SPECULATIVE, label=what)
    run_teacher_forced(wl, O.MODE_ON_DEMAND, label=what)


@pytest.mark.parametrize("mode", list(MODES))
def test_caption_reading_of_the_quasi_hidden_state(mode):
    run_teacher_forced(small_workload(name="caption", n_layers=4, tokens=4), MODES[mode], q_from_normalized=1)


@pytest.mark.parametrize("engine", ["COPY_DMA", "COPY_KERNEL", "COPY_DMA2"])
def test_prefetch_hint_refetch_into_a_slot_the_prefetch_just_filled(engine):
    # S = k: the true request of a layer reuses slots that the (mispredicted) prefetch for the same
    # layer filled one step earlier, before any kernel read them; with several DMA queues the second
    # copy must still land after the first
    from paper_2603_19289_amd import moe_spec as M
    wl = small_workload(name="hint_reuse", n_layers=4, hidden=264, n_experts=12, top_k=3, inter=200,
                        dtype="bf16", batch=1, tokens=6, slots=3, seed=17)
    run_teacher_forced(wl, O.MODE_PREFETCH_HINT, copy_engine=getattr(M, engine))


@pytest.mark.parametrize("layers", [None, [1, 3]], ids=["est_pf", "hybrid_pf"])
@pytest.mark.parametrize("dtype,B", [("bf16", 1), ("f32", 1), ("bf16", 5)])
def test_estimator_predictions(layers, dtype, B):
    # the estimator's forward pass (random weights in the paper's shapes) replaces the router-based
    # prediction at all layers (Est-PF) or at some (Hybrid-PF); the speculated experts are executed
    wl = small_workload(name="estimator", n_layers=5, hidden=264, n_experts=12, top_k=3, inter=200,
                        dtype=dtype, batch=B, tokens=4, slots=6, seed=51)
    est = W.make_estimator(wl, m=3, n=2)            # latent 88, feed-forward 176
    use = list(range(wl.n_layers)) if layers is None else layers
    run_teacher_forced(wl, O.MODE_SPECULATIVE, oracle_kw=dict(estimator=O.Estimator(**est), estimator_layers=use),
                       estimator=est, estimator_layers=use)


@pytest.mark.parametrize("mode", ["speculative", "prefetch_hint"])
@pytest.mark.parametrize("dtype,B,S,engine", [("bf16", 1, 4, "COPY_DMA2"), ("f32", 3, 5, "COPY_KERNEL"), ("bf16", 20, 6, "COPY_DMA"),
                                             ("bf16", 1, 3, "COPY_DMA2")])
def test_two_layer_lookahead(mode, dtype, B, S, engine):
    # layer l also requests what layer l+2's router selects on LN_{l+2}(r_l + d_l) into pool l+2 (a cache hint one
    # layer before the regular prefetch): executed ids and outputs as without it, cache traffic and the second
    # recall counter equal to the checker's; S = k makes the regular prefetch overwrite slots the hint just filled
    from paper_2603_19289_amd import moe_spec as M
    wl = small_workload(name="lookahead", n_layers=6, hidden=264, n_experts=12, top_k=3, inter=200, dtype=dtype,
                        batch=B, tokens=5, slots=S, seed=19)
    run_teacher_forced(wl, MODES[mode], oracle_kw=dict(lookahead=2), lookahead=2, copy_engine=getattr(M, engine))


def test_crafted_ties_pick_the_lower_index():
    # identical router rows give exactly equal logits: the lower expert index must win on the GPU too
    from paper_2603_19289_amd.engine import engine_for
    wl = small_workload(name="ties", n_layers=2, n_experts=8, top_k=3, tokens=2, dtype="f32")
    res, ex, model = build(wl)
    res["router_w"][:, 5] = res["router_w"][:, 2]
    res["router_w"][:, 7] = res["router_w"][:, 2]
    x0, eps = W.make_inputs(wl)
    orc = O.MoEOracle(model, O.MODE_ON_DEMAND, wl.slots)
    trace = O.run_tokens(orc, x0, make_advance(wl, eps))
    eng = engine_for(wl, O.MODE_ON_DEMAND, res, ex)
    try:
        for t in range(wl.tokens):
            eng.begin_token()
            for l in range(wl.n_layers):
                r = torch.from_numpy(trace[t][l][0].astype(np.float32)).cuda()
                _, ids = eng.layer_step(l, r, want_ids=True)
                torch.cuda.synchronize()
                np.testing.assert_array_equal(ids["true_ids"].cpu().numpy(), trace[t][l][1].true_ids)
    finally:
        eng.close()


@pytest.mark.parametrize("seed", [11, 12])
def test_randomised_configurations(seed):
    """Sixty seeded draws per seed of everything a configuration can vary within the documented limits (sizes that
    are no multiple of a tile, one expert, k = E, S = k, batches up to 64, every mode, copy engine and reading of
    q_l, the two-layer lookahead), each teacher-forced against the checker for a few tokens."""
    from paper_2603_19289_amd import moe_spec as M   # noqa: F401
    rng = np.random.default_rng(seed)
    hiddens = [8, 16, 24, 40, 64, 72, 136, 256, 520, 1000, 1024, 2056]
    inters = [8, 16, 40, 48, 104, 256, 520]
    batches = [1, 1, 1, 2, 3, 5, 8, 17, 33, 64]
    for case in range(60):
        H, I = int(rng.choice(hiddens)), int(rng.choice(inters))
        E = int(rng.integers(1, 65)) if rng.random() < 0.85 else int(rng.integers(65, 257))
        k = int(rng.integers(1, min(E, 16) + 1))
        S = int(rng.integers(k, E + 3))
        B = int(rng.choice(batches))
        dtype = "bf16" if rng.random() < 0.7 else "f32"
        mode = list(MODES)[int(rng.integers(0, 3))]
        L, T = int(rng.integers(1, 5)), int(rng.integers(1, 4))
        while L * E * 3 * H * I > 1.2e8:             # the pool is drawn on the CPU
            if I > 48:
                I = 48
            elif H > 136:
                H = 136
            else:
                E = max(k, E // 2)
                S = max(k, min(S, E + 2))
        while B * k * L * T * 3 * H * I > 6e8 and B > 1:   # the checker's work
            B = max(1, B // 2)
        look = mode != "on_demand" and L >= 3 and rng.random() < 0.3
        wl = small_workload(name=f"draw{seed}_{case}", n_layers=L, hidden=H, n_experts=E, top_k=k, inter=I, dtype=dtype,
                            batch=B, tokens=T, slots=S, seed=1000 * seed + case)
        kw = dict(copy_engine=int(rng.integers(0, 3)))
        if look:
            kw["lookahead"] = 2
        run_teacher_forced(wl, MODES[mode], q_from_normalized=int(rng.random() < 0.2),
                           oracle_kw=dict(lookahead=2) if look else None, **kw)


def test_randomised_configurations_of_the_one_routing_kernel_paths():
    """Sixty seeded draws through the paths that keep one kernel per routing: estimator at a random subset of layers
    (Est-PF / Hybrid-PF), the baseline signal, per-layer diagnostics; sizes, batches, modes and copy engines vary."""
    rng = np.random.default_rng(31)
    for case in range(60):
        m, n = int(rng.choice([1, 2, 3, 4])), int(rng.choice([1, 2, 3]))
        H = int(rng.choice([8, 16, 24, 40, 88, 128, 264])) * m          # latent size H/m, a multiple of 8
        I = int(rng.choice([8, 16, 40, 48, 104]))
        E = int(rng.integers(1, 65)) if rng.random() < 0.85 else int(rng.integers(65, 257))
        k = int(rng.integers(1, min(E, 16) + 1))
        S = int(rng.integers(k, E + 3))
        B = int(rng.choice([1, 1, 2, 3, 5, 8, 17, 33, 64]))
        dtype = "bf16" if rng.random() < 0.7 else "f32"
        mode = list(MODES)[int(rng.integers(0, 3))]
        L, T = int(rng.integers(2, 6)), int(rng.integers(1, 4))
        while L * E * 3 * H * I > 1.0e8:             # the pool is drawn on the CPU
            if I > 16:
                I = 16
            else:
                E = max(k, E // 2)
                S = max(k, min(S, E + 2))
        while B * k * L * T * 3 * H * I > 6e8 and B > 1:   # the checker's work
            B = max(1, B // 2)
        wl = small_workload(name=f"odraw{case}", n_layers=L, hidden=H, n_experts=E, top_k=k, inter=I, dtype=dtype,
                            batch=B, tokens=T, slots=S, seed=9000 + case)
        kind = int(rng.integers(0, 3))
        kw, okw = dict(copy_engine=int(rng.integers(0, 3))), {}
        if kind == 0:
            est = W.make_estimator(wl, m=m, n=n)
            use = [l for l in range(L) if rng.random() < 0.6] or [0]
            kw.update(estimator=est, estimator_layers=use)
            okw.update(estimator=O.Estimator(**est), estimator_layers=use)
        elif kind == 1:
            kw.update(predict_signal=1)
            okw.update(predict_signal=1)
        else:
            kw.update(diagnostics=1)
        run_teacher_forced(wl, MODES[mode], oracle_kw=okw, **kw)


def test_randomised_long_streams_on_tiny_layers():
    """Fifty seeded draws of tiny layers run for 10 to 40 tokens: cache churn, slot reuse, unions larger than the pool,
    every mode and copy engine, the lookahead; counters and ids equal to the checker's at every step."""
    rng = np.random.default_rng(41)
    for case in range(50):
        H, I = int(rng.choice([8, 16, 40, 64])), int(rng.choice([8, 16, 24]))
        E = int(rng.integers(2, 40))
        k = int(rng.integers(1, min(E, 8) + 1))
        S = int(rng.integers(k, min(E, k + 6) + 1))
        B = int(rng.choice([1, 1, 2, 4, 7, 16]))
        dtype = "bf16" if rng.random() < 0.6 else "f32"
        mode = list(MODES)[int(rng.integers(0, 3))]
        L, T = int(rng.integers(2, 8)), int(rng.integers(10, 41))
        look = mode != "on_demand" and L >= 3 and rng.random() < 0.4
        wl = small_workload(name=f"ldraw{case}", n_layers=L, hidden=H, n_experts=E, top_k=k, inter=I, dtype=dtype,
                            batch=B, tokens=T, slots=S, seed=7000 + case)
        kw = dict(copy_engine=int(rng.integers(0, 3)))
        if look:
            kw["lookahead"] = 2
        run_teacher_forced(wl, MODES[mode], oracle_kw=dict(lookahead=2) if look else None, **kw)
