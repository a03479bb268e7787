"""GPU parity at the full layer shapes of the benchmark workloads (hidden size, experts, top-k,
intermediate size, batch, slots per layer: the launch configuration bench.py times), on a few
layers and tokens so that the CPU checker finishes in seconds.  The expert pool is drawn on the
GPU and copied to pinned memory; the checker reads those same bytes."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2603_19289_amd import workload as W
from tests.helpers import oracle_model
from tests.test_gpu_parity import MODES, run_teacher_forced

pytestmark = pytest.mark.gpu


def prebuilt(wl):
    res = W.make_resident(wl)
    tdtype = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    pool = torch.empty((wl.n_layers, wl.n_experts, wl.expert_elems), dtype=tdtype, pin_memory=True)
    W.fill_experts_gpu(wl, pool)
    pool_np = pool.view(torch.int16).numpy().view(np.uint16) if wl.dtype == "bf16" else pool.numpy()
    return res, oracle_model(wl, res, pool_np), pool


def first_layers(pre, wl):
    """The same tables and pool cut down to the first wl.n_layers layers (a model of its own for the checker)."""
    res, model, pool = pre
    res = {k: v[:wl.n_layers] for k, v in res.items()}
    return res, oracle_model(wl, res, model.experts[:wl.n_layers]), pool[:wl.n_layers]


# layers x tokens per case; the checker decodes every executed expert block to float64, so its time
# goes with layers * tokens * batch * k * expert bytes (c5: 256 blocks of 9.4 MB per layer step)
CASES = {
    "c2_qwen3_30b_a3b": dict(n_layers=6, tokens=5),
    "c3_gpt_oss_20b": dict(n_layers=4, tokens=3),
    "c3_gpt_oss_20b_b8": dict(n_layers=2, tokens=2),
    "c4_mixtral_8x7b": dict(n_layers=2, tokens=3),
    "c5_qwen3_b32": dict(n_layers=6, tokens=4),
}
# the other two modes of the large-batch case run fewer tokens (the checker needs about 2 s per layer step there)
OTHER_MODES = {"c5_qwen3_b32": dict(n_layers=3, tokens=1)}


@pytest.mark.parametrize("name", list(CASES))
def test_full_layer_shape_all_modes(name):
    wl = W.CONFIGS[name].with_(**CASES[name])
    pre = prebuilt(wl)
    for mode in MODES:
        if mode != "speculative" and name in OTHER_MODES:
            small = wl.with_(**OTHER_MODES[name])
            run_teacher_forced(small, MODES[mode], prebuilt=first_layers(pre, small))
        else:
            run_teacher_forced(wl, MODES[mode], prebuilt=pre)


@pytest.mark.parametrize("engine", ["COPY_DMA", "COPY_DMA2"])
def test_full_layer_shape_with_dma_copy_engines(engine):
    from paper_2603_19289_amd import moe_spec as M
    wl = W.CONFIGS["c2_qwen3_30b_a3b"].with_(n_layers=2, tokens=2)
    run_teacher_forced(wl, O.MODE_SPECULATIVE, prebuilt=prebuilt(wl), copy_engine=getattr(M, engine))


@pytest.mark.parametrize("name,tokens", [("c2_qwen3_30b_a3b", 80), ("c5_qwen3_b32", 24)])
def test_free_running_decode_is_bitwise_repeatable_at_full_shape(name, tokens):
    """Two free runs of the same tokens through one context (reset in between) at the benchmark's layer
    shape: every routing decision and every output bit must repeat.  The hand-over of logits between
    workgroups, the slot cache and the copy/compute ordering are all deterministic by design; a stale read
    or a missed wait would show up here as a difference."""
    from paper_2603_19289_amd import moe_spec as M
    from paper_2603_19289_amd.engine import engine_for
    wl = W.CONFIGS[name].with_(n_layers=4, tokens=tokens)
    res, _, pool = prebuilt(wl)
    x0, eps = W.make_inputs(wl)
    x0 = torch.from_numpy(x0).cuda()
    eps = torch.from_numpy(eps).cuda()
    eng = engine_for(wl, M.MODE_SPECULATIVE, res, pool, copy_engine=M.COPY_DMA2)

    def run():
        ids_log, out_log = [], []
        for t in range(tokens):
            eng.begin_token()
            r = x0[t]
            for l in range(wl.n_layers):
                out, ids = eng.layer_step(l, r, want_ids=True)
                ids_log.append(torch.stack([ids["true_ids"], ids["exec_ids"], ids["next_ids"]]))
                out_log.append(out)
                if l + 1 < wl.n_layers:
                    r = eng.advance(r, out, eps[t, l], wl.res_a, wl.res_b)
        torch.cuda.synchronize()
        return torch.stack(ids_log).cpu(), torch.stack(out_log).cpu(), eng.stats()

    try:
        ids_a, out_a, st_a = run()
        eng.reset()
        ids_b, out_b, st_b = run()
    finally:
        eng.close()
    assert torch.equal(ids_a, ids_b)
    assert torch.equal(out_a.view(torch.int32), out_b.view(torch.int32))
    for key in ("hits", "predictions", "cache_hits", "cache_misses", "h2d_bytes"):
        assert st_a[key] == st_b[key], key


@pytest.mark.parametrize("mode", ["speculative", "on_demand"])
def test_free_running_bf16_at_the_c2_layer_shape_with_margin_audit(mode):
    """The GPU runs free at the benchmark's layer shape: its own float32 outputs feed the residual driver,
    layer after layer.  The checker runs free in float64 on the same seeded inputs.  With bf16 weights the two
    trajectories differ at rounding level (a SwiGLU value or an element of s_l that lands on the neighbouring
    bf16 value), which moves router logits by a few 1e-4; so expert sets must agree layer by layer unless the
    checker's deciding margin (k-th against (k+1)-th logit) is that small.  A token is compared up to its
    first disagreement (after it the trajectories are different tokens); a disagreement beside a comfortable
    margin is a bug."""
    from paper_2603_19289_amd import moe_spec as M
    from paper_2603_19289_amd.engine import engine_for
    from tests.helpers import make_advance, output_errors
    wl = W.CONFIGS["c2_qwen3_30b_a3b"].with_(n_layers=6, tokens=12)
    res, model, pool = prebuilt(wl)
    x0, eps = W.make_inputs(wl)
    orc = O.MoEOracle(model, MODES[mode], wl.slots)
    trace = O.run_tokens(orc, x0, make_advance(wl, eps))
    dev_x0, dev_eps = torch.from_numpy(x0).cuda(), torch.from_numpy(eps).cuda()
    eng = engine_for(wl, MODES[mode], res, pool, copy_engine=M.COPY_DMA2)
    compared = disagreements = 0
    worst_margin_at_disagreement = worst_l2 = worst_elem = 0.0
    try:
        for t in range(wl.tokens):
            eng.begin_token()
            r = dev_x0[t].clone()
            steps = []
            for l in range(wl.n_layers):
                out, ids = eng.layer_step(l, r, want_ids=True)
                steps.append((out, ids))
                if l + 1 < wl.n_layers:
                    with torch.cuda.stream(eng.compute):
                        r = eng.advance(r, out, dev_eps[t, l], wl.res_a, wl.res_b)
            torch.cuda.synchronize()
            for l, (out, ids) in enumerate(steps):
                want = trace[t][l][1]
                # as sets: two selected experts whose logits nearly tie may swap ranks, which changes nothing
                # but the order of the k terms of the sums
                as_set = lambda a: np.sort(np.asarray(a), axis=-1)
                same_true = np.array_equal(as_set(ids["true_ids"].cpu().numpy()), as_set(want.true_ids))
                same_next = want.next_ids is None or np.array_equal(as_set(ids["next_ids"].cpu().numpy()), as_set(want.next_ids))
                if not (same_true and same_next):
                    margin = float(want.true_margin.min() if not same_true else want.next_margin.min())
                    disagreements += 1
                    worst_margin_at_disagreement = max(worst_margin_at_disagreement, margin)
                    assert margin < 2e-3, (t, l, margin, ids["true_ids"].cpu().numpy(), want.true_ids)
                    break
                np.testing.assert_array_equal(as_set(ids["exec_ids"].cpu().numpy()), as_set(want.exec_ids))
                # the two sides no longer see the same r_l (a few elements of s_l sit on neighbouring bf16
                # values), so the element-wise bound is wider than in the teacher-forced tests
                l2, elem = output_errors(out.cpu().numpy(), want.out)
                worst_l2, worst_elem = max(worst_l2, l2), max(worst_elem, elem)
                assert l2 <= 2e-2 and elem <= 5e-2, (t, l, l2, elem)
                compared += 1
    finally:
        eng.close()
    print(f"[free-running c2 shape] mode={mode}: {compared} layer steps agree in ids and outputs, {disagreements} "
          f"tokens left the checker's trajectory (largest deciding margin there {worst_margin_at_disagreement:.2e}); "
          f"worst relative L2 error {worst_l2:.3e}, worst element error {worst_elem:.3e} of the row RMS", flush=True)
    assert compared >= wl.tokens          # at least the first layers of every token


def test_routing_hand_off_at_the_widest_shape_against_the_checker():
    """E = 256 experts, k = 16, 64 tokens per step: the largest routing launch the library accepts (four keys
    per lane in the rank sort, 64 token groups handing logits between workgroups).  True and predicted ids of
    every token against the checker over a few hundred layer steps, stopping at the first difference."""
    from paper_2603_19289_amd import moe_spec as M
    from paper_2603_19289_amd.engine import engine_for
    from tests.helpers import build, make_advance, small_workload
    wl = small_workload(name="widest_router", n_layers=3, hidden=136, n_experts=256, top_k=16, inter=8, dtype="bf16",
                        batch=64, tokens=100, slots=256, seed=97)
    res, ex, model = build(wl, "random")
    x0, eps = W.make_inputs(wl)
    orc = O.MoEOracle(model, O.MODE_ON_DEMAND, wl.slots, predict=True)
    trace = O.run_tokens(orc, x0, make_advance(wl, eps))
    eng = engine_for(wl, M.MODE_ON_DEMAND, res, ex, predict_in_on_demand=1)
    steps = 0
    try:
        for t in range(wl.tokens):
            eng.begin_token()
            for l in range(wl.n_layers):
                r_np, want = trace[t][l]
                _, ids = eng.layer_step(l, torch.from_numpy(r_np.astype(np.float32)).cuda(), want_ids=True)
                torch.cuda.synchronize()
                np.testing.assert_array_equal(ids["true_ids"].cpu().numpy(), want.true_ids, err_msg=f"token {t} layer {l}")
                if want.next_ids is not None:
                    np.testing.assert_array_equal(ids["next_ids"].cpu().numpy(), want.next_ids, err_msg=f"token {t} layer {l}")
                steps += 1
        st = eng.stats()
        assert st["hits"] == orc.stats.hits and st["predictions"] == orc.stats.predictions
    finally:
        eng.close()
    print(f"[widest router] {steps} layer steps x 64 tokens: every true and predicted id equals the checker's", flush=True)
