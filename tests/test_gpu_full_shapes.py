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


CASES = {
    "c2_qwen3_30b_a3b": dict(n_layers=3, tokens=3),
    "c3_gpt_oss_20b": dict(n_layers=3, tokens=2),
    "c3_gpt_oss_20b_b8": dict(n_layers=2, tokens=1),
    "c4_mixtral_8x7b": dict(n_layers=2, tokens=2),
    "c5_qwen3_b32": dict(n_layers=2, tokens=1),
}


@pytest.mark.parametrize("name", list(CASES))
def test_full_layer_shape_both_modes(name):
    wl = W.CONFIGS[name].with_(**CASES[name])
    pre = prebuilt(wl)
    for mode in MODES:
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
