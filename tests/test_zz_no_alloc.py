"""The allocation-free entry point, moe_spec_layer_step_static, against moe_spec_layer_step.

Both run the same kernels; the static one keeps the scratch of a layer step in the library's static
device array instead of in the caller's arena.  Two contexts are fed the same seeded inputs, one
through each entry point: ids, gates and outputs must be equal bit for bit (which also puts the
static path inside the tolerances the other entry point is held to against the CPU checker), on
several calls in a row, the later ones with a smaller batch than the first, so that whatever the
earlier calls left in the array lies beyond what the later ones write.  Runs last: see the file name."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2603_19289_amd import moe_spec as M
from paper_2603_19289_amd import workload as W
from tests.helpers import build, check_output, make_advance, small_workload

pytestmark = pytest.mark.gpu


def _step_both(eng_arena, eng_static, layer, r):
    out_a, ids_a = eng_arena.layer_step(layer, r, want_ids=True)
    out_s, ids_s = eng_static.layer_step(layer, r, want_ids=True, static_scratch=True)
    torch.cuda.synchronize()
    for key in ids_a:
        assert torch.equal(ids_a[key].view(torch.int32), ids_s[key].view(torch.int32)), (layer, key)
    assert torch.equal(out_a.view(torch.int32), out_s.view(torch.int32)), layer
    return out_s, ids_s


@pytest.mark.parametrize("dtype,mode", [("bf16", M.MODE_SPECULATIVE), ("f32", M.MODE_ON_DEMAND), ("bf16", M.MODE_PREFETCH_HINT)])
def test_static_scratch_entry_point_equals_the_arena_one(dtype, mode):
    from paper_2603_19289_amd.engine import engine_for
    big = small_workload(name="static_big", n_layers=3, hidden=264, n_experts=12, top_k=3, inter=200, dtype=dtype,
                         batch=6, tokens=2, slots=5, seed=29)
    small = big.with_(name="static_small", batch=2, tokens=2, seed=30)
    res, ex, model = build(big, "random")
    eng_a = engine_for(big, mode, res, ex)
    eng_s = engine_for(big, mode, res, ex)
    # the checker sees the same sequence of tokens: two of batch 6, then two of batch 2
    orc = O.MoEOracle(model, mode, big.slots)
    try:
        for wl in (big, small):
            x0, eps = W.make_inputs(wl)
            trace = O.run_tokens(orc, x0, make_advance(wl, eps))
            for t in range(wl.tokens):
                eng_a.begin_token()
                eng_s.begin_token()
                for l in range(wl.n_layers):
                    r_np, want = trace[t][l]
                    r = torch.from_numpy(r_np.astype(np.float32)).cuda()
                    out, ids = _step_both(eng_a, eng_s, l, r)
                    np.testing.assert_array_equal(ids["exec_ids"].cpu().numpy(), want.exec_ids)
                    np.testing.assert_array_equal(ids["true_ids"].cpu().numpy(), want.true_ids)
                    check_output(out.cpu().numpy(), want.out, dtype, f"batch {wl.batch} token {t} layer {l}")
        st_a, st_s = eng_a.stats(), eng_s.stats()
        for key in ("tokens", "layer_steps", "predictions", "hits", "cache_hits", "cache_misses", "h2d_bytes"):
            assert st_a[key] == st_s[key] == getattr(orc.stats, key), key
    finally:
        eng_a.close()
        eng_s.close()


def test_static_scratch_batch_one_and_matrix_core_paths_one_after_the_other():
    # the three expert paths share the array: batch 1 (register-resident GEMVs), then a matrix-core batch,
    # then batch 1 again, each compared with the arena entry point
    from paper_2603_19289_amd.engine import engine_for
    wl = small_workload(name="static_paths", n_layers=2, hidden=256, n_experts=10, top_k=2, inter=136, dtype="bf16",
                        batch=20, tokens=1, slots=4, seed=31)
    res, ex, _ = build(wl, "random")
    eng_a = engine_for(wl, M.MODE_SPECULATIVE, res, ex)
    eng_s = engine_for(wl, M.MODE_SPECULATIVE, res, ex)
    g = torch.Generator(device="cuda").manual_seed(5)
    try:
        for batch in (1, 20, 1, 3):
            eng_a.begin_token()
            eng_s.begin_token()
            r = torch.randn((batch, wl.hidden), generator=g, device="cuda")
            for l in range(wl.n_layers):
                out, _ = _step_both(eng_a, eng_s, l, r)
                r = (r + out).contiguous()
    finally:
        eng_a.close()
        eng_s.close()


def test_static_scratch_refuses_what_does_not_fit():
    from paper_2603_19289_amd.engine import engine_for
    # step scratch grows with max_batch * k * (I + H): this one needs more than the array holds
    wl = small_workload(name="static_too_big", n_layers=2, hidden=2048, n_experts=8, top_k=8, inter=4096, dtype="bf16",
                        batch=64, tokens=1, slots=8)
    res = W.make_resident(wl)
    pool = torch.zeros((wl.n_layers, wl.n_experts, wl.expert_elems), dtype=torch.bfloat16).pin_memory()
    eng = engine_for(wl, M.MODE_ON_DEMAND, res, pool)
    r = torch.zeros((64, wl.hidden), device="cuda")
    try:
        eng.begin_token()
        with pytest.raises(M.MoeSpecError) as ei:
            eng.layer_step(0, r, static_scratch=True)
        assert ei.value.code == M.EINVAL and "static array" in str(ei.value)
        eng.layer_step(0, r)                                 # the arena entry point still works
        torch.cuda.synchronize()
    finally:
        eng.close()
    small = small_workload(n_layers=2)
    res, ex, _ = build(small)
    eng = engine_for(small, M.MODE_ON_DEMAND, res, ex, profile=1)
    try:
        eng.begin_token()
        with pytest.raises(M.MoeSpecError) as ei:
            eng.layer_step(0, torch.zeros((1, small.hidden), device="cuda"), static_scratch=True)
        assert ei.value.code == M.ESTATE
    finally:
        eng.close()
