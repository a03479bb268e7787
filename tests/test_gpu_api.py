"""GPU-side checks of the C ABI's state machine and error returns, of reset/repeatability, of the
two copy engines agreeing, and free-running parity with a margin audit."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2603_19289_amd import moe_spec as M
from paper_2603_19289_amd import workload as W
from tests.helpers import build, check_output, make_advance, small_workload

pytestmark = pytest.mark.gpu


def _engine(wl, mode, res, ex, **kw):
    from paper_2603_19289_amd.engine import engine_for
    return engine_for(wl, mode, res, ex, **kw)


def test_state_machine_errors():
    wl = small_workload(n_layers=3, tokens=1)
    res, ex, _ = build(wl)
    eng = _engine(wl, M.MODE_SPECULATIVE, res, ex)
    r = torch.randn(1, wl.hidden, device="cuda")
    out = torch.empty_like(r)
    lib = M.lib()
    step = lambda layer, batch=1: lib.moe_spec_layer_step(eng.ctx, layer, r.data_ptr(), batch, out.data_ptr(), None)
    assert step(0) == M.ESTATE                                   # before begin_token
    assert b"begin_token" in lib.moe_spec_last_error(eng.ctx)
    eng.begin_token()
    assert step(1) == M.ESTATE                                   # out of order
    assert step(0, batch=2) == M.EINVAL                          # beyond max_batch
    assert lib.moe_spec_layer_step(eng.ctx, 0, None, 1, out.data_ptr(), None) == M.EINVAL
    assert step(0) == M.OK
    assert step(0) == M.ESTATE                                   # layer 0 twice
    assert step(1) == M.OK and step(2) == M.OK
    assert step(3) == M.ESTATE                                   # past the last layer: token is closed
    torch.cuda.synchronize()
    # registration errors
    assert lib.moe_spec_set_layer_resident(eng.ctx, 9, 1, 1, 1) == M.EINVAL
    assert lib.moe_spec_load_host_experts(eng.ctx, 0, 0, wl.n_experts + 1, eng.pool.data_ptr(), 0) == M.EINVAL
    assert lib.moe_spec_load_host_experts(eng.ctx, 0, 0, 1, eng.pool.data_ptr(), 7) == M.EINVAL          # wrong size
    pageable = np.zeros(eng.expert_bytes, dtype=np.uint8)
    assert lib.moe_spec_load_host_experts(eng.ctx, 0, 0, 1, pageable.ctypes.data, eng.expert_bytes) == M.EINVAL
    assert b"pinned" in lib.moe_spec_last_error(eng.ctx)
    eng.close()


def test_stepping_a_layer_whose_tables_or_experts_are_missing():
    wl = small_workload(n_layers=2, tokens=1)
    cfg = M.Config(n_layers=2, hidden=wl.hidden, n_experts=wl.n_experts, top_k=wl.top_k, inter=wl.inter, max_batch=1,
                   slots_per_layer=wl.slots, dtype=M.BF16, mode=M.MODE_ON_DEMAND, rms_eps=1e-6, copy_engine=M.COPY_KERNEL)
    arena = torch.empty(M.moe_spec_arena_bytes(cfg), dtype=torch.uint8, device="cuda")
    cs, ks = torch.cuda.Stream(), torch.cuda.Stream()
    cfg.device_arena, cfg.device_arena_bytes = arena.data_ptr(), arena.numel()
    cfg.compute_stream, cfg.copy_stream = cs.cuda_stream, ks.cuda_stream
    ctx = M.moe_spec_create(cfg)
    r = torch.randn(1, wl.hidden, device="cuda"); out = torch.empty_like(r)
    torch.cuda.synchronize()
    lib = M.lib()
    M.moe_spec_begin_token(ctx)
    assert lib.moe_spec_layer_step(ctx, 0, r.data_ptr(), 1, out.data_ptr(), None) == M.ESTATE    # no tables
    res, ex, _ = build(wl)
    from paper_2603_19289_amd.engine import _np_to_torch_storage
    rw = _np_to_torch_storage(res["router_w"]).cuda(); dv = _np_to_torch_storage(res["dvecs"]).cuda()
    gn = torch.from_numpy(res["rms_gain"]).cuda()
    for l in range(2):
        M.moe_spec_set_layer_resident(ctx, l, rw[l].data_ptr(), gn[l].data_ptr(), dv[l].data_ptr())
    torch.cuda.synchronize()
    assert lib.moe_spec_layer_step(ctx, 0, r.data_ptr(), 1, out.data_ptr(), None) == M.ESTATE    # no experts registered
    assert b"never registered" in lib.moe_spec_last_error(ctx)
    M.moe_spec_destroy(ctx)


def _run_free(eng, wl, x0, eps):
    """GPU runs free: its own outputs feed the synthetic residual driver."""
    dev_x0, dev_eps = torch.from_numpy(x0).cuda(), torch.from_numpy(eps).cuda()
    ids_log, outs = [], []
    for t in range(x0.shape[0]):
        eng.begin_token()
        r = dev_x0[t].clone()
        for l in range(wl.n_layers):
            out, ids = eng.layer_step(l, r, want_ids=True)
            ids_log.append({k: v for k, v in ids.items()})
            outs.append(out)
            if l + 1 < wl.n_layers:
                with torch.cuda.stream(eng.compute):
                    r = eng.advance(r, out, dev_eps[t, l], wl.res_a, wl.res_b)
    torch.cuda.synchronize()
    return ids_log, outs


@pytest.mark.parametrize("mode", [M.MODE_ON_DEMAND, M.MODE_SPECULATIVE])
def test_free_running_c1_matches_the_checker_with_margin_audit(mode):
    # The GPU computes its own residual trajectory in float32.  Expert sets must still match the
    # checker's unless the deciding logit margin is at rounding level; any mismatch with a
    # comfortable margin is a bug.
    wl = W.CONFIGS["c1_tiny"]
    res, ex, model = build(wl, gains="ones")
    x0, eps = W.make_inputs(wl)
    orc = O.MoEOracle(model, mode, wl.slots)
    trace = O.run_tokens(orc, x0, make_advance(wl, eps))
    eng = _engine(wl, mode, res, ex)
    ids_log, outs = _run_free(eng, wl, x0, eps)
    mismatches = 0
    i = 0
    for t in range(wl.tokens):
        for l in range(wl.n_layers):
            want = trace[t][l][1]
            got = ids_log[i]["true_ids"].cpu().numpy()
            if not np.array_equal(np.sort(got), np.sort(want.true_ids)):
                mismatches += 1
                assert want.true_margin.min() < 1e-4, (t, l, got, want.true_ids, want.true_margin)
            i += 1
    st = eng.stats()
    eng.close()
    if mismatches == 0:
        assert st["hits"] == orc.stats.hits and st["cache_misses"] == orc.stats.cache_misses
        err = np.linalg.norm(outs[-1].cpu().numpy() - trace[-1][-1][1].out) / np.linalg.norm(trace[-1][-1][1].out)
        assert err < 1e-4
    print(f"[free-running] mode={mode} mismatching layer steps: {mismatches}", flush=True)


def test_reset_makes_runs_repeatable_and_copy_engines_agree():
    wl = small_workload(n_layers=4, hidden=264, n_experts=12, top_k=3, inter=200, tokens=6, slots=4, seed=21)
    res, ex, _ = build(wl)
    x0, eps = W.make_inputs(wl)
    results = []
    for engine_kind in (M.COPY_KERNEL, M.COPY_DMA, M.COPY_DMA2):
        eng = _engine(wl, M.MODE_SPECULATIVE, res, ex, copy_engine=engine_kind)
        for rep in range(2):
            eng.reset()
            ids_log, outs = _run_free(eng, wl, x0, eps)
            st = eng.stats()
            results.append((torch.stack(outs).cpu().numpy(), torch.stack([d["exec_ids"] for d in ids_log]).cpu().numpy(),
                            {k: st[k] for k in ("hits", "predictions", "cache_hits", "cache_misses", "h2d_bytes", "tokens")}))
        eng.close()
    for other in results[1:]:
        np.testing.assert_array_equal(other[0], results[0][0])          # bit-identical outputs
        np.testing.assert_array_equal(other[1], results[0][1])
        assert other[2] == results[0][2]


def test_smallest_pool_reuses_every_slot_without_corruption():
    # S = k: every token overwrites every slot of every layer; with repeated inputs the outputs must
    # repeat exactly, which fails if a copy ever lands in a slot that is still being read
    wl = small_workload(n_layers=3, hidden=264, n_experts=12, top_k=3, inter=200, tokens=8, slots=3, seed=33)
    res, ex, _ = build(wl)
    x0, eps = W.make_inputs(wl)
    x0[4:] = x0[:4]
    eps[4:] = eps[:4]
    eng = _engine(wl, M.MODE_SPECULATIVE, res, ex)
    _, outs = _run_free(eng, wl, x0, eps)
    eng.close()
    o = torch.stack(outs).cpu().numpy().reshape(8, wl.n_layers, -1)
    np.testing.assert_array_equal(o[:4], o[4:])


@pytest.mark.parametrize("signal", [0, 1])
@pytest.mark.parametrize("dtype,B", [("bf16", 1), ("f32", 3), ("bf16", 20)])
def test_per_layer_diagnostics_match_the_checker(signal, dtype, B):
    # recall, per-rank agreement and cosine similarity per layer, for the quasi-hidden state and for
    # the baseline signal s_l; teacher-forced so that both sides see the same inputs
    wl = small_workload(n_layers=5, hidden=264, n_experts=12, top_k=3, inter=200, dtype=dtype, batch=B,
                        tokens=4, slots=12, seed=41)
    res, ex, model = build(wl, gains="random")
    x0, eps = W.make_inputs(wl)
    orc = O.MoEOracle(model, O.MODE_SPECULATIVE, wl.slots, predict_signal=signal)
    trace = O.run_tokens(orc, x0, make_advance(wl, eps))
    eng = _engine(wl, M.MODE_SPECULATIVE, res, ex, predict_signal=signal, diagnostics=1)
    for t in range(wl.tokens):
        eng.begin_token()
        for l in range(wl.n_layers):
            r = torch.from_numpy(trace[t][l][0].astype(np.float32)).cuda()
            _, ids = eng.layer_step(l, r, want_ids=True)
            torch.cuda.synchronize()
            np.testing.assert_array_equal(ids["exec_ids"].cpu().numpy(), trace[t][l][1].exec_ids)
    for l in range(wl.n_layers):
        got, want = eng.layer_diagnostics(l), orc.diag[l]
        assert got["predictions"] == want.predictions and got["hits"] == want.hits, l
        assert got["rank_match"][:wl.top_k] == want.rank_match, l
        assert got["cos_count"] == want.cos_count
        assert abs(got["cos_sum"] - want.cos_sum) <= 1e-6 * max(1, want.cos_count), (l, got["cos_sum"], want.cos_sum)
    st = eng.stats()
    assert st["hits"] == orc.stats.hits and st["predictions"] == orc.stats.predictions
    eng.close()


@pytest.mark.parametrize("dtype,B,mode", [("f32", 1, M.MODE_ON_DEMAND), ("bf16", 1, M.MODE_SPECULATIVE), ("f32", 3, M.MODE_ON_DEMAND),
                                           ("bf16", 3, M.MODE_SPECULATIVE), ("bf16", 20, M.MODE_ON_DEMAND)])
def test_accumulated_default_vectors_match_the_checker(dtype, B, mode):
    # the offline statistic behind d_{l,e}: mean un-gated output per executed expert, with counts
    wl = small_workload(n_layers=3, hidden=264, n_experts=12, top_k=3, inter=200, dtype=dtype, batch=B,
                        tokens=5, slots=5, seed=61)
    res, ex, model = build(wl, gains="random")
    x0, eps = W.make_inputs(wl)
    orc = O.MoEOracle(model, mode, wl.slots)
    trace = O.run_tokens(orc, x0, make_advance(wl, eps))
    eng = _engine(wl, mode, res, ex, accumulate_defaults=1)
    for t in range(wl.tokens):
        eng.begin_token()
        for l in range(wl.n_layers):
            out, _ = eng.layer_step(l, torch.from_numpy(trace[t][l][0].astype(np.float32)).cuda())
            torch.cuda.synchronize()
            check_output(out.cpu().numpy(), trace[t][l][1].out, dtype, f"token {t} layer {l}")
    for l in range(wl.n_layers):
        mean, counts = eng.read_default_vectors(l)
        assert counts == orc.dacc_cnt[l].tolist()
        got, want = mean.cpu().numpy().astype(np.float64), orc.default_vectors(l)
        for e in range(wl.n_experts):
            if counts[e]:
                check_output(got[e], want[e], dtype, f"default vector of layer {l}, expert {e}")
            else:
                assert not got[e].any()
    eng.close()
    # a context without the flag refuses
    eng = _engine(wl, mode, res, ex)
    buf = torch.empty((wl.n_experts, wl.hidden), device="cuda")
    assert M.lib().moe_spec_read_default_vectors(eng.ctx, 0, buf.data_ptr(), None) == M.ESTATE
    eng.close()


def test_time_kernel_modes_and_their_byte_counts():
    # the measurement aid: every mode runs, reports the weight bytes of its launch, and refuses what it cannot do
    wl = small_workload(n_layers=3, hidden=128, n_experts=12, top_k=3, inter=96, dtype="bf16", batch=20, slots=5)
    res, ex, _ = build(wl)
    eng = _engine(wl, M.MODE_SPECULATIVE, res, ex)
    w = 2
    want = {0: wl.top_k * 2 * wl.inter * wl.hidden * w, 1: wl.top_k * wl.inter * wl.hidden * w,
            2: wl.n_experts * wl.hidden * w, 3: wl.top_k * 2 * wl.inter * wl.hidden * w,
            4: 5 * 2 * wl.inter * wl.hidden * w, 5: 5 * wl.inter * wl.hidden * w,     # 5 = min(S, E, B*k) slots
            6: wl.n_experts * wl.hidden * w, 7: (2 * wl.n_experts + wl.batch * wl.top_k) * wl.hidden * w,
            9: wl.top_k * wl.inter * wl.hidden * w}
    for which, nbytes in want.items():
        ms, got = eng.time_kernel(which, 6)
        assert ms > 0 and got == nbytes, (which, ms, got, nbytes)
    with pytest.raises(M.MoeSpecError):
        eng.time_kernel(10, 1)
    eng.begin_token()
    with pytest.raises(M.MoeSpecError) as ei:
        eng.time_kernel(0, 1)                    # not inside a decode step
    assert ei.value.code == M.ESTATE
    eng.close()
    wl32 = small_workload(dtype="f32")
    res, ex, _ = build(wl32)
    eng = _engine(wl32, M.MODE_ON_DEMAND, res, ex)
    with pytest.raises(M.MoeSpecError) as ei:
        eng.time_kernel(4, 1)                    # matrix-core kernels are bf16 only
    assert ei.value.code == M.ESTATE
    eng.close()


@pytest.mark.parametrize("dtype,B", [("f32", 1), ("bf16", 1), ("bf16", 6)])
def test_non_finite_inputs_keep_expert_ids_in_range(dtype, B):
    # NaN or infinite activations give NaN logits; the ranking must still hand out k distinct ids inside
    # [0, E) (they index weight rows and host tables), outputs are NaN, and the context stays usable
    wl = small_workload(n_layers=3, hidden=128, n_experts=70, top_k=4, inter=64, dtype=dtype, batch=B, slots=8, tokens=2)
    res, ex, model = build(wl, "random")
    x0, eps = W.make_inputs(wl)
    for mode in (M.MODE_SPECULATIVE, M.MODE_ON_DEMAND):
        eng = _engine(wl, mode, res, ex)
        try:
            for bad in (float("nan"), float("inf")):
                eng.begin_token()
                r = torch.from_numpy(x0[0]).cuda()
                r[0, 5] = bad
                for l in range(wl.n_layers):
                    out, ids = eng.layer_step(l, r, want_ids=True)
                    torch.cuda.synchronize()
                    for key in ("true_ids", "exec_ids") + (("next_ids",) if l + 1 < wl.n_layers else ()):
                        got = ids[key].cpu().numpy()
                        assert ((got >= 0) & (got < wl.n_experts)).all(), (key, got)
                        assert all(len(set(row)) == wl.top_k for row in got.tolist()), (key, got)
                    assert torch.isnan(out[0]).all()
                    r = r + out
            # a clean token afterwards matches the checker again
            eng.reset()
            orc = O.MoEOracle(model, mode, wl.slots)
            trace = O.run_tokens(orc, x0[:1], make_advance(wl, eps))
            eng.begin_token()
            for l in range(wl.n_layers):
                r_np, want = trace[0][l]
                out, ids = eng.layer_step(l, torch.from_numpy(r_np.astype(np.float32)).cuda(), want_ids=True)
                torch.cuda.synchronize()
                np.testing.assert_array_equal(ids["exec_ids"].cpu().numpy(), want.exec_ids)
        finally:
            eng.close()


def test_a_wait_that_runs_out_is_reported_and_reset_recovers():
    # The fused kernels wait, boundedly, for results of other workgroups of the same launch.  With the bound
    # forced down to one poll from the host, waiters give up early: every kernel still runs to its end, ids
    # stay inside [0, E), the next call (or moe_spec_stats) reports the failure, and moe_spec_reset brings
    # the context back.  With the default bound the same inputs match the checker.
    wl = small_workload(n_layers=3, hidden=512, n_experts=64, top_k=4, inter=256, dtype="bf16", slots=8, tokens=3, seed=77)
    res, ex, model = build(wl, "random")
    x0, eps = W.make_inputs(wl)
    orc = O.MoEOracle(model, O.MODE_SPECULATIVE, wl.slots)
    trace = O.run_tokens(orc, x0, make_advance(wl, eps))
    eng = _engine(wl, M.MODE_SPECULATIVE, res, ex, wait_spin_limit=1)
    gave_up = False
    try:
        for t in range(wl.tokens):
            try:
                eng.begin_token()
                for l in range(wl.n_layers):
                    _, ids = eng.layer_step(l, torch.from_numpy(trace[t][l][0].astype(np.float32)).cuda(), want_ids=True)
                    torch.cuda.synchronize()
                    got = ids["exec_ids"].cpu().numpy()
                    assert ((got >= 0) & (got < wl.n_experts)).all()
            except M.MoeSpecError as err:
                assert err.code == M.EHIP and "bounded wait" in str(err)
                gave_up = True
                break
        if not gave_up:
            try:
                eng.stats()
            except M.MoeSpecError as err:
                assert err.code == M.EHIP and "bounded wait" in str(err)
                gave_up = True
        print(f"[bounded wait] one poll allowed: waiters gave up = {gave_up}", flush=True)
        eng.reset()
        assert eng.stats()["tokens"] == 0                        # the context answers again
    finally:
        eng.close()
    eng = _engine(wl, M.MODE_SPECULATIVE, res, ex)
    try:
        for t in range(wl.tokens):
            eng.begin_token()
            for l in range(wl.n_layers):
                _, ids = eng.layer_step(l, torch.from_numpy(trace[t][l][0].astype(np.float32)).cuda(), want_ids=True)
                torch.cuda.synchronize()
                np.testing.assert_array_equal(ids["exec_ids"].cpu().numpy(), trace[t][l][1].exec_ids)
        assert eng.stats()["hits"] == orc.stats.hits
    finally:
        eng.close()


def test_random_call_sequences_leave_a_working_context():
    """Forty seeded contexts, each put through 10 to 60 random calls, valid and invalid (steps in and out of order,
    oversized batches, null pointers, resets and statistics in the middle of a token, timing and prefill calls at the
    wrong moment, both entry points of the layer step): invalid calls must be refused with EINVAL / ESTATE, and
    afterwards a clean token through the context must equal, bit for bit, the same token through a context that saw
    none of it."""
    rng = np.random.default_rng(61)
    modes = [M.MODE_ON_DEMAND, M.MODE_SPECULATIVE, M.MODE_PREFETCH_HINT]

    def clean_token(eng, wl, x, static):
        eng.reset()
        eng.begin_token()
        outs, r = [], x
        for l in range(wl.n_layers):
            out, _ = eng.layer_step(l, r, static_scratch=static)
            torch.cuda.synchronize()
            outs.append(out.clone())
            r = (r + out).contiguous()
        return outs

    for case in range(40):
        L, E = int(rng.integers(2, 6)), int(rng.integers(2, 24))
        k = int(rng.integers(1, min(E, 6) + 1))
        S, Bmax = int(rng.integers(k, E + 1)), int(rng.choice([1, 2, 5, 16]))
        mode = modes[int(rng.integers(0, 3))]
        wl = small_workload(name=f"calls{case}", n_layers=L, hidden=int(rng.choice([16, 64, 264])), n_experts=E, top_k=k,
                            inter=int(rng.choice([8, 40, 104])), dtype="bf16" if rng.random() < 0.6 else "f32",
                            batch=Bmax, tokens=1, slots=S, seed=6100 + case)
        look = 2 if (mode != M.MODE_ON_DEMAND and L >= 3 and rng.random() < 0.3) else 0
        kw = dict(copy_engine=int(rng.integers(0, 3)), lookahead=look, max_prefill_tokens=int(rng.choice([0, 0, 32])))
        res, ex, _ = build(wl, "random")
        eng, ref = _engine(wl, mode, res, ex, **kw), _engine(wl, mode, res, ex, **kw)
        g = torch.Generator(device="cuda").manual_seed(case)
        is_open, nxt, batch = False, 0, 0
        try:
            for _ in range(int(rng.integers(10, 60))):
                op = rng.choice(["begin", "step", "step", "step", "wrong_layer", "bad_batch", "reset", "stats", "time",
                                 "prefill", "null"])
                must_fail = must_pass = False
                try:
                    if op == "begin":
                        must_pass = True
                        eng.begin_token()
                        is_open, nxt = True, 0
                    elif op == "step":
                        B = int(rng.integers(1, Bmax + 1)) if nxt == 0 else batch
                        must_pass, must_fail = is_open, not is_open
                        r = torch.randn((B, wl.hidden), generator=g, device="cuda")
                        eng.layer_step(nxt if is_open else 0, r, static_scratch=bool(rng.random() < 0.5))
                        batch, nxt = B, nxt + 1
                        is_open = nxt < L
                    elif op == "wrong_layer":
                        must_fail = True
                        r = torch.randn((max(batch, 1), wl.hidden), generator=g, device="cuda")
                        eng.layer_step(nxt + 1, r)
                    elif op == "bad_batch":
                        must_fail = True
                        eng.layer_step(nxt, torch.randn((Bmax + 1, wl.hidden), generator=g, device="cuda"))
                    elif op == "reset":
                        must_pass = True
                        eng.reset()
                        is_open, nxt = False, 0
                    elif op == "stats":
                        must_pass = True
                        eng.stats()
                    elif op == "time":
                        must_fail = is_open
                        eng.time_kernel(int(rng.choice([0, 1, 2, 3, 9])), 3)
                    elif op == "prefill":
                        must_fail = kw["max_prefill_tokens"] == 0 or is_open
                        must_pass = not must_fail
                        r = torch.randn((int(rng.integers(1, 33)), wl.hidden), generator=g, device="cuda")
                        for l in range(L):
                            eng.prefill_layer_step(l, r)
                    else:
                        must_fail = True
                        M.moe_spec_layer_step(eng.ctx, nxt, 0, 1, 0)
                    assert not must_fail, (case, op)
                except M.MoeSpecError as e:
                    assert e.code in (M.EINVAL, M.ESTATE), (case, op, e)
                    assert not must_pass, (case, op, e)
            torch.cuda.synchronize()
            x = torch.randn((Bmax, wl.hidden), generator=torch.Generator(device="cuda").manual_seed(999), device="cuda")
            for static in (False, True):
                a, b = clean_token(eng, wl, x, static), clean_token(ref, wl, x, static)
                for l in range(L):
                    assert torch.equal(a[l].view(torch.int32), b[l].view(torch.int32)), (case, static, l)
        finally:
            eng.close()
            ref.close()
