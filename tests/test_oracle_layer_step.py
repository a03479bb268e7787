"""Pins for the checker's layer step (Algorithm 1) and its two execution modes.

The constructions make the quasi-hidden state coincide with the next layer's true router
input, which fixes where d_l enters, which gates weight it and which layer's norm is used;
the remaining tests pin the mode logic, the counters and the pairing of experts with gates."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2603_19289_amd import workload as W
from tests.helpers import build, make_advance, oracle_model, small_workload


def _run(model, wl, mode, x0, adv, **kw):
    orc = O.MoEOracle(model, mode, wl.slots, **kw)
    return orc, O.run_tokens(orc, x0, adv)


def test_zero_default_vectors_zero_update_gives_hit_rate_one():
    # d = 0, no residual noise and W_down = 0 (the block adds nothing): q_l is s_{l+1} bit for bit
    wl = small_workload(n_layers=5, dtype="bf16", res_a=1.0, res_b=0.0, d_std=0.0)
    res, ex, _ = build(wl)
    H, I = wl.hidden, wl.inter
    ex[:, :, 2 * I * H:] = 0
    model = oracle_model(wl, res, ex)
    x0, eps = W.make_inputs(wl)
    adv = make_advance(wl, eps)
    spec, tr_s = _run(model, wl, O.MODE_SPECULATIVE, x0, adv)
    ond, tr_o = _run(model, wl, O.MODE_ON_DEMAND, x0, adv)
    assert spec.stats.predictions == wl.top_k * (wl.n_layers - 1) * wl.tokens
    assert spec.stats.hits == spec.stats.predictions
    for t in range(wl.tokens):
        for l in range(wl.n_layers):
            np.testing.assert_array_equal(tr_s[t][l][1].out, tr_o[t][l][1].out)
            if l + 1 < wl.n_layers:
                np.testing.assert_array_equal(tr_s[t][l][1].q, tr_s[t][l + 1][1].s)


@pytest.mark.parametrize("dtype", ["f32"])
def test_one_sample_default_vectors_make_q_equal_next_router_input(dtype):
    # d_{l,e} := what expert e really outputs for this token, no noise: d_l = O_l, so
    # r_l + d_l = r_{l+1} and q_l = LN_{l+1}(r_{l+1}) = s_{l+1}.  Gains differ per layer so that
    # the wrong layer's norm, a d_l added after the norm, or d_l built from other gates all fail.
    wl = small_workload(n_layers=4, dtype=dtype, tokens=1, res_a=1.0, res_b=0.0)
    res, ex, model = build(wl, gains="random")
    x0, _ = W.make_inputs(wl)

    def adv(t, l, r, out):                     # exact r + O, no float32 stop
        return r + out

    dv = np.zeros((wl.n_layers, wl.n_experts, wl.hidden))           # float64 table
    model.dvecs = dv
    r = np.asarray(x0[0], dtype=np.float64)
    for l in range(wl.n_layers):                                    # fill the table layer by layer
        s = O.rmsnorm(r[0], model.rms_gain[l], model.rms_eps)
        for e in range(wl.n_experts):
            dv[l, e] = O.expert_ffn(*model.expert_mats(l, e), s, False)
        orc = O.MoEOracle(model, O.MODE_ON_DEMAND, wl.slots)
        tr = O.run_tokens(orc, x0, adv, n_layers=l + 1)
        r = adv(0, l, tr[0][l][0], tr[0][l][1].out)

    spec, tr_s = _run(model, wl, O.MODE_SPECULATIVE, x0, adv)
    ond, tr_o = _run(model, wl, O.MODE_ON_DEMAND, x0, adv)
    assert spec.stats.hits == spec.stats.predictions == wl.top_k * (wl.n_layers - 1)
    for l in range(wl.n_layers):
        np.testing.assert_allclose(tr_s[0][l][1].out, tr_o[0][l][1].out, rtol=0, atol=1e-13)
        if l + 1 < wl.n_layers:
            np.testing.assert_allclose(tr_s[0][l][1].q, tr_s[0][l + 1][1].s, rtol=0, atol=1e-13)
            np.testing.assert_allclose(tr_s[0][l][1].next_gates, tr_s[0][l + 1][1].true_gates, atol=1e-12)


@pytest.mark.parametrize("bad", ["gain_of_wrong_layer", "uniform_gates", "d_after_norm", "dropped_d"])
def test_planted_mistakes_in_the_quasi_hidden_state_are_caught(bad, monkeypatch):
    # the construction above must tell these mistakes apart from the definition
    wl = small_workload(n_layers=3, dtype="f32", tokens=1, res_a=1.0, res_b=0.0)
    res, ex, model = build(wl, gains="random")
    x0, _ = W.make_inputs(wl)
    adv = lambda t, l, r, out: r + out
    dv = np.zeros((wl.n_layers, wl.n_experts, wl.hidden))
    model.dvecs = dv
    r = np.asarray(x0[0], dtype=np.float64)
    for l in range(wl.n_layers):
        s = O.rmsnorm(r[0], model.rms_gain[l], model.rms_eps)
        for e in range(wl.n_experts):
            dv[l, e] = O.expert_ffn(*model.expert_mats(l, e), s, False)
        tr = O.run_tokens(O.MoEOracle(model, O.MODE_ON_DEMAND, wl.slots), x0, adv, n_layers=l + 1)
        r = adv(0, l, tr[0][l][0], tr[0][l][1].out)

    good_q, good_d = O.quasi_hidden, O.layer_default_vector
    if bad == "gain_of_wrong_layer":
        gains = model.rms_gain
        monkeypatch.setattr(O, "quasi_hidden", lambda r_, s_, d_, g_, eps, bf, fn=False:
                            good_q(r_, s_, d_, gains[[np.array_equal(g_, gains[i]) for i in range(len(gains))].index(True) - 1], eps, bf, fn))
    elif bad == "uniform_gates":
        monkeypatch.setattr(O, "layer_default_vector", lambda dvl, ids, g: good_d(dvl, ids, np.full(len(g), 1 / len(g))))
    elif bad == "d_after_norm":
        monkeypatch.setattr(O, "quasi_hidden", lambda r_, s_, d_, g_, eps, bf, fn=False: O.rmsnorm(r_, g_, eps) + d_)
    else:
        monkeypatch.setattr(O, "layer_default_vector", lambda dvl, ids, g: 0 * good_d(dvl, ids, g))
    _, tr_s = _run(model, wl, O.MODE_ON_DEMAND, x0, adv)
    worst = max(np.abs(tr_s[0][l][1].q - tr_s[0][l + 1][1].s).max() for l in range(wl.n_layers - 1))
    assert worst > 1e-4


@pytest.mark.parametrize("dtype,B", [("f32", 1), ("bf16", 1), ("bf16", 3)])
def test_mode_logic_counters_and_gate_pairing(dtype, B):
    wl = small_workload(n_layers=4, dtype=dtype, batch=B, tokens=5, slots=4)
    res, ex, model = build(wl, gains="random")
    x0, eps = W.make_inputs(wl)
    adv = make_advance(wl, eps)
    spec, tr_s = _run(model, wl, O.MODE_SPECULATIVE, x0, adv)
    ond, tr_o = _run(model, wl, O.MODE_ON_DEMAND, x0, adv)
    k, L, T = wl.top_k, wl.n_layers, wl.tokens
    F = torch.nn.functional
    recount = 0
    for t in range(T):
        # layer 0 is a cold start: identical in both modes
        np.testing.assert_array_equal(tr_s[t][0][1].out, tr_o[t][0][1].out)
        np.testing.assert_array_equal(tr_s[t][0][1].exec_ids, tr_s[t][0][1].true_ids)
        assert tr_s[t][L - 1][1].next_ids is None                 # nothing to predict after the last layer
        for l in range(L):
            rs, ro = tr_s[t][l][1], tr_o[t][l][1]
            np.testing.assert_array_equal(ro.exec_ids, ro.true_ids)          # on-demand executes the routed set
            np.testing.assert_allclose(rs.true_gates.sum(-1), 1.0, atol=1e-15)
            if l > 0:
                prev = tr_s[t][l - 1][1]
                np.testing.assert_array_equal(rs.exec_ids, prev.next_ids)    # speculated experts ...
                np.testing.assert_array_equal(rs.exec_gates, prev.next_gates)  # ... with their predicted gates
                for b in range(B):
                    recount += len(set(prev.next_ids[b].tolist()) & set(rs.true_ids[b].tolist()))
            # output = sum over executed experts of (its gate) * SwiGLU on the TRUE s_l (library arithmetic)
            for b in range(B):
                s = torch.from_numpy(rs.s[b])
                want = torch.zeros(wl.hidden, dtype=torch.float64)
                for j in range(k):
                    wg, wu, wd = (torch.from_numpy(O.decode_weights(m)) for m in model.expert_mats(l, int(rs.exec_ids[b, j])))
                    h = F.silu(F.linear(s, wg)) * F.linear(s, wu)
                    if dtype == "bf16":
                        h = torch.from_numpy(O.bf16_round(h.numpy()))
                    want += rs.exec_gates[b, j] * F.linear(h, wd)
                np.testing.assert_allclose(rs.out[b], want.numpy(), rtol=1e-10, atol=1e-14)
    assert spec.stats.predictions == k * B * (L - 1) * T
    assert 0 <= spec.stats.hits <= spec.stats.predictions
    assert spec.stats.hits == recount
    assert 0 < spec.stats.hits < spec.stats.predictions            # the random workload is neither trivial case
    assert spec.stats.tokens == ond.stats.tokens == T
    assert spec.stats.layer_steps == ond.stats.layer_steps == L * T
    for st in (spec.stats, ond.stats):
        assert st.h2d_bytes == st.cache_misses * wl.expert_bytes
    if B == 1:
        assert ond.stats.cache_hits + ond.stats.cache_misses == k * L * T
        assert spec.stats.cache_hits + spec.stats.cache_misses == k * L * T
        assert spec.stats.cache_waves == ond.stats.cache_waves == L * T     # k <= S: one wave per layer step


def test_router_input_is_rounded_to_bf16_only_in_bf16_mode():
    for dtype in ("f32", "bf16"):
        wl = small_workload(dtype=dtype, tokens=1)
        res, ex, model = build(wl)
        x0, eps = W.make_inputs(wl)
        _, tr = _run(model, wl, O.MODE_ON_DEMAND, x0, make_advance(wl, eps))
        s = tr[0][0][1].s
        assert np.array_equal(s, O.bf16_round(s)) == (dtype == "bf16")


def test_wave_execution_requests_when_the_union_exceeds_the_pool():
    # B*k distinct experts can exceed S: the union is served in waves of S; only wave 0 of a
    # prediction is requested one layer early, later waves when their turn comes
    wl = small_workload(n_layers=3, dtype="f32", batch=4, tokens=3, slots=2, n_experts=8, top_k=2)
    res, ex, model = build(wl)
    x0, eps = W.make_inputs(wl)
    adv = make_advance(wl, eps)
    for mode in (O.MODE_ON_DEMAND, O.MODE_SPECULATIVE):
        orc, tr = _run(model, wl, mode, x0, adv)
        expect = waves = 0
        for t in range(wl.tokens):
            for l in range(wl.n_layers):
                distinct = len(set(tr[t][l][1].exec_ids.reshape(-1).tolist()))
                expect += distinct
                waves += -(-distinct // wl.slots)
        assert orc.stats.cache_waves == waves > wl.tokens * wl.n_layers
        # every executed expert is requested exactly once per layer step; in speculative mode the
        # prefetch of wave 0 happens during the previous step but is still one request per expert
        assert orc.stats.cache_hits + orc.stats.cache_misses == expect
        assert sum(p.clock for p in orc.pools) >= wl.tokens * wl.n_layers


def test_step_order_is_enforced_and_slots_must_cover_k():
    wl = small_workload()
    res, ex, model = build(wl)
    with pytest.raises(ValueError):
        O.MoEOracle(model, O.MODE_ON_DEMAND, wl.top_k - 1)
    orc = O.MoEOracle(model, O.MODE_ON_DEMAND, wl.slots)
    orc.begin_token()
    with pytest.raises(RuntimeError):
        orc.layer_step(1, np.zeros((1, wl.hidden)))


def test_prefetch_hint_mode_executes_the_true_experts_and_counts_the_refetches():
    # the prior-work policy: same outputs as on-demand, prefetch requests as in speculative mode,
    # plus an on-demand request for the true set at every layer (hits where the prediction was right)
    wl = small_workload(n_layers=4, dtype="bf16", batch=2, tokens=5, slots=4)
    res, ex, model = build(wl, gains="random")
    x0, eps = W.make_inputs(wl)
    adv = make_advance(wl, eps)
    hint, tr_h = _run(model, wl, O.MODE_PREFETCH_HINT, x0, adv)
    ond, tr_o = _run(model, wl, O.MODE_ON_DEMAND, x0, adv)
    requested = 0
    for t in range(wl.tokens):
        for l in range(wl.n_layers):
            np.testing.assert_array_equal(tr_h[t][l][1].out, tr_o[t][l][1].out)
            np.testing.assert_array_equal(tr_h[t][l][1].exec_ids, tr_h[t][l][1].true_ids)
            requested += len(set(tr_h[t][l][1].true_ids.reshape(-1).tolist()))
            if tr_h[t][l][1].next_ids is not None:
                requested += min(wl.slots, len(set(tr_h[t][l][1].next_ids.reshape(-1).tolist())))
    assert hint.stats.hits == ond.stats.hits and hint.stats.predictions == ond.stats.predictions
    assert hint.stats.cache_hits + hint.stats.cache_misses == requested
    assert hint.stats.cache_misses >= ond.stats.cache_misses - wl.slots * wl.n_layers   # mispredictions cost transfers


def test_per_layer_diagnostics_in_the_exact_prediction_construction():
    # d = 0, no noise, W_down = 0: the predicting signal IS the next router input, so every rank
    # agrees, cosine is 1 and recall is 1 at every layer; layer 0 is never predicted
    wl = small_workload(n_layers=4, dtype="bf16", res_a=1.0, res_b=0.0, d_std=0.0, batch=2, tokens=3)
    res, ex, _ = build(wl)
    ex[:, :, 2 * wl.inter * wl.hidden:] = 0
    model = oracle_model(wl, res, ex)
    x0, eps = W.make_inputs(wl)
    for signal in (0, 1):            # with unit gains and no drift the baseline signal s_l is exact too
        orc = O.MoEOracle(model, O.MODE_SPECULATIVE, wl.slots, predict_signal=signal)
        O.run_tokens(orc, x0, make_advance(wl, eps))
        assert orc.diag[0].predictions == 0 and orc.diag[0].cos_count == 0
        for l in range(1, wl.n_layers):
            d = orc.diag[l]
            assert d.predictions == wl.top_k * wl.batch * wl.tokens == d.hits
            assert d.rank_match == [wl.batch * wl.tokens] * wl.top_k
            assert d.cos_count == wl.batch * wl.tokens and abs(d.cos_sum / d.cos_count - 1.0) < 1e-12
        assert sum(d.hits for d in orc.diag) == orc.stats.hits


def test_quasi_hidden_state_predicts_better_than_the_baseline_signal_when_defaults_carry_the_update():
    # one-sample default vectors (d_{l,e} := the expert's real output): q_l is exact, while s_l
    # ignores the block's contribution and the change of norm, so it must do worse
    wl = small_workload(n_layers=4, dtype="f32", tokens=1, res_a=1.0, res_b=0.0, w_std=0.3)
    res, ex, model = build(wl, gains="random")
    x0, _ = W.make_inputs(wl)
    adv = lambda t, l, r, out: r + out
    dv = np.zeros((wl.n_layers, wl.n_experts, wl.hidden))
    model.dvecs = dv
    r = np.asarray(x0[0], dtype=np.float64)
    for l in range(wl.n_layers):
        s = O.rmsnorm(r[0], model.rms_gain[l], model.rms_eps)
        for e in range(wl.n_experts):
            dv[l, e] = O.expert_ffn(*model.expert_mats(l, e), s, False)
        tr = O.run_tokens(O.MoEOracle(model, O.MODE_ON_DEMAND, wl.slots), x0, adv, n_layers=l + 1)
        r = adv(0, l, tr[0][l][0], tr[0][l][1].out)
    q_orc = O.MoEOracle(model, O.MODE_ON_DEMAND, wl.slots, predict_signal=0)
    s_orc = O.MoEOracle(model, O.MODE_ON_DEMAND, wl.slots, predict_signal=1)
    O.run_tokens(q_orc, x0, adv)
    O.run_tokens(s_orc, x0, adv)
    for l in range(1, wl.n_layers):
        assert abs(q_orc.diag[l].cos_sum - 1.0) < 1e-12
        assert s_orc.diag[l].cos_sum < 1.0 - 1e-4
    assert q_orc.stats.hits == q_orc.stats.predictions


def test_estimator_replaces_the_router_only_at_the_named_layers():
    wl = small_workload(n_layers=4, dtype="bf16", tokens=3)
    res, ex, model = build(wl, gains="random")
    x0, eps = W.make_inputs(wl)
    adv = make_advance(wl, eps)
    e = W.make_estimator(wl, m=4, n=2)
    est = O.Estimator(**e)
    plain, tr_p = _run(model, wl, O.MODE_ON_DEMAND, x0, adv)
    hybrid, tr_h = _run(model, wl, O.MODE_ON_DEMAND, x0, adv, estimator=est, estimator_layers=[1])
    for t in range(wl.tokens):
        np.testing.assert_array_equal(tr_h[t][0][1].next_ids, tr_p[t][0][1].next_ids)      # layer 0: router
        np.testing.assert_array_equal(tr_h[t][2][1].next_ids, tr_p[t][2][1].next_ids)      # layer 2: router
        z = O.estimator_logits(est, tr_h[t][1][1].q[0], 1)
        assert tr_h[t][1][1].next_ids[0].tolist() == O.topk_desc(z, wl.top_k).tolist()     # layer 1: estimator
    assert any(not np.array_equal(tr_h[t][1][1].next_ids, tr_p[t][1][1].next_ids) for t in range(wl.tokens))


def test_accumulated_default_vectors_are_the_mean_expert_output_and_close_the_loop():
    wl = small_workload(n_layers=3, dtype="f32", batch=2, tokens=6, slots=4)
    res, ex, model = build(wl, gains="random")
    x0, eps = W.make_inputs(wl)
    orc, tr = _run(model, wl, O.MODE_ON_DEMAND, x0, make_advance(wl, eps))
    F = torch.nn.functional
    for l in range(wl.n_layers):
        acc = {}
        for t in range(wl.tokens):
            st = tr[t][l][1]
            for b in range(wl.batch):
                for j in range(wl.top_k):
                    e = int(st.exec_ids[b, j])
                    wg, wu, wd = (torch.from_numpy(O.decode_weights(m)) for m in model.expert_mats(l, e))
                    s_ = torch.from_numpy(st.s[b])
                    acc.setdefault(e, []).append(F.linear(F.silu(F.linear(s_, wg)) * F.linear(s_, wu), wd).numpy())
        dv = orc.default_vectors(l)
        for e in range(wl.n_experts):
            want = np.mean(acc[e], axis=0) if e in acc else np.zeros(wl.hidden)
            np.testing.assert_allclose(dv[e], want, rtol=1e-10, atol=1e-14)
            assert orc.dacc_cnt[l, e] == len(acc.get(e, []))
    # one token, no noise: the table collected on a first pass makes the prediction exact on a second pass
    wl1 = small_workload(n_layers=4, dtype="f32", tokens=1, res_a=1.0, res_b=0.0)
    res, ex, model = build(wl1, gains="random")
    x0, _ = W.make_inputs(wl1)
    adv = lambda t, l, r, out: r + out
    first, _ = _run(model, wl1, O.MODE_ON_DEMAND, x0, adv)
    model.dvecs = np.stack([first.default_vectors(l) for l in range(wl1.n_layers)])
    second, _ = _run(model, wl1, O.MODE_SPECULATIVE, x0, adv)
    assert second.stats.hits == second.stats.predictions > 0


def test_prefill_is_the_standard_block_on_every_token_and_loads_every_expert():
    wl = small_workload(n_layers=2, dtype="bf16", batch=7, tokens=1, slots=4)
    res, ex, model = build(wl, gains="random")
    x0, _ = W.make_inputs(wl)
    pre = O.MoEOracle(model, O.MODE_SPECULATIVE, wl.slots)
    ond = O.MoEOracle(model, O.MODE_ON_DEMAND, wl.slots)
    ond.begin_token()
    a = pre.prefill_layer_step(0, x0[0])
    b = ond.layer_step(0, x0[0])
    np.testing.assert_array_equal(a.out, b.out)                 # same arithmetic as a decode step on the true experts
    np.testing.assert_array_equal(a.true_ids, b.true_ids)
    assert pre.stats.cache_misses == wl.n_experts and pre.stats.h2d_bytes == wl.n_experts * wl.expert_bytes
    assert pre.stats.predictions == 0
    assert pre.pools[0].slot_expert == [-1] * wl.slots          # nothing is kept for the decode cache


def test_two_layer_lookahead_changes_traffic_and_nothing_else():
    # lookahead = 2 adds one cache request per layer (the experts predicted for layer l+2) and a second recall
    # counter; ids, gates and outputs are those of lookahead = 1 bit for bit, in both prefetching modes
    wl = small_workload(n_layers=5, dtype="bf16", batch=2, tokens=4, slots=4)
    res, ex, model = build(wl, gains="random")
    x0, eps = W.make_inputs(wl)
    adv = make_advance(wl, eps)
    for mode in (O.MODE_SPECULATIVE, O.MODE_PREFETCH_HINT):
        one = O.MoEOracle(model, mode, wl.slots)
        two = O.MoEOracle(model, mode, wl.slots, lookahead=2)
        tr1, tr2 = O.run_tokens(one, x0, adv), O.run_tokens(two, x0, adv)
        for t in range(wl.tokens):
            for l in range(wl.n_layers):
                a, b = tr1[t][l][1], tr2[t][l][1]
                np.testing.assert_array_equal(a.exec_ids, b.exec_ids)
                np.testing.assert_array_equal(a.out, b.out)
                np.testing.assert_array_equal(a.exec_gates, b.exec_gates)
        assert (two.stats.hits, two.stats.predictions) == (one.stats.hits, one.stats.predictions)
        assert two.stats.predictions2 == wl.top_k * wl.batch * (wl.n_layers - 2) * wl.tokens
        assert 0 <= two.stats.hits2 <= two.stats.predictions2 and one.stats.predictions2 == 0
        # every expert is requested at least as often; whatever the hint loaded that was not needed is extra traffic
        assert two.stats.cache_hits + two.stats.cache_misses > one.stats.cache_hits + one.stats.cache_misses
        assert two.stats.h2d_bytes == two.stats.cache_misses * model.expert_bytes
    # on-demand loading has nothing to look ahead with
    ond = O.MoEOracle(model, O.MODE_ON_DEMAND, wl.slots, lookahead=2)
    O.run_tokens(ond, x0, adv)
    assert ond.stats.predictions2 == 0


def test_two_layer_lookahead_is_exact_when_the_residual_stands_still():
    # d = 0, no residual noise and W_down = 0: r_{l+2} = r_{l+1} = r_l, so LN_{l+2}(r_l + d_l) IS s_{l+2} and the
    # two-layer prediction must hit every time, with per-layer gains that differ (the gain of the wrong layer
    # would miss).  With a pool as large as the expert set the hint then loads exactly what layer l+2 needs:
    # no more transfers than without it.
    wl = small_workload(n_layers=5, n_experts=8, top_k=2, slots=8, dtype="f32", tokens=3, res_a=1.0, res_b=0.0)
    res, ex, model = build(wl, gains="random")
    model.dvecs = np.zeros_like(model.dvecs)
    H, I = wl.hidden, wl.inter
    ex = ex.copy()
    ex[:, :, 2 * I * H:] = 0            # W_down of every expert
    model.experts = ex
    x0, _ = W.make_inputs(wl)
    adv = lambda t, l, r, out: r + out
    two = O.MoEOracle(model, O.MODE_SPECULATIVE, wl.slots, lookahead=2)
    one = O.MoEOracle(model, O.MODE_SPECULATIVE, wl.slots)
    O.run_tokens(two, x0, adv)
    O.run_tokens(one, x0, adv)
    assert two.stats.hits2 == two.stats.predictions2 == wl.top_k * (wl.n_layers - 2) * wl.tokens
    assert two.stats.cache_misses == one.stats.cache_misses
    # the same with the gain of layer l+1 in place of layer l+2's: no longer exact
    wrong = O.MoEOracle(model, O.MODE_SPECULATIVE, wl.slots, lookahead=2)
    good_q = O.quasi_hidden
    gains = model.rms_gain
    try:
        O.quasi_hidden = lambda r_, s_, d_, g_, eps, bf, fn=False: good_q(
            r_, s_, d_, gains[max(0, [np.array_equal(g_, gains[i]) for i in range(len(gains))].index(True) - 1)], eps, bf, fn)
        O.run_tokens(wrong, x0, adv)
    finally:
        O.quasi_hidden = good_q
    assert wrong.stats.hits2 < wrong.stats.predictions2
