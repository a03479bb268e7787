"""Pins for the CPU checker: each piece is tied to something other than itself -- a closed
form, a hand-worked value, brute force, an invariant, or a library routine used as an
independent reference -- so that a dropped term, a wrong index or a transposed operand fails."""
import itertools
import math

import numpy as np
import pytest
import torch

from oracle import moe_oracle as O


# ------------------------------------------------------------------ bf16 rounding / decoding
def test_bf16_round_matches_library_conversion_on_float32_inputs():
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(20000) * np.exp(rng.uniform(-20, 20, 20000))).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(O.bf16_round(x.astype(np.float64)), want)


def test_bf16_round_ties_to_even_and_rounds_once():
    assert O.bf16_round(1.0 + 2.0 ** -8) == 1.0                    # tie, even mantissa below
    assert O.bf16_round(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6    # tie, even mantissa above
    assert O.bf16_round(-(1.0 + 2.0 ** -8)) == -1.0
    # just above a tie: a float32 stop on the way would drop the 2^-40 and round down
    assert O.bf16_round(1.0 + 2.0 ** -8 + 2.0 ** -40) == 1.0 + 2.0 ** -7
    assert O.bf16_round(0.0) == 0.0
    assert O.bf16_round(255.5) == 256.0 and O.bf16_round(0.1) == 0.10009765625


def test_decode_weights_known_bit_patterns():
    w = np.array([0x3F80, 0xC000, 0x3E00, 0x0000, 0x4049], dtype=np.uint16)
    np.testing.assert_array_equal(O.decode_weights(w), [1.0, -2.0, 0.125, 0.0, 3.140625])
    f = np.array([1.5, -2.25], dtype=np.float32)
    np.testing.assert_array_equal(O.decode_weights(f), [1.5, -2.25])


# ------------------------------------------------------------------ RMSNorm
def test_rmsnorm_hand_value_and_invariants():
    got = O.rmsnorm([3.0, 4.0], [1.0, 2.0], 0.0)
    np.testing.assert_allclose(got, [3 / math.sqrt(12.5), 8 / math.sqrt(12.5)], rtol=1e-15)
    rng = np.random.default_rng(1)
    x = rng.standard_normal(257)
    y = O.rmsnorm(x, np.ones(257), 0.0)
    assert abs(np.sqrt(np.mean(y * y)) - 1.0) < 1e-14            # unit RMS with gain 1
    np.testing.assert_allclose(O.rmsnorm(7.5 * x, np.ones(257), 0.0), y, rtol=1e-14)   # scale free
    # eps enters under the root, next to the mean square
    np.testing.assert_allclose(O.rmsnorm([2.0], [1.0], 5.0), [2.0 / 3.0], rtol=1e-15)


def test_rmsnorm_matches_library():
    rng = np.random.default_rng(2)
    x, g = rng.standard_normal(300), rng.standard_normal(300)
    want = torch.nn.functional.rms_norm(torch.from_numpy(x), (300,), torch.from_numpy(g), 1e-6).numpy()
    np.testing.assert_allclose(O.rmsnorm(x, g, 1e-6), want, rtol=1e-13)


# ------------------------------------------------------------------ router GEMV
def test_router_logits_rowwise_dot_products_exact_sum():
    rng = np.random.default_rng(3)
    E, H = 5, 37                                            # not square: a transposed W cannot pass
    w = rng.standard_normal((E, H)).astype(np.float32)
    s = rng.standard_normal(H)
    want = [math.fsum(float(w[e, i]) * s[i] for i in range(H)) for e in range(E)]
    np.testing.assert_allclose(O.router_logits(w, s), want, rtol=1e-13)
    # bf16 storage is decoded, not reinterpreted
    wb = np.array([[0x3F80, 0x4000], [0xBF80, 0x0000]], dtype=np.uint16)     # [[1,2],[-1,0]]
    np.testing.assert_array_equal(O.router_logits(wb, [10.0, 1.0]), [12.0, -10.0])


# ------------------------------------------------------------------ top-k
@pytest.mark.parametrize("E,k", [(8, 2), (6, 3), (5, 5), (7, 1)])
def test_topk_is_the_max_sum_subset(E, k):
    rng = np.random.default_rng(E * 10 + k)
    for _ in range(20):
        z = rng.standard_normal(E)
        ids = O.topk_desc(z, k)
        best = max(itertools.combinations(range(E), k), key=lambda c: sum(z[list(c)]))
        assert set(ids.tolist()) == set(best)
        assert all(z[ids[i]] >= z[ids[i + 1]] for i in range(k - 1))       # descending order


def test_topk_ties_go_to_lower_index():
    z = np.array([1.0, 3.0, 3.0, 0.5, 3.0, 1.0])
    assert O.topk_desc(z, 2).tolist() == [1, 2]
    assert O.topk_desc(z, 4).tolist() == [1, 2, 4, 0]
    assert O.topk_desc(np.zeros(8), 3).tolist() == [0, 1, 2]


# ------------------------------------------------------------------ gates
def test_gates_sum_shift_equal_and_restricted_softmax():
    from scipy.special import softmax
    rng = np.random.default_rng(4)
    z = rng.standard_normal(16) * 3
    ids = O.topk_desc(z, 4)
    g = O.gates_of(z, ids)
    assert abs(g.sum() - 1.0) < 1e-15
    np.testing.assert_allclose(O.gates_of(z + 123.0, ids), g, rtol=1e-12)
    full = softmax(z)
    np.testing.assert_allclose(g, full[ids] / full[ids].sum(), rtol=1e-12)
    np.testing.assert_allclose(O.gates_of(np.full(8, -2.5), [1, 5, 6]), [1 / 3] * 3, rtol=1e-15)
    # the gate belongs to the expert in the same position of ids
    np.testing.assert_allclose(O.gates_of([0.0, math.log(3.0)], [1, 0]), [0.75, 0.25], rtol=1e-15)


# ------------------------------------------------------------------ default vector, quasi-hidden state
def test_layer_default_vector():
    dv = np.array([[1.0, 0.0, 2.0], [0.0, 1.0, -2.0], [5.0, 5.0, 5.0]], dtype=np.float32)
    np.testing.assert_allclose(O.layer_default_vector(dv, [2, 0], [0.25, 0.75]), [2.0, 1.25, 2.75])
    same = np.tile(np.array([[0.5, -1.5]], dtype=np.float32), (4, 1))
    np.testing.assert_allclose(O.layer_default_vector(same, [3, 1], [0.3, 0.7]), [0.5, -1.5], rtol=1e-15)
    np.testing.assert_array_equal(O.layer_default_vector(dv, [1], [1.0]), [0.0, 1.0, -2.0])


def test_quasi_hidden_definition():
    r = np.array([1.0, -2.0, 2.0])
    d = np.array([2.0, 2.0, -2.0])
    g_next = np.array([1.0, 2.0, 3.0])
    # r + d = [3, 0, 0]  ->  rms = sqrt(3)  ->  [sqrt(3), 0, 0] * gain
    np.testing.assert_allclose(O.quasi_hidden(r, None, d, g_next, 0.0, False), [math.sqrt(3), 0, 0], atol=1e-15)
    # d = 0 gives LN_{l+1}(r_l)
    np.testing.assert_allclose(O.quasi_hidden(r, None, 0 * d, g_next, 0.0, False),
                               r * g_next / math.sqrt(3.0), rtol=1e-15)
    # caption reading: the normalised s_l takes the place of r_l
    s = np.array([0.0, 1.0, 0.0])
    np.testing.assert_allclose(O.quasi_hidden(r, s, np.array([0.0, 0.0, 1.0]), np.ones(3), 0.0, False, True),
                               [0, math.sqrt(1.5), math.sqrt(1.5)], rtol=1e-15)
    # bf16 mode rounds q
    q = O.quasi_hidden(r, None, d, np.array([0.1, 1, 1]), 0.0, True)
    assert q[0] == O.bf16_round(0.1 * math.sqrt(3))


# ------------------------------------------------------------------ expert FFN
def test_expert_ffn_hand_value():
    y = O.expert_ffn(np.array([[1.0]], np.float32), np.array([[2.0]], np.float32),
                     np.array([[3.0]], np.float32), [1.0], False)
    np.testing.assert_allclose(y, [3.0 * 2.0 / (1.0 + math.exp(-1.0))], rtol=1e-15)


def test_expert_ffn_matches_library_swiglu():
    rng = np.random.default_rng(5)
    H, I = 24, 40
    wg, wu = (rng.standard_normal((I, H)).astype(np.float32) for _ in range(2))
    wd = rng.standard_normal((H, I)).astype(np.float32)
    s = rng.standard_normal(H)
    F = torch.nn.functional
    ts = torch.from_numpy(s)
    want = F.linear(F.silu(F.linear(ts, torch.from_numpy(wg).double())) * F.linear(ts, torch.from_numpy(wu).double()),
                    torch.from_numpy(wd).double()).numpy()
    np.testing.assert_allclose(O.expert_ffn(wg, wu, wd, s, False), want, rtol=1e-12)
    # swapping gate and up must not be the same thing
    assert np.abs(O.expert_ffn(wu, wg, wd, s, False) - want).max() > 1e-3


def test_expert_ffn_bf16_rounds_the_swiglu_product():
    wg = np.array([[0x3F80]], np.uint16)      # 1
    wu = np.array([[0x3F80]], np.uint16)      # 1
    wd = np.array([[0x3F80]], np.uint16)      # 1
    s = 1.5
    h = s / (1 + math.exp(-s)) * s
    assert O.expert_ffn(wg, wu, wd, [s], True)[0] == O.bf16_round(h)
    assert O.expert_ffn(wg, wu, wd, [s], True)[0] != h


# ------------------------------------------------------------------ cache simulator
def test_lru_hand_worked_sequence():
    p = O.LRUPool(2)
    assert p.request([1])[:2] == (0, 1)
    assert p.request([2])[:2] == (0, 1)
    assert p.request([1])[:2] == (1, 0)
    h, m, where = p.request([3])              # evicts 2, the least recently used
    assert (h, m) == (0, 1) and where[3] == 1
    assert p.request([2])[:2] == (0, 1)       # evicts 1 (stamp 3) rather than 3 (stamp 4)
    assert p.request([3])[:2] == (1, 0)
    assert sorted(p.slot_expert) == [2, 3]


def test_lru_never_evicts_a_member_of_the_request_and_fills_empty_slots_first():
    p = O.LRUPool(3)
    p.request([5, 6])
    assert p.slot_expert == [5, 6, -1]
    p.request([7])
    assert p.slot_expert == [5, 6, 7]                 # the empty slot, not an eviction
    h, m, _ = p.request([5, 8, 9])                    # 5 is the oldest but is requested: keep it
    assert (h, m) == (1, 2) and 5 in p.slot_expert and set(p.slot_expert) == {5, 8, 9}


def _textbook_lru(n_slots, experts):
    """The textbook cache for requests of ONE expert at a time (no ties to break): an ordered dictionary, a hit
    moves the key to the fresh end, a miss on a full cache drops the key at the stale end."""
    from collections import OrderedDict
    cache, log = OrderedDict(), []
    for e in experts:
        if e in cache:
            cache.move_to_end(e)
            log.append((1, 0))
        else:
            if len(cache) == n_slots:
                cache.popitem(last=False)
            cache[e] = True
            log.append((0, 1))
    return log


@pytest.mark.parametrize("S,E", [(2, 5), (4, 8), (16, 128)])
def test_lru_equals_the_textbook_cache_on_single_expert_requests(S, E):
    rng = np.random.default_rng(S + E)
    seq = rng.integers(0, E, size=600).tolist()
    p = O.LRUPool(S)
    assert [p.request([e])[:2] for e in seq] == _textbook_lru(S, seq)


def _lru_by_expert_records(n_slots, requests):
    """The policy restated around the experts instead of the slots: a record (time of last request, slot) per
    resident expert and a sorted list of free slots.  Whole sets are requested, so experts touched together share
    a time; a miss takes the lowest free slot, else evicts the resident expert outside the request with the
    oldest time (lowest slot among equally old ones)."""
    resident, free, log = {}, list(range(n_slots)), []
    for now, req in enumerate(requests, start=1):
        req = sorted(set(req))
        hits = [e for e in req if e in resident]
        for e in hits:
            resident[e] = (now, resident[e][1])
        misses = [e for e in req if e not in resident]
        for e in misses:
            if free:
                slot = free.pop(0)
            else:
                victim = min((x for x in resident if x not in req), key=lambda x: resident[x])
                slot = resident.pop(victim)[1]
            resident[e] = (now, slot)
        log.append((len(hits), len(misses)))
    return log


@pytest.mark.parametrize("S,E,qmax", [(4, 8, 2), (3, 8, 3), (8, 32, 8), (16, 128, 8)])
def test_lru_against_the_expert_record_restatement_on_random_requests(S, E, qmax):
    rng = np.random.default_rng(S * 100 + E)
    reqs = [rng.choice(E, size=rng.integers(1, qmax + 1), replace=False).tolist() for _ in range(400)]
    p = O.LRUPool(S)
    got = [p.request(r)[:2] for r in reqs]
    assert got == _lru_by_expert_records(S, reqs)


def test_lru_pool_as_large_as_the_expert_set_misses_each_expert_once():
    rng = np.random.default_rng(9)
    p = O.LRUPool(8)
    misses = sum(p.request(rng.choice(8, size=2, replace=False).tolist())[1] for _ in range(200))
    assert misses == 8


def test_chunks_of():
    assert O.chunks_of([1, 2, 3, 4, 5], 2) == [[1, 2], [3, 4], [5]]
    assert O.chunks_of([1, 2], 4) == [[1, 2]]


# ------------------------------------------------------------------ estimator forward
def test_layernorm_hand_value_and_library():
    np.testing.assert_allclose(O.layernorm([1.0, 3.0], [2.0, 1.0], [0.5, -1.0], 0.0), [-1.5, 0.0], rtol=1e-15)
    rng = np.random.default_rng(6)
    x, g, b = rng.standard_normal(70), rng.standard_normal(70), rng.standard_normal(70)
    want = torch.nn.functional.layer_norm(torch.from_numpy(x), (70,), torch.from_numpy(g), torch.from_numpy(b), 1e-5).numpy()
    np.testing.assert_allclose(O.layernorm(x, g, b, 1e-5), want, rtol=1e-12, atol=1e-14)


def _random_estimator(rng, H, dm, F, E, L):
    f = lambda *s: rng.standard_normal(s).astype(np.float32)
    return O.Estimator(proj=f(dm, H), layer_emb=f(L, dm), ffn_in=f(F, dm), ffn_out=f(dm, F),
                       ln_gain=f(dm), ln_bias=f(dm), head=f(E, dm))


def test_estimator_forward_matches_library_modules():
    rng = np.random.default_rng(7)
    H, dm, F, E, L = 24, 6, 18, 10, 3
    est = _random_estimator(rng, H, dm, F, E, L)
    q = rng.standard_normal(H)
    Fn = torch.nn.functional
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    for layer in range(L):
        u = Fn.linear(t(q), t(est.proj)) + t(est.layer_emb[layer])
        v = u + Fn.linear(Fn.silu(Fn.linear(u, t(est.ffn_in))), t(est.ffn_out))
        w = Fn.layer_norm(v, (dm,), t(est.ln_gain), t(est.ln_bias), est.ln_eps)
        np.testing.assert_allclose(O.estimator_logits(est, q, layer), Fn.linear(w, t(est.head)).numpy(), rtol=1e-11, atol=1e-13)
    # the layer embedding matters, and so does the residual connection
    assert np.abs(O.estimator_logits(est, q, 0) - O.estimator_logits(est, q, 1)).max() > 1e-3


def test_estimator_special_cases():
    rng = np.random.default_rng(8)
    H, dm, F, E, L = 8, 4, 8, 4, 2
    est = _random_estimator(rng, H, dm, F, E, L)
    est.ffn_out[:] = 0                                     # dead feed-forward branch: only the residual path is left
    est.head = np.eye(E, dm, dtype=np.float32)             # logits = LayerNorm output
    est.ln_gain[:] = 1
    est.ln_bias[:] = 0
    q = rng.standard_normal(H)
    u = est.proj.astype(np.float64) @ q + est.layer_emb[1]
    want = (u - u.mean()) / np.sqrt(u.var() + est.ln_eps)
    np.testing.assert_allclose(O.estimator_logits(est, q, 1), want, rtol=1e-12)


# --------------------------------------------------------------------------------------
# Analytic decode-time model (Sec. 5.1)
# --------------------------------------------------------------------------------------
def _golden_tpot_cases():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "tpot_model.txt")
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, comp, copy, t_ond, t_pf, delta = [f.strip() for f in line.split("|")]
        yield (name, [float(x) for x in comp.split()], [float(x) for x in copy.split()],
               float(t_ond), float(t_pf), float(delta))


def test_tpot_model_matches_the_stated_cases():
    cases = list(_golden_tpot_cases())
    assert len(cases) >= 4
    for name, comp, copy, t_ond, t_pf, delta in cases:
        got = O.tpot_model(comp, copy)
        np.testing.assert_allclose(got, (t_ond, t_pf, delta), rtol=1e-12, err_msg=name)


def test_tpot_model_invariants():
    rng = np.random.default_rng(5)
    for _ in range(50):
        L = int(rng.integers(1, 40))
        comp, copy = rng.random(L) * 3, rng.random(L) * 3
        t_ond, t_pf, delta = O.tpot_model(comp, copy)
        assert abs((t_ond - t_pf) - delta) < 1e-9            # what prefetching saves is the improvement
        assert delta <= min(comp.sum(), copy.sum()) + 1e-12   # bounded by total compute and by total copy
        assert t_ond / t_pf <= 2.0 + 1e-12                    # the 2x ceiling of Sec. 5.1
        # brute force, layer by layer
        assert abs(t_pf - sum(max(a, b) for a, b in zip(comp, copy))) < 1e-9
    t_ond, t_pf, _ = O.tpot_model([2.0] * 7, [2.0] * 7)
    assert t_ond / t_pf == 2.0


# --------------------------------------------------------------------------------------
# Expert block size against the paper's model table
# --------------------------------------------------------------------------------------
def test_expert_block_size_reproduces_the_papers_expert_memory():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "model_config.txt")
    rows = [[f.strip() for f in line.split("|")] for line in open(path) if line.strip() and not line.startswith("#")]
    assert len(rows) == 2
    empty = np.zeros((0,))
    for name, L, E, H, I, printed_gb in rows:
        model = O.OracleModel(n_layers=int(L), hidden=int(H), n_experts=int(E), top_k=8, inter=int(I), dtype=O.DTYPE_BF16,
                              router_w=empty, rms_gain=empty, dvecs=empty, experts=empty)
        total_gib = model.expert_bytes * int(L) * int(E) / 2 ** 30
        assert abs(total_gib - float(printed_gb)) <= 1.0, (name, total_gib)
    # the benchmark workload has the first row's shapes, and the library's block size is the same number
    from paper_2603_19289_amd import workload as W
    wl = W.CONFIGS["c2_qwen3_30b_a3b"]
    assert (wl.n_layers, wl.n_experts, wl.hidden, wl.inter) == (48, 128, 2048, 768)
    assert wl.expert_bytes == 3 * 2048 * 768 * 2
