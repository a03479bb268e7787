"""CPU oracle for the decode-time MoE layer step with speculative expert prefetch.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain, fp64 statement of what the
method computes, written from the paper.  Only the tests, the smoke check and the
benchmark's cpu-baseline leg may import it.  It shares no code with the HIP library and
never imports the GPU package; the product path never routes through it.

Everything here is numpy in float64.  Each function names the passage of the paper
(section / equation / algorithm) it follows.  Where the paper is silent the reading taken
is written next to the code and listed again in the design notes of the repository.

Parity status: every function below is pinned by tests that do not go through this module's
own arithmetic (closed forms, brute force, invariants, library routines used as independent
references).  Real-model hit rates and accuracy are "parity unpinned": they need trained
weights and datasets that are not available.

Notation (paper, Sec. 3 and Sec. 5.1): L layers, E experts per layer, k experts per token,
H hidden size, I expert intermediate size, B decode batch, S device cache slots per layer,
r_l post-attention residual, s_l = LN_l(r_l) router input, d_{l,e} per-expert default
vector, d_l layer-level default vector, q_l quasi-hidden state.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

MODE_ON_DEMAND = 0
MODE_SPECULATIVE = 1
MODE_PREFETCH_HINT = 2

DTYPE_F32 = 0
DTYPE_BF16 = 1


# --------------------------------------------------------------------------------------
# Number formats
# --------------------------------------------------------------------------------------

def bf16_round(x):
    """Round float64 values to the nearest bfloat16 (8 significant bits), ties to even.

    The paper runs every evaluation in bf16 (Sec. 5.1.1, "Models") and says nothing finer,
    so the rounding points are a reading: activations that feed a matrix product (s_l, q_l
    and the SwiGLU product) are rounded to bf16 first, exactly as a bf16 engine would hold
    them.  The rounding is done straight from the float64 value (no float32 stop on the way,
    which could round twice).  Domain: finite values whose magnitude is a normal bf16
    number or zero; the workloads here are O(1).
    """
    x = np.asarray(x, dtype=np.float64)
    m, e = np.frexp(x)                 # x = m * 2**e with 0.5 <= |m| < 1
    return np.ldexp(np.rint(m * 256.0), e - 8)   # np.rint rounds halves to even


def decode_weights(w):
    """Stored weights -> float64.  uint16 arrays hold bf16 bit patterns; float arrays pass."""
    w = np.asarray(w)
    if w.dtype == np.uint16:
        return (w.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return w.astype(np.float64)


# --------------------------------------------------------------------------------------
# The pieces of one layer (one token row)
# --------------------------------------------------------------------------------------

def rmsnorm(x, gamma, eps):
    """LN(.) of Sec. 3.2 read as RMSNorm with gain (pre-norm MoE blocks): x*gamma/sqrt(mean(x^2)+eps).

    The paper only writes "LN"; the models it evaluates normalise with RMSNorm (no mean
    subtraction, no bias), and eps is not given: it is a parameter here.
    """
    x = np.asarray(x, dtype=np.float64)
    ms = np.sum(x * x) / x.shape[-1]
    return x * np.asarray(gamma, dtype=np.float64) / np.sqrt(ms + eps)


def router_logits(w_router, s):
    """Gate_l(X) of Algorithm 1: z_e = sum_i W[e, i] * s[i]; W is [E, H] row-major."""
    return decode_weights(w_router) @ np.asarray(s, dtype=np.float64)


def topk_desc(z, k):
    """TopK of Algorithm 1: the k largest logits, reported by descending logit.

    Ties (not addressed by the paper) go to the lower expert index.
    """
    z = np.asarray(z, dtype=np.float64)
    order = sorted(range(z.shape[0]), key=lambda e: (-z[e], e))
    return np.array(order[:k], dtype=np.int64)


def gates_of(z, ids):
    """Mixing weights G_l: softmax over the k selected logits only (they sum to one).

    Identical, in exact arithmetic, to a softmax over all experts followed by keeping the
    top-k and renormalising; the paper does not say which its engine does.
    """
    zs = np.asarray(z, dtype=np.float64)[np.asarray(ids)]
    p = np.exp(zs - np.max(zs))
    return p / np.sum(p)


def layer_default_vector(dvecs_l, ids, gates):
    """Sec. 3.1 display equation: d_l = sum over the selected experts of g_{l,e} * d_{l,e}."""
    d = decode_weights(dvecs_l)
    out = np.zeros(d.shape[1], dtype=np.float64)
    for e, g in zip(ids, gates):
        out += g * d[int(e)]
    return out


def quasi_hidden(r, s, d, gamma_next, eps, bf16, from_normalized=False):
    """Sec. 3.2 display equation: q_l = LN_{l+1}(d_l + r_l).

    `from_normalized=True` takes the reading of the caption of Fig. 1 instead (the
    normalised s_l in place of r_l); the equation is the default.
    """
    u = (np.asarray(s, dtype=np.float64) if from_normalized else np.asarray(r, dtype=np.float64)) + d
    q = rmsnorm(u, gamma_next, eps)
    return bf16_round(q) if bf16 else q


def silu(a):
    return a / (1.0 + np.exp(-a))


def expert_ffn(w_gate, w_up, w_down, s, bf16):
    """MoE_l's per-expert FFN (Algorithm 1, last line), read as plain SwiGLU without bias:
    y = W_down ( silu(W_gate s) * (W_up s) ).  W_gate, W_up are [I, H]; W_down is [H, I].
    In bf16 mode the SwiGLU product is rounded to bf16 before the down projection.
    """
    s = np.asarray(s, dtype=np.float64)
    a = decode_weights(w_gate) @ s
    c = decode_weights(w_up) @ s
    h = silu(a) * c
    if bf16:
        h = bf16_round(h)
    return decode_weights(w_down) @ h


# --------------------------------------------------------------------------------------
# Neural expert estimator (forward pass only)
# --------------------------------------------------------------------------------------

@dataclass
class Estimator:
    """Weights of the estimator of Sec. 6 / Appendix A, every matrix stored [out, in] row-major in the
    model's weight dtype: proj [dm, H] (the paper's A, transposed storage), layer_emb [L, dm],
    ffn_in [F, dm] (B), ffn_out [dm, F] (C), head [E, dm] (W_head); LayerNorm gain and bias [dm]
    float.  dm = H/m, F = n*dm.  Only the forward pass exists here: training needs real activations."""
    proj: np.ndarray
    layer_emb: np.ndarray
    ffn_in: np.ndarray
    ffn_out: np.ndarray
    ln_gain: np.ndarray
    ln_bias: np.ndarray
    head: np.ndarray
    ln_eps: float = 1e-5


def layernorm(x, gain, bias, eps):
    """Standard LayerNorm: (x - mean) / sqrt(biased variance + eps) * gain + bias."""
    x = np.asarray(x, dtype=np.float64)
    mu = np.sum(x) / x.shape[-1]
    var = np.sum((x - mu) * (x - mu)) / x.shape[-1]
    return (x - mu) / np.sqrt(var + eps) * np.asarray(gain, dtype=np.float64) + np.asarray(bias, dtype=np.float64)


def estimator_logits(est: Estimator, q, layer: int):
    """Appendix A, in its order: project q_l to the latent size, add the embedding of layer l, feed
    forward (linear, SiLU, linear) with a residual connection over it, LayerNorm, linear head to E
    logits for layer l+1.  No rounding inside (the paper fixes none); weights as stored."""
    u = decode_weights(est.proj) @ np.asarray(q, dtype=np.float64) + decode_weights(est.layer_emb[layer])
    t = silu(decode_weights(est.ffn_in) @ u)
    v = u + decode_weights(est.ffn_out) @ t
    w = layernorm(v, est.ln_gain, est.ln_bias, est.ln_eps)
    return decode_weights(est.head) @ w


# --------------------------------------------------------------------------------------
# Device expert cache, simulated (integers only)
# --------------------------------------------------------------------------------------

class LRUPool:
    """One layer's pool of S expert slots with least-recently-used replacement.

    The paper's engine keeps no cache across tokens (double buffers, Sec. 5.1
    "Implementation Details"); the capped slot cache and its policy come from the workload
    definition.  Rule: a logical clock ticks once per request.  A request is a set Q of at
    most S experts, visited by ascending expert id.  A resident expert is a hit and is
    stamped with the clock.  Each missing expert takes the slot with the smallest stamp
    among slots that hold no member of Q (empty slots have stamp -1; ties go to the lowest
    slot index), and is stamped with the clock.
    """

    def __init__(self, n_slots: int):
        self.slot_expert = [-1] * n_slots
        self.slot_stamp = [-1] * n_slots
        self.clock = 0

    def request(self, experts: Sequence[int]) -> Tuple[int, int, Dict[int, int]]:
        q = sorted(set(int(e) for e in experts))
        if len(q) > len(self.slot_expert):
            raise ValueError("request larger than the pool")
        self.clock += 1
        hits = misses = 0
        where: Dict[int, int] = {}
        for e in q:
            if e in self.slot_expert:
                s = self.slot_expert.index(e)
                self.slot_stamp[s] = self.clock
                where[e] = s
                hits += 1
        for e in q:
            if e in where:
                continue
            cand = [s for s in range(len(self.slot_expert)) if self.slot_expert[s] not in q]
            s = min(cand, key=lambda t: (self.slot_stamp[t], t))
            self.slot_expert[s] = e
            self.slot_stamp[s] = self.clock
            where[e] = s
            misses += 1
        return hits, misses, where


def chunks_of(q_sorted: Sequence[int], n: int) -> List[List[int]]:
    """Split an ascending expert list into consecutive waves of at most n experts."""
    q = list(q_sorted)
    return [q[i:i + n] for i in range(0, len(q), n)]


# --------------------------------------------------------------------------------------
# Model, state and the layer step (Algorithm 1)
# --------------------------------------------------------------------------------------

@dataclass
class OracleModel:
    """Weights as stored (bf16 bit patterns in uint16, or float32), never modified.

    router_w [L, E, H]; rms_gain [L, H] float; dvecs [L, E, H];
    experts [L, E, 3*H*I] laid out per expert as W_gate [I,H] | W_up [I,H] | W_down [H,I].
    """
    n_layers: int
    hidden: int
    n_experts: int
    top_k: int
    inter: int
    dtype: int
    router_w: np.ndarray
    rms_gain: np.ndarray
    dvecs: np.ndarray
    experts: np.ndarray
    rms_eps: float = 1e-6

    def expert_mats(self, layer: int, e: int):
        H, I = self.hidden, self.inter
        blk = self.experts[layer, e]
        return (blk[:I * H].reshape(I, H), blk[I * H:2 * I * H].reshape(I, H),
                blk[2 * I * H:].reshape(H, I))

    @property
    def expert_bytes(self) -> int:
        return 3 * self.hidden * self.inter * (2 if self.dtype == DTYPE_BF16 else 4)


@dataclass
class OracleStats:
    tokens: int = 0
    layer_steps: int = 0
    predictions: int = 0
    hits: int = 0
    cache_hits: int = 0
    cache_misses: int = 0
    h2d_bytes: int = 0
    cache_waves: int = 0       # chunks of at most S experts the executed unions were split into (one expert pass each)
    predictions2: int = 0      # two-layer lookahead: predictions made two layers ahead, scored like the others
    hits2: int = 0


@dataclass
class LayerDiagnostics:
    """Statistics of the predictions made FOR one layer (at the layer before it), as in the
    paper's per-layer figures: recall@k (Fig. 3), agreement per routing-weight rank (Fig. 4) and
    cosine similarity between the predicting signal and the true router input (Fig. 2)."""
    predictions: int = 0
    hits: int = 0
    rank_match: Optional[List[int]] = None
    cos_sum: float = 0.0
    cos_count: int = 0


@dataclass
class StepResult:
    out: np.ndarray            # [B, H] float64: O_l
    true_ids: np.ndarray       # [B, k] by descending logit
    true_gates: np.ndarray     # [B, k]
    exec_ids: np.ndarray       # [B, k] what was executed
    exec_gates: np.ndarray     # [B, k]
    next_ids: Optional[np.ndarray]    # [B, k] prediction for layer l+1, or None
    next_gates: Optional[np.ndarray]
    true_margin: np.ndarray    # [B] logit_(k) - logit_(k+1) of the true router (inf if k == E)
    next_margin: Optional[np.ndarray]
    s: np.ndarray              # [B, H] router input actually used
    q: Optional[np.ndarray]    # [B, H] quasi-hidden state fed to layer l+1's router, or None


def _margin(z, k):
    zs = np.sort(np.asarray(z, dtype=np.float64))[::-1]
    return float(zs[k - 1] - zs[k]) if k < zs.shape[0] else float("inf")


class MoEOracle:
    """Algorithm 1 (MoE block with expert prefetch, decode) in both execution modes.

    mode = MODE_ON_DEMAND: route, make the routed experts resident (blocking), execute them
    (the baseline of Sec. 5.1).  mode = MODE_SPECULATIVE: layer 0 is a cold start (route, blocking
    load); every later layer executes the experts *and mixing weights* predicted one layer
    earlier from the quasi-hidden state, and never re-fetches the true ones (Sec. 4).
    mode = MODE_PREFETCH_HINT: the policy of prior work that the paper argues against (Sec. 2,
    Sec. 4): the prediction is only a cache hint -- the predicted experts are prefetched, but the
    true router-selected experts are executed and whatever the prefetch missed is loaded on demand.

    The true router runs at every layer in both modes: d_l is built from what "the router
    selects" at layer l (Sec. 3.1), and GetNextExperts is handed a fresh Gate_l(X).
    """

    def __init__(self, model: OracleModel, mode: int, slots_per_layer: int,
                 q_from_normalized: bool = False, predict: bool = True, predict_signal: int = 0,
                 estimator: Optional[Estimator] = None, estimator_layers: Optional[Sequence[int]] = None,
                 lookahead: int = 1):
        if slots_per_layer < model.top_k:
            raise ValueError("need at least k slots per layer")
        self.m = model
        self.mode = mode
        self.S = slots_per_layer
        self.q_from_normalized = q_from_normalized
        self.predict = predict or mode in (MODE_SPECULATIVE, MODE_PREFETCH_HINT)
        self.bf16 = model.dtype == DTYPE_BF16
        self.pools = [LRUPool(slots_per_layer) for _ in range(model.n_layers)]
        self.stats = OracleStats()
        self.pending: Optional[Tuple[np.ndarray, np.ndarray]] = None
        self.pending_signal: Optional[np.ndarray] = None
        self.next_layer = 0
        # 0: predict with the quasi-hidden state q_l; 1: with s_l, the baseline signal of Sec. 3.3
        # (layer l+1's router applied to the normalised residual of layer l as it is)
        self.predict_signal = predict_signal
        # Est-PF / Hybrid-PF of Sec. 6: at the layers named here the prediction for layer l+1 comes from
        # the estimator's logits instead of layer l+1's router (all layers: Est-PF; some: Hybrid-PF)
        # offline statistic of Sec. 3.1: running sum and count of the un-gated outputs of every executed
        # expert; the per-expert default vector d_{l,e} is their mean (read it with default_vectors())
        self.dacc_sum = np.zeros((model.n_layers, model.n_experts, model.hidden))
        self.dacc_cnt = np.zeros((model.n_layers, model.n_experts), dtype=np.int64)
        self.estimator = estimator
        self.estimator_layers = set(estimator_layers or []) if estimator is not None else set()
        self.diag = [LayerDiagnostics(rank_match=[0] * model.top_k) for _ in range(model.n_layers)]
        # Multi-layer prefetching with the expert cache (the paper's Future Work names it and gives no
        # algorithm; this is a reading).  lookahead = 2: at layer l, besides the prediction for layer l+1,
        # layer l+2's router is applied to the same quasi-hidden vector normalised with layer l+2's gain,
        # q2_l = LN_{l+2}(r_l + d_l), and the predicted experts are requested into layer l+2's pool as a cache
        # hint, one layer earlier than the regular prefetch.  Nothing else changes: layer l+2 still executes
        # what layer l+1 predicts for it, so outputs equal those of lookahead = 1; only the cache traffic and
        # its timing differ.  Prefetching modes only.
        if lookahead not in (1, 2):
            raise ValueError("lookahead must be 1 or 2")
        self.lookahead = lookahead if mode in (MODE_SPECULATIVE, MODE_PREFETCH_HINT) else 1
        self.pending2: Dict[int, np.ndarray] = {}      # layer -> ids predicted for it two layers earlier

    # -- cache bookkeeping ---------------------------------------------------------
    def _request(self, layer: int, experts: Sequence[int]):
        h, m, _ = self.pools[layer].request(experts)
        self.stats.cache_hits += h
        self.stats.cache_misses += m
        self.stats.h2d_bytes += m * self.m.expert_bytes

    def begin_token(self):
        """A new decode step: no prediction is carried into layer 0 (cold start)."""
        self.pending = None
        self.pending_signal = None
        self.pending2 = {}
        self.next_layer = 0
        self.stats.tokens += 1

    def route(self, layer: int, x):
        """Router + top-k + gates for one already normalised row x (s_l, or q_{l-1} for a prediction)."""
        m = self.m
        z = router_logits(m.router_w[layer], x)
        ids = topk_desc(z, m.top_k)
        return ids, gates_of(z, ids), _margin(z, m.top_k)

    def default_vectors(self, layer: int):
        """Mean un-gated output per expert over the steps that executed it (zero where never executed)."""
        return self.dacc_sum[layer] / np.maximum(self.dacc_cnt[layer], 1)[:, None]

    def prefill_layer_step(self, layer: int, r) -> StepResult:
        """Prefill (Sec. 5.2): all prompt tokens at once.  Nothing is predicted: with enough tokens every
        expert is active, so every expert of the layer is loaded (streamed one layer ahead) and the true
        router-selected experts are executed, i.e. the standard MoE block.  Traffic: E experts per layer.
        The layer's pool is left empty for the decode cache."""
        m = self.m
        r = np.asarray(r, dtype=np.float64)
        P, k = r.shape[0], m.top_k
        out = np.zeros((P, m.hidden))
        s = np.zeros((P, m.hidden))
        ids = np.zeros((P, k), dtype=np.int64)
        g = np.zeros((P, k))
        margin = np.zeros(P)
        for b in range(P):
            sb = rmsnorm(r[b], m.rms_gain[layer], m.rms_eps)
            s[b] = bf16_round(sb) if self.bf16 else sb
            ids[b], g[b], margin[b] = self.route(layer, s[b])
        y = np.zeros((P, k, m.hidden))
        for e in range(m.n_experts):              # expert by expert, so that each is decoded once
            where = np.argwhere(ids == e)
            if len(where):
                mats = m.expert_mats(layer, e)
                for b, j in where:
                    y[b, j] = expert_ffn(*mats, s[b], self.bf16)
                    self.dacc_sum[layer, e] += y[b, j]        # statistic behind the default vectors (Sec. 3.1)
                    self.dacc_cnt[layer, e] += 1
        for b in range(P):
            for j in range(k):
                out[b] += g[b, j] * y[b, j]
        self.pools[layer] = LRUPool(self.S)
        self.stats.cache_misses += m.n_experts
        self.stats.h2d_bytes += m.n_experts * m.expert_bytes
        self.stats.layer_steps += 1
        return StepResult(out, ids, g, ids.copy(), g.copy(), None, None, margin, None, s, None)

    def layer_step(self, layer: int, r) -> StepResult:
        m = self.m
        if layer != self.next_layer:
            raise RuntimeError("layers must be stepped in order after begin_token")
        r = np.asarray(r, dtype=np.float64)
        B, H, k = r.shape[0], m.hidden, m.top_k
        last = layer == m.n_layers - 1

        s = np.zeros((B, H))
        t_ids = np.zeros((B, k), dtype=np.int64)
        t_g = np.zeros((B, k))
        t_margin = np.zeros(B)
        for b in range(B):
            sb = rmsnorm(r[b], m.rms_gain[layer], m.rms_eps)
            s[b] = bf16_round(sb) if self.bf16 else sb
            t_ids[b], t_g[b], t_margin[b] = self.route(layer, s[b])

        # recall@k of the prediction made one layer earlier (Sec. 3.3)
        if self.pending is not None:
            dg = self.diag[layer]
            for b in range(B):
                h = len(set(self.pending[0][b].tolist()) & set(t_ids[b].tolist()))
                self.stats.hits += h
                self.stats.predictions += k
                dg.hits += h
                dg.predictions += k
                for j in range(k):                      # same expert at the same routing-weight rank
                    dg.rank_match[j] += int(self.pending[0][b, j] == t_ids[b, j])
                sig = self.pending_signal[b]
                dg.cos_sum += float(np.dot(sig, s[b]) / np.sqrt(np.dot(sig, sig) * np.dot(s[b], s[b])))
                dg.cos_count += 1

        # recall@k of the prediction made two layers earlier (lookahead = 2)
        if layer in self.pending2:
            ids2 = self.pending2.pop(layer)
            for b in range(B):
                self.stats.hits2 += len(set(ids2[b].tolist()) & set(t_ids[b].tolist()))
                self.stats.predictions2 += k

        # which experts run, with which mixing weights (Algorithm 1, the if/else at the top)
        if self.mode == MODE_SPECULATIVE and self.pending is not None:
            x_ids, x_g = self.pending
        else:
            x_ids, x_g = t_ids, t_g

        # GetNextExperts: d_l from the TRUE routing of layer l, q_l, then layer l+1's router
        n_ids = n_g = n_margin = q_all = None
        if not last and self.predict:
            q_all = np.zeros((B, H))
            n_ids = np.zeros((B, k), dtype=np.int64)
            n_g = np.zeros((B, k))
            n_margin = np.zeros(B)
            for b in range(B):
                if self.predict_signal == 1:
                    q = s[b]
                else:
                    d = layer_default_vector(m.dvecs[layer], t_ids[b], t_g[b])
                    q = quasi_hidden(r[b], s[b], d, m.rms_gain[layer + 1], m.rms_eps, self.bf16,
                                     self.q_from_normalized)
                q_all[b] = q
                if layer in self.estimator_layers:
                    z = estimator_logits(self.estimator, q, layer)
                    n_ids[b] = topk_desc(z, k)
                    n_g[b], n_margin[b] = gates_of(z, n_ids[b]), _margin(z, k)
                else:
                    n_ids[b], n_g[b], n_margin[b] = self.route(layer + 1, q)

        # cache traffic: what has to be resident, in waves of at most S experts
        exec_union = sorted(set(x_ids.reshape(-1).tolist()))
        waves = chunks_of(exec_union, self.S)
        self.stats.cache_waves += len(waves)
        prefetched = self.mode == MODE_SPECULATIVE and self.pending is not None
        for w, wave in enumerate(waves):
            if prefetched and w == 0:
                continue          # requested during the previous layer step
            self._request(layer, wave)
        if self.mode in (MODE_SPECULATIVE, MODE_PREFETCH_HINT) and n_ids is not None:
            nxt = chunks_of(sorted(set(n_ids.reshape(-1).tolist())), self.S)
            self._request(layer + 1, nxt[0])
            if self.lookahead == 2 and layer + 2 < m.n_layers:
                ids2 = np.zeros((B, k), dtype=np.int64)
                for b in range(B):
                    d = layer_default_vector(m.dvecs[layer], t_ids[b], t_g[b])
                    q2 = quasi_hidden(r[b], s[b], d, m.rms_gain[layer + 2], m.rms_eps, self.bf16, self.q_from_normalized)
                    ids2[b], _, _ = self.route(layer + 2, q2)
                self.pending2[layer + 2] = ids2
                self._request(layer + 2, chunks_of(sorted(set(ids2.reshape(-1).tolist())), self.S)[0])

        # experts and the gate-weighted combine
        out = np.zeros((B, H))
        for b in range(B):
            for j in range(k):
                wg, wu, wd = m.expert_mats(layer, int(x_ids[b, j]))
                y = expert_ffn(wg, wu, wd, s[b], self.bf16)
                out[b] += x_g[b, j] * y
                self.dacc_sum[layer, int(x_ids[b, j])] += y
                self.dacc_cnt[layer, int(x_ids[b, j])] += 1

        self.pending = None if n_ids is None else (n_ids, n_g)
        self.pending_signal = q_all
        self.next_layer = layer + 1
        self.stats.layer_steps += 1
        return StepResult(out, t_ids, t_g, np.array(x_ids), np.array(x_g), n_ids, n_g,
                          t_margin, n_margin, s, q_all)


def tpot_model(t_compute, t_copy):
    """Analytic decode-time model of Sec. 5.1: per-layer compute times (attention + routing + expert
    FFN) and per-layer expert-copy times give
        T_ond = sum_l (t_compute_l + t_copy_l)          on-demand loading, copies on the critical path
        T_pf  = sum_l max(t_compute_l, t_copy_l)        prefetching, copy overlapped with compute
        dT    = sum_l min(t_copy_l, t_compute_l)        the equation labelled "improvement"
    under the paper's assumption that consecutive layers copy the same amount (the copy that
    overlaps layer l's compute is the one for layer l+1).  Returns (T_ond, T_pf, dT)."""
    t_compute = np.asarray(t_compute, dtype=np.float64)
    t_copy = np.asarray(t_copy, dtype=np.float64)
    t_ond = float(np.sum(t_compute + t_copy))
    t_pf = float(np.sum(np.maximum(t_compute, t_copy)))
    delta = float(np.sum(np.minimum(t_copy, t_compute)))
    return t_ond, t_pf, delta


def run_tokens(oracle: MoEOracle, x0, advance, n_layers: Optional[int] = None):
    """Drive the oracle over decode steps.  x0 is [T, B, H]; `advance(t, l, r, O)` is the
    caller's residual update (the stand-in for everything between two MoE blocks) and
    returns r_{l+1}.  Returns, per token, the list of (r_l, StepResult)."""
    L = oracle.m.n_layers if n_layers is None else n_layers
    trace = []
    for t in range(x0.shape[0]):
        oracle.begin_token()
        r = np.asarray(x0[t], dtype=np.float64)
        per_layer = []
        for l in range(L):
            res = oracle.layer_step(l, r)
            per_layer.append((r, res))
            if l + 1 < L:
                r = advance(t, l, r, res.out)
        trace.append(per_layer)
    return trace
