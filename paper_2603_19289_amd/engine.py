"""Plumbing around the C ABI for tests, the smoke check and the benchmark: device memory and
streams come from PyTorch, everything else is a call into libmoe_spec.so."""
from __future__ import annotations

import ctypes as C
from typing import Dict, Optional

import numpy as np
import torch

from . import moe_spec as M


def _np_to_torch_storage(a: np.ndarray) -> torch.Tensor:
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16)
    return torch.from_numpy(a)


class Engine:
    """Owns a context plus the torch tensors it borrows (arena, resident tables, host pool)."""

    def __init__(self, *, n_layers, hidden, n_experts, top_k, inter, dtype, max_batch, slots, mode,
                 resident: Dict[str, np.ndarray], experts, rms_eps=1e-6, q_from_normalized=0,
                 predict_in_on_demand=1, profile=0, copy_engine=M.COPY_KERNEL, predict_signal=0, diagnostics=0, accumulate_defaults=0, estimator=None,
                 estimator_layers=None, max_prefill_tokens=0, wait_spin_limit=0, lookahead=0, device="cuda:0"):
        self.dev = torch.device(device)
        self.L, self.H, self.E, self.k, self.I = n_layers, hidden, n_experts, top_k, inter
        self.max_batch = max_batch
        self.compute = torch.cuda.Stream(device=self.dev)
        self.copy = torch.cuda.Stream(device=self.dev)
        cfg = M.Config(n_layers=n_layers, hidden=hidden, n_experts=n_experts, top_k=top_k, inter=inter,
                       max_batch=max_batch, slots_per_layer=slots,
                       dtype=M.BF16 if dtype == "bf16" else M.F32, mode=mode, rms_eps=rms_eps,
                       q_from_normalized=q_from_normalized, predict_in_on_demand=predict_in_on_demand,
                       profile=profile, copy_engine=copy_engine, predict_signal=predict_signal,
                       diagnostics=diagnostics, accumulate_defaults=accumulate_defaults,
                       max_prefill_tokens=max_prefill_tokens, wait_spin_limit=wait_spin_limit, lookahead=lookahead,
                       est_latent=0 if estimator is None else estimator["proj"].shape[0],
                       est_ffn=0 if estimator is None else estimator["ffn_in"].shape[0])
        need = M.moe_spec_arena_bytes(cfg)
        if need == 0:
            raise ValueError("invalid configuration")
        self.arena = torch.empty(need, dtype=torch.uint8, device=self.dev)
        cfg.device_arena = self.arena.data_ptr()
        cfg.device_arena_bytes = need
        cfg.compute_stream = self.compute.cuda_stream
        cfg.copy_stream = self.copy.cuda_stream
        self.cfg = cfg
        self.expert_bytes = M.moe_spec_expert_bytes(cfg)
        self.ctx = M.moe_spec_create(cfg)

        # resident tables
        self.router_w = _np_to_torch_storage(resident["router_w"]).to(self.dev)
        self.rms_gain = torch.from_numpy(np.ascontiguousarray(resident["rms_gain"], dtype=np.float32)).to(self.dev)
        self.dvecs = _np_to_torch_storage(resident["dvecs"]).to(self.dev)
        for l in range(n_layers):
            M.moe_spec_set_layer_resident(self.ctx, l, self.router_w[l].data_ptr(), self.rms_gain[l].data_ptr(),
                                          self.dvecs[l].data_ptr())
        if estimator is not None:
            self.est = {k: (torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32)) if k.startswith("ln_")
                            else _np_to_torch_storage(v)).to(self.dev) for k, v in estimator.items()}
            M.moe_spec_set_estimator(self.ctx, *(self.est[k].data_ptr() for k in
                                                 ("proj", "layer_emb", "ffn_in", "ffn_out", "ln_gain", "ln_bias", "head")),
                                     1e-5)
            use = [0] * n_layers
            for l in (estimator_layers if estimator_layers is not None else range(n_layers)):
                use[l] = 1
            M.moe_spec_set_estimator_layers(self.ctx, use)
        # host pool: [L, E, 3*H*I] in storage dtype, pinned
        if isinstance(experts, np.ndarray):
            t = _np_to_torch_storage(experts)
            pool = torch.empty(t.shape, dtype=t.dtype, pin_memory=True)
            pool.copy_(t)
        else:
            pool = experts                      # a pinned tensor [L,E,n] or a list of per-layer pinned tensors
            assert all(pool[l].is_pinned() and pool[l].is_contiguous() for l in range(n_layers))
        self.pool = pool
        for l in range(n_layers):
            M.moe_spec_load_host_experts(self.ctx, l, 0, n_experts, pool[l].data_ptr(),
                                         n_experts * self.expert_bytes)
        torch.cuda.synchronize(self.dev)

    # ------------------------------------------------------------------ calls
    def begin_token(self):
        M.moe_spec_begin_token(self.ctx)

    def layer_step(self, layer: int, r: torch.Tensor, out: Optional[torch.Tensor] = None, want_ids=False,
                   sync_input=True, static_scratch=False):
        """r: [B,H] float32 on the device.  With sync_input the compute stream first waits for the
        caller's current torch stream (where r was produced); callers that already work on
        `self.compute` pass False."""
        B = r.shape[0]
        assert r.dtype == torch.float32 and r.is_contiguous() and r.shape[1] == self.H
        if out is None:
            out = torch.empty_like(r)
        outs = None
        bufs = None
        if want_ids:
            mk_i = lambda: torch.full((B, self.k), -1, dtype=torch.int32, device=self.dev)
            mk_f = lambda: torch.full((B, self.k), float("nan"), dtype=torch.float32, device=self.dev)
            bufs = {"true_ids": mk_i(), "true_gates": mk_f(), "exec_ids": mk_i(), "exec_gates": mk_f(),
                    "next_ids": mk_i(), "next_gates": mk_f()}
            outs = M.StepOutputs(**{k: v.data_ptr() for k, v in bufs.items()})
        if sync_input:
            self.compute.wait_stream(torch.cuda.current_stream(self.dev))
        step = M.moe_spec_layer_step_static if static_scratch else M.moe_spec_layer_step
        step(self.ctx, layer, r.data_ptr(), B, out.data_ptr(), outs)
        if sync_input:
            self._hand_back(r, out, *(bufs.values() if bufs else ()))
        return out, bufs

    def _hand_back(self, *tensors):
        """The tensors were allocated on the caller's stream but are read or written by kernels on the
        compute stream: tell torch's allocator so (a freed block must not be reused before those
        kernels ran) and make the caller's stream wait for them."""
        for t in tensors:
            if t is not None:
                t.record_stream(self.compute)
        torch.cuda.current_stream(self.dev).wait_stream(self.compute)

    def prefill_layer_step(self, layer: int, r: torch.Tensor, out: Optional[torch.Tensor] = None, want_ids=False,
                           sync_input=True):
        """r: [P,H] float32 on the device, all prompt tokens of one layer."""
        P = r.shape[0]
        assert r.dtype == torch.float32 and r.is_contiguous() and r.shape[1] == self.H
        if out is None:
            out = torch.empty_like(r)
        ids = gates = None
        if want_ids:
            ids = torch.full((P, self.k), -1, dtype=torch.int32, device=self.dev)
            gates = torch.full((P, self.k), float("nan"), dtype=torch.float32, device=self.dev)
        if sync_input:
            self.compute.wait_stream(torch.cuda.current_stream(self.dev))
        M.moe_spec_prefill_layer_step(self.ctx, layer, r.data_ptr(), P, out.data_ptr(),
                                      ids.data_ptr() if want_ids else None, gates.data_ptr() if want_ids else None)
        if sync_input:
            self._hand_back(r, out, ids, gates)
        return out, ids, gates

    def advance(self, r, out, eps, a, b, r_next=None):
        if r_next is None:
            r_next = torch.empty_like(r)
        foreign = torch.cuda.current_stream(self.dev) != self.compute     # the caller works on another stream
        if foreign:
            self.compute.wait_stream(torch.cuda.current_stream(self.dev))
        M.moe_spec_synth_advance(self.compute.cuda_stream, r.data_ptr(), out.data_ptr(), eps.data_ptr(),
                                 a, b, r.shape[0], r.shape[1], r_next.data_ptr())
        if foreign:
            self._hand_back(r, out, eps, r_next)
        return r_next

    def stats(self) -> dict:
        return M.moe_spec_stats(self.ctx)

    def layer_diagnostics(self, layer: int) -> dict:
        return M.moe_spec_layer_diagnostics(self.ctx, layer)

    def read_default_vectors(self, layer: int):
        mean = torch.empty((self.E, self.H), dtype=torch.float32, device=self.dev)
        counts = M.moe_spec_read_default_vectors(self.ctx, layer, mean.data_ptr(), self.E)
        return mean, counts

    def reset(self):
        M.moe_spec_reset(self.ctx)

    def time_kernel(self, which: int, reps: int):
        return M.moe_spec_time_kernel(self.ctx, which, reps)

    def close(self):
        if self.ctx:
            M.moe_spec_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def engine_for(wl, mode, resident, experts, **kw) -> Engine:
    return Engine(n_layers=wl.n_layers, hidden=wl.hidden, n_experts=wl.n_experts, top_k=wl.top_k,
                  inter=wl.inter, dtype=wl.dtype, max_batch=kw.pop("max_batch", wl.batch), slots=wl.slots,
                  mode=mode, resident=resident, experts=experts, **kw)
