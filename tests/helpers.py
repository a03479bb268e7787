"""Glue used by the tests only: build the checker's model from generated inputs."""
import numpy as np

from oracle import moe_oracle as O
from paper_2603_19289_amd import workload as W


def oracle_model(wl, resident, experts, eps=1e-6):
    return O.OracleModel(
        n_layers=wl.n_layers, hidden=wl.hidden, n_experts=wl.n_experts, top_k=wl.top_k,
        inter=wl.inter, dtype=O.DTYPE_BF16 if wl.dtype == "bf16" else O.DTYPE_F32,
        router_w=resident["router_w"], rms_gain=resident["rms_gain"], dvecs=resident["dvecs"],
        experts=experts, rms_eps=eps)


def small_workload(**kw):
    base = dict(name="small", n_layers=3, hidden=64, n_experts=8, top_k=2, inter=48, dtype="bf16",
                batch=1, tokens=4, slots=4, seed=7, res_a=0.9, res_b=float(np.sqrt(1 - 0.81)))
    base.update(kw)
    return W.Workload(**base)


def build(wl, gains="ones"):
    res = W.make_resident(wl, gains=gains)
    ex = W.make_experts_host(wl)
    return res, ex, oracle_model(wl, res, ex)


def make_advance(wl, eps):
    def adv(t, l, r, out):
        return W.advance_residual(wl, r, out, eps[t, l])
    return adv
