"""Glue used by the tests only: build the checker's model from generated inputs."""
import numpy as np

from oracle import moe_oracle as O
from paper_2603_19289_amd import workload as W


# Layer outputs are compared two ways.  Per token row, the relative L2 error must stay within the
# workload definition's figures (1e-5 with float32 weights, 2e-2 with bf16 weights).  Element by
# element, |got - want| must stay within ELEM_TOL times the root mean square of the row: a single
# wrong element (which an L2 norm over thousands of columns would let through) is of the order of
# the RMS itself.  Where the figures come from: float32 accumulation of n <= 32768 products is off by
# about sqrt(n) * 6e-8; with bf16 weights the kernels round the SwiGLU product to bf16 from a float32
# pre-image where the checker rounds from float64, so now and then one h_i lands on the neighbouring
# bf16 value (2^-8 relative) and moves every output element by g * W_down[row, i] * ulp(h_i).  The
# constants are four to five times the worst values the GPU tests print (2.0e-6 and 2.5e-3).
# An output element is a sum of k*I terms, its row's RMS about sqrt(k*I) times one term's spread; one flipped
# h_i moves one term by up to 2^-7 of itself, and a term can be a few times the spread, so a single flip shows as
# up to about 0.1 / sqrt(k*I) of the RMS: below 1e-2 from some 250 terms on (every benchmark shape has thousands),
# above it for the tiny layers the randomised tests draw (k*I = 24: 1.1e-2 seen, reproduced to the last bit by a
# float32 emulation of the kernel's SwiGLU step).  elem_tol widens the bound for those and only for those.
L2_TOL = {"f32": 1e-5, "bf16": 2e-2}
ELEM_TOL = {"f32": 1e-5, "bf16": 1e-2}


def elem_tol(dtype, terms=None):
    if dtype != "bf16" or not terms:
        return ELEM_TOL[dtype]
    return max(ELEM_TOL[dtype], 0.16 / float(np.sqrt(terms)))


def output_errors(got, want):
    """(worst relative L2 error of a row, worst |difference| of an element in units of its row's RMS)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    l2 = np.linalg.norm(got - want, axis=-1) / np.maximum(np.linalg.norm(want, axis=-1), 1e-30)
    rms = np.sqrt(np.mean(want * want, axis=-1, keepdims=True))
    elem = np.abs(got - want) / np.maximum(rms, 1e-30)
    return float(l2.max()), float(elem.max())


def check_output(got, want, dtype, where="", terms=None):
    """terms: k * I, the number of products an output element sums (see elem_tol)."""
    l2, elem = output_errors(got, want)
    assert l2 <= L2_TOL[dtype], f"{where}: relative L2 error {l2:.3e}"
    assert elem <= elem_tol(dtype, terms), f"{where}: an element is off by {elem:.3e} of its row's RMS"
    return l2, elem


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
