"""Seeded synthetic workloads: model shapes, weights, token inputs and residual noise.

This module only *generates inputs*.  It holds none of the method's arithmetic (no norm, no
router, no top-k, no expert FFN, no cache policy) and is used by the tests, the benchmark
and the smoke check to feed the same bytes to the HIP library and to the CPU checker.

The workloads stand in for the paper's evaluation models (Sec. 5.1.1, Table 2): the same
layer shapes with random weights, which is what the paper itself does for two of its four
models.  Decode steps are independent draws; the only state carried from token to token
is the content of the device expert cache.
"""
from __future__ import annotations

import ctypes
from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np

_FAMILY = {"router": 1, "dvec": 2, "expert": 3, "x0": 4, "eps": 5, "center": 6, "eta0": 7,
           "eps_cluster": 8, "gain": 9, "estimator": 10}


@dataclass(frozen=True)
class Workload:
    name: str
    n_layers: int          # L
    hidden: int            # H
    n_experts: int         # E
    top_k: int             # k
    inter: int             # I
    dtype: str             # "f32" | "bf16"  (storage type of all weights)
    batch: int             # B
    tokens: int            # decode steps
    slots: int             # S, device cache slots per layer
    seed: int
    res_a: float           # residual driver: r' = a*v + b*(|v|/sqrt(H))*eps, v = r + O
    res_b: float
    clusters: int = 0      # >0: batch rows follow `clusters` shared noise streams
    tau: float = 0.1       # per-row share of the noise when clustered
    w_std: float = 0.02
    d_std: float = 0.05
    per_layer_dvec: bool = False   # True: d_{l,e} identical for all e (literal per-layer reading)
    pool_layers: int = 0           # >0: the host pool holds this many layers' expert blocks and layer l reads those
                                   # of layer l % pool_layers (for pools larger than the box can page-lock)

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == "bf16" else 4

    @property
    def expert_elems(self) -> int:
        return 3 * self.hidden * self.inter

    @property
    def expert_bytes(self) -> int:
        return self.expert_elems * self.elem_bytes

    @property
    def distinct_pool_layers(self) -> int:
        return min(self.pool_layers, self.n_layers) if self.pool_layers > 0 else self.n_layers

    @property
    def pool_bytes(self) -> int:
        return self.distinct_pool_layers * self.n_experts * self.expert_bytes

    @property
    def pinnable(self) -> bool:
        """The GPU machines page-lock at most about 72 GB of host memory (hipHostMalloc fails beyond)."""
        return self.pool_bytes <= PIN_LIMIT_BYTES

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


PIN_LIMIT_BYTES = 70 * 10 ** 9
_RHO = 0.9
CONFIGS: Dict[str, Workload] = {
    # tiny fp32 stack: residual update is additive Gaussian noise with std 0.1*|v|/sqrt(H)
    "c1_tiny": Workload("c1_tiny", 4, 256, 8, 2, 512, "f32", 1, 32, 4, 0, 1.0, 0.1),
    # Qwen3-30B-A3B-shaped layers, AR(1) residual stream with correlation 0.9
    "c2_qwen3_30b_a3b": Workload("c2_qwen3_30b_a3b", 48, 2048, 128, 8, 768, "bf16", 1, 256, 16, 1,
                                 _RHO, float(np.sqrt(1 - _RHO ** 2))),
    "c3_gpt_oss_20b": Workload("c3_gpt_oss_20b", 24, 2880, 32, 4, 2880, "bf16", 1, 256, 8, 2,
                               _RHO, float(np.sqrt(1 - _RHO ** 2))),
    "c3_gpt_oss_20b_b8": Workload("c3_gpt_oss_20b_b8", 24, 2880, 32, 4, 2880, "bf16", 8, 256, 8, 2,
                                  _RHO, float(np.sqrt(1 - _RHO ** 2))),
    # 32 layers x 8 experts x 352 MB = 90.2 GB of expert blocks; the GPU machines page-lock about 72 GB, so the host
    # pool holds 24 layers' blocks (67.6 GB) and layers 24-31 read the blocks of layers 0-7.  Every layer still has
    # its own router, default vectors, slot cache and transfers: bytes moved, kernels and cache behaviour per layer
    # are those of 32 distinct layers; only the values of a quarter of the expert weights repeat.
    "c4_mixtral_8x7b": Workload("c4_mixtral_8x7b", 32, 4096, 8, 2, 14336, "bf16", 1, 128, 3, 3,
                                _RHO, float(np.sqrt(1 - _RHO ** 2)), pool_layers=24),
    # the same layers, 24 of them, each with its own blocks
    "c4_mixtral_8x7b_l24": Workload("c4_mixtral_8x7b_l24", 24, 4096, 8, 2, 14336, "bf16", 1, 128, 3, 3,
                                    _RHO, float(np.sqrt(1 - _RHO ** 2))),
    "c5_qwen3_b32": Workload("c5_qwen3_b32", 48, 2048, 128, 8, 768, "bf16", 32, 256, 48, 4,
                             _RHO, float(np.sqrt(1 - _RHO ** 2)), clusters=4),
}


def _rng(seed: int, family: str, *keys: int) -> np.random.Generator:
    """Counter-based stream keyed by (seed, family) with the tensor's coordinates as the
    starting counter, so every tensor can be drawn on its own in any order."""
    ctr = list(keys) + [0] * (3 - len(keys))
    return np.random.Generator(np.random.Philox(key=[seed, _FAMILY[family]],
                                                counter=[0, ctr[2], ctr[1], ctr[0]]))


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """float values -> stored weights: float32 as is, bf16 as uint16 bit patterns (round to
    nearest even from float32, done by torch's own conversion)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    import torch
    return torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def make_resident(wl: Workload, gains: str = "ones") -> Dict[str, np.ndarray]:
    """Router weights [L,E,H], RMSNorm gains [L,H] (float32) and default vectors [L,E,H]."""
    L, E, H = wl.n_layers, wl.n_experts, wl.hidden
    router = np.stack([_rng(wl.seed, "router", l).standard_normal((E, H), dtype=np.float32) * wl.w_std
                       for l in range(L)])
    if wl.per_layer_dvec:
        dv = np.stack([np.broadcast_to(_rng(wl.seed, "dvec", l).standard_normal((1, H), dtype=np.float32)
                                       * wl.d_std, (E, H)) for l in range(L)])
    else:
        dv = np.stack([_rng(wl.seed, "dvec", l).standard_normal((E, H), dtype=np.float32) * wl.d_std
                       for l in range(L)])
    if gains == "ones":
        gain = np.ones((L, H), dtype=np.float32)
    else:   # distinct per layer, used by tests that must tell LN_l from LN_{l+1}
        gain = np.stack([1.0 + 0.25 * _rng(wl.seed, "gain", l).standard_normal(H, dtype=np.float32)
                         for l in range(L)]).astype(np.float32)
    return {"router_w": to_storage(router, wl.dtype), "rms_gain": gain,
            "dvecs": to_storage(dv, wl.dtype)}


def make_estimator(wl: Workload, m: int = 4, n: int = 2) -> Dict[str, np.ndarray]:
    """Random weights in the shapes of the paper's estimator (Appendix A; trained weights do not exist
    here): latent size dm = H/m, feed-forward size F = n*dm.  Every matrix is stored [out, in]."""
    H, E, L = wl.hidden, wl.n_experts, wl.n_layers
    dm, F = H // m, n * (H // m)
    g = lambda i, shape, std: _rng(wl.seed, "estimator", i).standard_normal(shape, dtype=np.float32) * std
    return {"proj": to_storage(g(0, (dm, H), 1.0 / np.sqrt(H)), wl.dtype),
            "layer_emb": to_storage(g(1, (L, dm), 0.5), wl.dtype),
            "ffn_in": to_storage(g(2, (F, dm), 1.0 / np.sqrt(dm)), wl.dtype),
            "ffn_out": to_storage(g(3, (dm, F), 1.0 / np.sqrt(F)), wl.dtype),
            "ln_gain": (1.0 + 0.1 * g(4, (dm,), 1.0)).astype(np.float32),
            "ln_bias": (0.1 * g(5, (dm,), 1.0)).astype(np.float32),
            "head": to_storage(g(6, (E, dm), 1.0 / np.sqrt(dm)), wl.dtype)}


def make_experts_host(wl: Workload, out: Optional[np.ndarray] = None) -> np.ndarray:
    """Expert pool [L, E, 3*H*I] in storage dtype, each block W_gate[I,H] | W_up[I,H] | W_down[H,I],
    drawn on the CPU.  Meant for pools up to a few GB; larger pools use fill_experts_gpu."""
    L, E, n = wl.n_layers, wl.n_experts, wl.expert_elems
    st = np.uint16 if wl.dtype == "bf16" else np.float32
    if out is None:
        out = np.empty((L, E, n), dtype=st)
    for l in range(L):
        for e in range(E):
            w = _rng(wl.seed, "expert", l, e).standard_normal(n, dtype=np.float32) * wl.w_std
            out[l, e] = to_storage(w, wl.dtype)
    return out


_hip_runtime = None


def pinned_empty(n_elems: int, dtype: str):
    """A page-locked host buffer of exactly n_elems weights as a 1-D torch tensor (bf16 or float32),
    straight from hipHostMalloc.  torch's own pinned allocator rounds every request up to a power of
    two, which the 38-90 GB pools cannot afford.  The buffer lives until free_pinned_pool or the end of the process."""
    import torch
    global _hip_runtime
    if _hip_runtime is None:
        _hip_runtime = ctypes.CDLL("libamdhip64.so")
        _hip_runtime.hipHostMalloc.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_size_t, ctypes.c_uint]
    nbytes = n_elems * (2 if dtype == "bf16" else 4)
    ptr = ctypes.c_void_p()
    rc = _hip_runtime.hipHostMalloc(ctypes.byref(ptr), nbytes, 0)
    if rc != 0 or not ptr.value:
        raise MemoryError(f"hipHostMalloc of {nbytes} bytes failed with error {rc}")
    raw = np.frombuffer((ctypes.c_uint8 * nbytes).from_address(ptr.value), dtype=np.uint8)
    t = torch.from_numpy(raw.view(np.int16)).view(torch.bfloat16) if dtype == "bf16" else torch.from_numpy(raw.view(np.float32))
    _pinned[t.data_ptr()] = ptr.value
    return t


_pinned: Dict[int, int] = {}


def free_pinned_pool(pool) -> None:
    """Unpins and frees what alloc_pinned_pool allocated (a list of per-layer tensors).  The tensors must not be
    used afterwards, and no context may still read the pool.  Without this the process would unpin tens of
    gigabytes while it exits."""
    for t in pool:
        ptr = _pinned.pop(t.data_ptr(), None)
        if ptr is not None:
            _hip_runtime.hipHostFree(ctypes.c_void_p(ptr))


def free_all_pinned() -> None:
    """Unpins and frees every buffer pinned_empty handed out that is still held (after a failed run)."""
    for ptr in list(_pinned.values()):
        _hip_runtime.hipHostFree(ctypes.c_void_p(ptr))
    _pinned.clear()


def alloc_pinned_pool(wl: Workload):
    """Pinned host pool as a list of per-layer torch tensors [E, 3*H*I] in the storage dtype (entries repeat
    when the workload's pool holds fewer layers than the model has)."""
    held = [pinned_empty(wl.n_experts * wl.expert_elems, wl.dtype).view(wl.n_experts, wl.expert_elems)
            for _ in range(wl.distinct_pool_layers)]
    return [held[l % len(held)] for l in range(wl.n_layers)]


class PoolView:
    """Read-only numpy view of a per-layer pool, indexable as pool[layer, expert] (bf16 as uint16)."""

    def __init__(self, layers):
        import torch
        self.layers = [t.view(torch.int16).numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.numpy()
                       for t in layers]

    def __getitem__(self, idx):
        layer, e = idx
        return self.layers[layer][e]


def fill_experts_gpu(wl: Workload, pool, device="cuda") -> None:
    """Fill a pinned pool (a torch tensor [L, E, 3*H*I] or a list of per-layer tensors) with
    N(0, w_std^2) drawn by torch's generator on the GPU, one layer at a time, and copy it down.
    The CPU checker then reads the very same bytes, so the device generator never has to be
    reproduced elsewhere."""
    import torch
    g = torch.Generator(device=device)
    for l in range(wl.distinct_pool_layers):
        g.manual_seed((wl.seed << 20) + l)
        buf = torch.empty(tuple(pool[l].shape), dtype=torch.float32, device=device)
        buf.normal_(0.0, wl.w_std, generator=g)
        pool[l].copy_(buf.to(pool[l].dtype))
        del buf
    torch.cuda.synchronize()


def make_inputs(wl: Workload, tokens: Optional[int] = None, n_layers: Optional[int] = None):
    """Token inputs x0 [T,B,H] and residual noise eps [T,L,B,H], float32, N(0,1).

    With clusters, row b follows cluster b mod C: x0_b = c_j + tau*eta_b and
    eps_b = sqrt(1-tau^2)*eps_cluster_j + tau*eta_b."""
    T = wl.tokens if tokens is None else tokens
    L = wl.n_layers if n_layers is None else n_layers
    B, H, C, tau = wl.batch, wl.hidden, wl.clusters, wl.tau
    x0 = np.empty((T, B, H), dtype=np.float32)
    eps = np.empty((T, L, B, H), dtype=np.float32)
    for t in range(T):
        if C == 0:
            x0[t] = _rng(wl.seed, "x0", t).standard_normal((B, H), dtype=np.float32)
        else:
            c = _rng(wl.seed, "center", t).standard_normal((C, H), dtype=np.float32)
            eta = _rng(wl.seed, "eta0", t).standard_normal((B, H), dtype=np.float32)
            x0[t] = c[np.arange(B) % C] + tau * eta
        for l in range(L):
            own = _rng(wl.seed, "eps", t, l).standard_normal((B, H), dtype=np.float32)
            if C == 0:
                eps[t, l] = own
            else:
                shared = _rng(wl.seed, "eps_cluster", t, l).standard_normal((C, H), dtype=np.float32)
                eps[t, l] = np.sqrt(1 - tau * tau) * shared[np.arange(B) % C] + tau * own
    return x0, eps


def advance_residual(wl: Workload, r: np.ndarray, out: np.ndarray, eps: np.ndarray) -> np.ndarray:
    """The stand-in for everything between two MoE blocks: v = r + O, then
    r' = a*v + b*(|v|_2/sqrt(H))*eps per row, returned as float32 values (in float64 storage)."""
    v = np.asarray(r, dtype=np.float64) + np.asarray(out, dtype=np.float64)
    scale = np.linalg.norm(v, axis=-1, keepdims=True) / np.sqrt(v.shape[-1])
    nxt = wl.res_a * v + wl.res_b * scale * np.asarray(eps, dtype=np.float64)
    return nxt.astype(np.float32).astype(np.float64)
