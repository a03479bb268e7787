"""ctypes binding of libmoe_spec.so: the same entry points as include/moe_spec.h, argument
marshalling only.  Every step of the path runs in the library's HIP kernels; if the library is
missing this module raises instead of falling back to anything else."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoe_spec.so")

OK, EINVAL, ENOMEM, ESTATE, EHIP = 0, -1, -2, -3, -4
MODE_ON_DEMAND, MODE_SPECULATIVE, MODE_PREFETCH_HINT = 0, 1, 2
F32, BF16 = 0, 1
COPY_DMA, COPY_KERNEL, COPY_DMA2 = 0, 1, 2
STATIC_SCRATCH_BYTES = 8 << 20


class Config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("hidden", C.c_int32), ("n_experts", C.c_int32),
                ("top_k", C.c_int32), ("inter", C.c_int32), ("max_batch", C.c_int32),
                ("slots_per_layer", C.c_int32), ("dtype", C.c_int32), ("mode", C.c_int32),
                ("rms_eps", C.c_float), ("q_from_normalized", C.c_int32),
                ("predict_in_on_demand", C.c_int32), ("profile", C.c_int32), ("copy_engine", C.c_int32),
                ("predict_signal", C.c_int32), ("diagnostics", C.c_int32),
                ("accumulate_defaults", C.c_int32), ("max_prefill_tokens", C.c_int32),
                ("wait_spin_limit", C.c_int32), ("lookahead", C.c_int32), ("est_latent", C.c_int32), ("est_ffn", C.c_int32),
                ("device_arena", C.c_void_p), ("device_arena_bytes", C.c_size_t),
                ("compute_stream", C.c_void_p), ("copy_stream", C.c_void_p)]


class Stats(C.Structure):
    _fields_ = [("tokens", C.c_int64), ("layer_steps", C.c_int64), ("predictions", C.c_int64),
                ("hits", C.c_int64), ("cache_hits", C.c_int64), ("cache_misses", C.c_int64),
                ("h2d_bytes", C.c_int64), ("hbm_bytes_algorithmic", C.c_int64),
                ("copy_ms", C.c_double), ("compute_ms", C.c_double), ("stall_ms", C.c_double),
                ("wall_ms", C.c_double), ("expert_ms", C.c_double), ("expert_launches", C.c_int64),
                ("prefill_tokens", C.c_int64), ("predictions2", C.c_int64), ("hits2", C.c_int64),
                ("cache_waves", C.c_int64)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class LayerDiag(C.Structure):
    _fields_ = [("predictions", C.c_int64), ("hits", C.c_int64), ("rank_match", C.c_int64 * 16),
                ("cos_sum", C.c_double), ("cos_count", C.c_int64)]


class StepOutputs(C.Structure):
    _fields_ = [("true_ids", C.c_void_p), ("true_gates", C.c_void_p), ("exec_ids", C.c_void_p),
                ("exec_gates", C.c_void_p), ("next_ids", C.c_void_p), ("next_gates", C.c_void_p)]


class MoeSpecError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"moe_spec error {code}: {msg}")
        self.code = code


_lib = None


def lib():
    """Loads the library once.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2603_19289_amd.build` "
                              "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        vp, i32, sz = C.c_void_p, C.c_int, C.c_size_t
        L.moe_spec_arena_bytes.restype = sz
        L.moe_spec_arena_bytes.argtypes = [C.POINTER(Config)]
        L.moe_spec_expert_bytes.restype = sz
        L.moe_spec_expert_bytes.argtypes = [C.POINTER(Config)]
        L.moe_spec_create.argtypes = [C.POINTER(Config), C.POINTER(vp)]
        L.moe_spec_set_layer_resident.argtypes = [vp, i32, vp, vp, vp]
        L.moe_spec_load_host_experts.argtypes = [vp, i32, i32, i32, vp, sz]
        L.moe_spec_set_estimator.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, C.c_float]
        L.moe_spec_set_estimator_layers.argtypes = [vp, C.POINTER(C.c_uint8), i32]
        L.moe_spec_begin_token.argtypes = [vp]
        L.moe_spec_layer_step.argtypes = [vp, i32, vp, i32, vp, C.POINTER(StepOutputs)]
        L.moe_spec_layer_step_static.argtypes = [vp, i32, vp, i32, vp, C.POINTER(StepOutputs)]
        L.moe_spec_prefill_layer_step.argtypes = [vp, i32, vp, i32, vp, vp, vp]
        L.moe_spec_stats.argtypes = [vp, C.POINTER(Stats)]
        L.moe_spec_layer_diagnostics.argtypes = [vp, i32, C.POINTER(LayerDiag)]
        L.moe_spec_read_default_vectors.argtypes = [vp, i32, vp, C.POINTER(C.c_int64)]
        L.moe_spec_reset.argtypes = [vp]
        L.moe_spec_destroy.argtypes = [vp]
        L.moe_spec_destroy.restype = None
        L.moe_spec_last_error.argtypes = [vp]
        L.moe_spec_last_error.restype = C.c_char_p
        L.moe_spec_time_kernel.argtypes = [vp, i32, i32, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        L.moe_spec_synth_advance.argtypes = [vp, vp, vp, vp, C.c_double, C.c_double, i32, i32, vp]
        _lib = L
    return _lib


def _check(rc, ctx=None):
    if rc != OK:
        raise MoeSpecError(rc, (lib().moe_spec_last_error(ctx) or b"").decode())


def moe_spec_arena_bytes(cfg: Config) -> int:
    return lib().moe_spec_arena_bytes(C.byref(cfg))


def moe_spec_expert_bytes(cfg: Config) -> int:
    return lib().moe_spec_expert_bytes(C.byref(cfg))


def moe_spec_create(cfg: Config) -> int:
    out = C.c_void_p()
    _check(lib().moe_spec_create(C.byref(cfg), C.byref(out)))
    return out.value


def moe_spec_set_layer_resident(ctx, layer, router_w_ptr, rms_gain_ptr, default_vecs_ptr):
    _check(lib().moe_spec_set_layer_resident(ctx, layer, router_w_ptr, rms_gain_ptr, default_vecs_ptr), ctx)


def moe_spec_load_host_experts(ctx, layer, first_expert, n_experts, pinned_host_ptr, nbytes):
    _check(lib().moe_spec_load_host_experts(ctx, layer, first_expert, n_experts, pinned_host_ptr, nbytes), ctx)


def moe_spec_set_estimator(ctx, proj, layer_emb, ffn_in, ffn_out, ln_gain, ln_bias, head, ln_eps):
    _check(lib().moe_spec_set_estimator(ctx, proj, layer_emb, ffn_in, ffn_out, ln_gain, ln_bias, head, ln_eps), ctx)


def moe_spec_set_estimator_layers(ctx, use):
    arr = (C.c_uint8 * len(use))(*[1 if u else 0 for u in use])
    _check(lib().moe_spec_set_estimator_layers(ctx, arr, len(use)), ctx)


def moe_spec_begin_token(ctx):
    _check(lib().moe_spec_begin_token(ctx), ctx)


def moe_spec_layer_step(ctx, layer, r_ptr, batch, out_ptr, outs: Optional[StepOutputs] = None):
    _check(lib().moe_spec_layer_step(ctx, layer, r_ptr, batch, out_ptr,
                                     C.byref(outs) if outs is not None else None), ctx)


def moe_spec_layer_step_static(ctx, layer, r_ptr, batch, out_ptr, outs: Optional[StepOutputs] = None):
    _check(lib().moe_spec_layer_step_static(ctx, layer, r_ptr, batch, out_ptr,
                                            C.byref(outs) if outs is not None else None), ctx)


def moe_spec_prefill_layer_step(ctx, layer, r_ptr, n_tokens, out_ptr, true_ids_ptr=None, true_gates_ptr=None):
    _check(lib().moe_spec_prefill_layer_step(ctx, layer, r_ptr, n_tokens, out_ptr, true_ids_ptr, true_gates_ptr), ctx)


def moe_spec_stats(ctx) -> dict:
    st = Stats()
    _check(lib().moe_spec_stats(ctx, C.byref(st)), ctx)
    return st.as_dict()


def moe_spec_layer_diagnostics(ctx, layer: int) -> dict:
    d = LayerDiag()
    _check(lib().moe_spec_layer_diagnostics(ctx, layer, C.byref(d)), ctx)
    return {"predictions": d.predictions, "hits": d.hits, "rank_match": list(d.rank_match),
            "cos_sum": d.cos_sum, "cos_count": d.cos_count}


def moe_spec_read_default_vectors(ctx, layer: int, mean_ptr, n_experts: int):
    counts = (C.c_int64 * n_experts)()
    _check(lib().moe_spec_read_default_vectors(ctx, layer, mean_ptr, counts), ctx)
    return list(counts)


def moe_spec_reset(ctx):
    _check(lib().moe_spec_reset(ctx), ctx)


def moe_spec_destroy(ctx):
    lib().moe_spec_destroy(ctx)


def moe_spec_time_kernel(ctx, which: int, reps: int):
    ms, nbytes = C.c_double(), C.c_int64()
    _check(lib().moe_spec_time_kernel(ctx, which, reps, C.byref(ms), C.byref(nbytes)), ctx)
    return ms.value, nbytes.value


def moe_spec_synth_advance(stream_ptr, r_ptr, out_ptr, eps_ptr, a, b, batch, hidden, r_next_ptr):
    rc = lib().moe_spec_synth_advance(stream_ptr, r_ptr, out_ptr, eps_ptr, a, b, batch, hidden, r_next_ptr)
    if rc != 0:
        raise MoeSpecError(rc, "moe_spec_synth_advance failed")
