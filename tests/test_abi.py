"""CPU-side checks of the C ABI: the library loads, exports every function the headers
declare, sizes its arena as documented and rejects bad configurations before touching a GPU."""
import ctypes as C
import os
import re

import pytest
import torch

from paper_2603_19289_amd import moe_spec as M

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = []
    for fn in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", fn)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"\b(moe_spec_[a-z_]+)\s*\(", text)
    return sorted(set(names))


def good_config(**kw):
    base = dict(n_layers=4, hidden=256, n_experts=8, top_k=2, inter=512, max_batch=1, slots_per_layer=4,
                dtype=M.F32, mode=M.MODE_SPECULATIVE, rms_eps=1e-6)
    base.update(kw)
    return M.Config(**base)


def test_library_exports_every_declared_function():
    names = declared_functions()
    assert {"moe_spec_create", "moe_spec_load_host_experts", "moe_spec_layer_step", "moe_spec_stats"} <= set(names)
    lib = M.lib()
    for n in names:
        assert hasattr(lib, n), n


def test_expert_and_arena_bytes():
    cfg = good_config()
    assert M.moe_spec_expert_bytes(cfg) == 3 * 256 * 512 * 4
    cfg16 = good_config(dtype=M.BF16, hidden=2048, inter=768, n_experts=128, top_k=8, slots_per_layer=16, n_layers=48)
    eb = M.moe_spec_expert_bytes(cfg16)
    assert eb == 9437184
    need = M.moe_spec_arena_bytes(cfg16)
    assert 48 * 16 * eb <= need <= 48 * 16 * eb + (8 << 20)      # slot cache plus a little scratch


@pytest.mark.parametrize("bad", [dict(n_layers=0), dict(hidden=250), dict(hidden=16384), dict(inter=100),
                                 dict(n_experts=0), dict(n_experts=300), dict(top_k=0), dict(top_k=9),
                                 dict(top_k=17, n_experts=32), dict(max_batch=0), dict(max_batch=65),
                                 dict(slots_per_layer=1), dict(dtype=7), dict(mode=5), dict(rms_eps=-1.0),
                                 dict(predict_signal=2), dict(copy_engine=9)])
def test_invalid_configurations_are_rejected(bad):
    cfg = good_config(**bad)
    assert M.moe_spec_arena_bytes(cfg) == 0
    assert M.moe_spec_expert_bytes(cfg) == 0
    out = C.c_void_p()
    rc = M.lib().moe_spec_create(C.byref(cfg), C.byref(out))
    assert rc == M.EINVAL and out.value is None
    assert M.lib().moe_spec_last_error(None)


def test_create_checks_the_arena_before_any_gpu_call():
    cfg = good_config()
    out = C.c_void_p()
    assert M.lib().moe_spec_create(C.byref(cfg), C.byref(out)) == M.EINVAL          # null arena
    cfg.device_arena = 0x1001
    cfg.device_arena_bytes = 1 << 40
    assert M.lib().moe_spec_create(C.byref(cfg), C.byref(out)) == M.EINVAL          # misaligned
    cfg.device_arena = 0x1000
    cfg.device_arena_bytes = 16
    assert M.lib().moe_spec_create(C.byref(cfg), C.byref(out)) == M.EINVAL          # too small
    assert b"arena" in M.lib().moe_spec_last_error(None)
    assert M.lib().moe_spec_create(C.byref(cfg), None) == M.EINVAL


@pytest.mark.skipif(torch.cuda.is_available(), reason="meant for a machine without a GPU")
def test_create_without_a_gpu_fails_loudly():
    cfg = good_config()
    cfg.device_arena = 0x1000
    cfg.device_arena_bytes = 1 << 40
    with pytest.raises(M.MoeSpecError) as ei:
        M.moe_spec_create(cfg)
    assert ei.value.code == M.EHIP


def test_null_context_is_an_error_not_a_crash():
    lib = M.lib()
    assert lib.moe_spec_begin_token(None) == M.EINVAL
    assert lib.moe_spec_reset(None) == M.EINVAL
    assert lib.moe_spec_stats(None, None) == M.EINVAL
    assert lib.moe_spec_layer_step(None, 0, None, 1, None, None) == M.EINVAL
    lib.moe_spec_destroy(None)


def test_prefill_entry_point_rejects_a_null_context():
    assert M.lib().moe_spec_prefill_layer_step(None, 0, None, 1, None, None, None) == M.EINVAL


def test_invalid_prefill_capacity_is_rejected():
    cfg = good_config()
    cfg.max_prefill_tokens = -1
    assert M.moe_spec_arena_bytes(cfg) == 0
    cfg.max_prefill_tokens = 1 << 20
    assert M.moe_spec_arena_bytes(cfg) == 0
    cfg.max_prefill_tokens = 0
    small = M.moe_spec_arena_bytes(cfg)
    cfg.max_prefill_tokens = 256
    assert M.moe_spec_arena_bytes(cfg) > small           # the prefill buffers are part of the arena


def test_bench_refuses_more_than_one_gpu(monkeypatch, capsys):
    import bench
    monkeypatch.setattr("sys.argv", ["bench.py", "--gpus", "2"])
    with pytest.raises(SystemExit) as ei:
        bench.main()
    assert ei.value.code == 2
    assert "ONE GPU" in capsys.readouterr().err


def test_workload_pools_fit_what_a_box_can_pin():
    """Every registered workload must be runnable: its host pool stays under the page-locking limit, if need be by
    holding fewer layers' expert blocks than the model has (layers then share blocks, everything else is per layer)."""
    from paper_2603_19289_amd import workload as W
    for wl in W.CONFIGS.values():
        assert wl.pinnable, wl.name
        assert 1 <= wl.distinct_pool_layers <= wl.n_layers
        assert wl.pool_bytes == wl.distinct_pool_layers * wl.n_experts * wl.expert_bytes
    c4 = W.CONFIGS["c4_mixtral_8x7b"]
    assert (c4.n_layers, c4.distinct_pool_layers) == (32, 24)
    assert c4.with_(n_layers=2).distinct_pool_layers == 2
    assert not c4.with_(pool_layers=0).pinnable          # 90 GB: what the box refuses


@pytest.mark.gpu
def test_c_client_of_the_library_runs():
    """csrc/abi_demo.c uses the boundary from plain C, without Python or torch: three modes, prefill, error returns,
    counter identities, run-to-run bit equality.  It ran as its own process before this session touched the GPU
    (tests/conftest.py); here its verdict is checked."""
    from tests.conftest import C_CLIENT
    if not C_CLIENT["ran"]:
        pytest.skip("the C client did not run (not built, or GPU tests were not selected with -m gpu)")
    assert C_CLIENT["rc"] == 0, C_CLIENT["output"]
    assert "abi demo ok" in C_CLIENT["output"]
