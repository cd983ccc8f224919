"""CPU-side checks: the C-ABI library loads and exports what include/ckv.h declares,
host-side argument validation works without a GPU, workload generators are deterministic."""
import ctypes as C
import os
import re
import subprocess
import sys

import numpy as np
import pytest

from paper_2601_16986_amd import ckv, workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ckv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ckv_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = ckv.load()
    names = declared_functions()
    assert len(names) >= 20
    for name in names:
        assert hasattr(lib, name), f"{name} is declared in include/ckv.h but not exported"
    assert sorted(ckv.EXPORTS) == names, "binding and header disagree on the entry points"


def test_workspace_bytes_validates_geometry_and_parameters():
    lib = ckv.load()

    def ws(lay, par):
        return lib.ckv_workspace_bytes(C.byref(lay), C.byref(par))

    lay = ckv.Layout(2, 2, 8, 2, 128, 256, ckv.F32, 0, 8 * 256)
    par = ckv.LrfuParams(0.5, 0.9, 0.0884, 0, 64, 1, 255)
    good = ws(lay, par)
    assert good > 0 and good % 256 == 0
    for field, bad in (("head_dim", 64), ("cap", 100), ("cap", 0), ("n_q_heads", 7), ("n_q_heads", 32),
                       ("n_layers", 0), ("out_dtype", 9), ("cap", 65536), ("pool_slots", 7 * 256), ("pool_slots", 8 * 256 + 32),
                       ("pool_slots", 0), ("headroom", -1), ("headroom", 256)):
        l2 = ckv.Layout(2, 2, 8, 2, 128, 256, ckv.F32, 0, 8 * 256)
        setattr(l2, field, bad)
        assert ws(l2, par) == 0, (field, bad)
    for field, bad in (("lambda_", 1.5), ("lambda_", -0.1), ("top_p", 0.0), ("softmax_scale", 0.0),
                       ("reward_mode", 7), ("t0", -1), ("budget_min", 0), ("budget_max", 256)):
        p2 = ckv.LrfuParams(0.5, 0.9, 0.0884, 0, 64, 1, 255)
        setattr(p2, field, bad)
        assert ws(lay, p2) == 0, (field, bad)
    # shared pools (headroom >= 1) may be smaller than units * cap: ckv_init checks them against the budgets
    l3 = ckv.Layout(2, 2, 8, 2, 128, 256, ckv.F32, 1, 4 * 256)
    assert ws(l3, par) > 0
    # a longer decay table (lambda closer to 1) needs a bigger workspace
    assert ws(lay, ckv.LrfuParams(0.99, 0.9, 0.0884, 0, 64, 1, 255)) > good


def test_init_rejects_bad_arguments_without_touching_the_gpu():
    lib = ckv.load()
    lay = ckv.Layout(1, 1, 8, 2, 128, 64, ckv.F32, 0, 2 * 256)
    par = ckv.LrfuParams(0.5, 0.9, 0.0884, 0, 0, 1, 63)
    ctx = C.c_void_p()
    budgets = np.full((1, 1, 2), 32, dtype=np.int32)
    bufs = ckv.Buffers()                                    # all NULL
    assert lib.ckv_init(C.byref(ctx), C.byref(lay), budgets.ctypes.data_as(C.c_void_p), C.byref(par),
                        C.byref(bufs), None) == ckv.EINVAL
    assert ctx.value is None
    assert lib.ckv_init(None, C.byref(lay), None, C.byref(par), C.byref(bufs), None) == ckv.EINVAL
    assert lib.ckv_decode_step(None, 0, None, None, None, None, 0, None) == ckv.EINVAL
    # every call that takes a context refuses a NULL one before anything else
    assert lib.ckv_evict(None, 0, None) == ckv.EINVAL and lib.ckv_evict_window(None, 0, 4, None) == ckv.EINVAL
    assert lib.ckv_seed_prompt(None, 0, None, 1, None) == ckv.EINVAL and lib.ckv_rebudget(None, None) == ckv.EINVAL
    assert lib.ckv_join(None, None) == ckv.EINVAL and lib.ckv_set_path(None, 0) == ckv.EINVAL
    assert lib.ckv_strerror(ckv.ECAPACITY).decode() == "unit full at append"
    assert lib.ckv_strerror(0).decode() == "ok"


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr


def test_workloads_are_seeded_and_budgets_conserved():
    cfg = wl.scaled(wl.CONFIGS["qwen14b"], n_layers=3, batch=2)
    b1, b2 = wl.draw_budgets(cfg), wl.draw_budgets(cfg)
    assert np.array_equal(b1, b2)
    assert b1.min() >= cfg.budget_min and b1.max() <= cfg.budget_max
    assert np.all(b1.sum(axis=(0, 2)) == cfg.n_layers * cfg.n_kv_heads * cfg.budget)
    s1 = wl.make_stream(wl.scaled(wl.CONFIGS["tiny"], decode_steps=5))
    s2 = wl.make_stream(wl.scaled(wl.CONFIGS["tiny"], decode_steps=5))
    assert np.array_equal(s1.q, s2.q) and np.array_equal(s1.prompt_k, s2.prompt_k)
    assert np.array_equal(wl.bf16_round(s1.q), s1.q)          # already on the bf16 grid
    u = wl.steady_unit(wl.CONFIGS["qwen14b"], 7, 300, 8704, wl.mean_query(cfg)[0, 0, 0])
    assert len(np.unique(u.pos)) == 300 and u.pos.max() < 8704 and np.all(u.tau >= u.pos)
    # bf16 rounding: ties to even
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -9], dtype=np.float32)
    assert wl.bf16_round(x).tolist() == [1.0, 1.015625, 1.0]
