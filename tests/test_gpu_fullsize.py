"""Parity at the full sizes of the benchmark workloads, in the launch configuration bench.py times
(all layers per call, steady-state caches built as in bench.py).

The oracle cannot step thousands of units in test time, so a sample of units spread over the
workload is filled from the host-side generator (the oracle and the GPU get the same arrays) and
compared entry by entry for a few decode steps; all other units are checked through properties
that hold at any size: caches sit at their budgets after eviction, outputs are finite, no
capacity overflow, time advanced, and (adaptive workloads) Alg. 2 conserves every sequence's total."""
import numpy as np
import pytest

from tests import parity

pytestmark = pytest.mark.gpu

N_SAMPLE = 10
N_STEPS = 3


def _run(name, n_sample=N_SAMPLE, n_steps=N_STEPS, rebudget_after=None):
    import torch
    import bench
    from oracle import crystal_kv as ok
    from paper_2601_16986_amd import workloads as wl

    cfg = wl.CONFIGS[name]
    dev = torch.device("cuda:0")
    g, budgets, (rq, rk, rv) = bench.build_workload(cfg, dev)
    t_now = cfg.prompt + cfg.decode_steps // 2
    flat = budgets.reshape(-1)
    # sample: smallest and largest budget plus units spread over the index range
    idx = sorted(set([int(np.argmin(flat)), int(np.argmax(flat))] +
                     [int(x) for x in np.linspace(0, flat.size - 1, n_sample).astype(int)]))
    keys = [tuple(int(v) for v in np.unravel_index(u, budgets.shape)) for u in idx]
    o = ok.CrystalKVOracle(cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, budgets,
                           lam=cfg.lam, top_p=cfg.top_p, t0=t_now, budget_min=cfg.budget_min, budget_max=cfg.budget_max)
    m = wl.mean_query(wl.scaled(cfg, n_layers=1, batch=1))
    for u, key in zip(idx, keys):
        c = wl.steady_unit(cfg, u, int(flat[u]), t_now, m[0, 0, key[2]])
        o.set_unit(key, c.K, c.V, c.pos, c.crf, c.tau)
        parity.sync_unit_to_gpu(g, o, key)
    stats = parity.LockstepStats()
    G = cfg.group
    for s in range(n_steps):
        out = g.decode_step(rq[s], rk[s], rv[s])
        qh, kh, vh = rq[s].float().cpu().numpy(), rk[s].float().cpu().numpy(), rv[s].float().cpu().numpy()
        outh = out.cpu().numpy()
        recs = {}
        for key in keys:
            l, b, h = key
            recs[key] = o.step_unit(key, qh[l, b, h * G:(h + 1) * G], kh[l, b, h], vh[l, b, h])
            err = parity.out_error(outh[l, b, h * G:(h + 1) * G], recs[key].y)
            stats.max_out_err = max(stats.max_out_err, err)
            assert err <= parity.OUT_TOL, (key, s, err)
        o.t += 1
        for key in keys:
            parity.compare_unit(g, o, key, recs[key], stats, check_kv=(s == n_steps - 1))
        # properties over every unit
        assert np.isfinite(outh).all()
        assert np.array_equal(g.lengths(), g.budgets())
        assert g.status() == 0 and g.time() == t_now + s + 1
    print(f"{name}: {len(keys)} sampled units x {n_steps} steps, max out err {stats.max_out_err:.2e}, "
          f"resynced {stats.resynced}")
    assert stats.resynced <= 2, stats.notes
    if rebudget_after:
        # Alg. 2 at full size: totals conserved, bounds kept, next step evicts down to the new budgets
        before = g.budgets()
        g.rebudget()
        after = g.budgets()
        assert np.array_equal(after.sum(axis=(0, 2)), before.sum(axis=(0, 2)))
        assert after.min() >= cfg.budget_min and after.max() <= cfg.budget_max
        assert not np.array_equal(after, before)
        g.decode_step(rq[n_steps], rk[n_steps], rv[n_steps])
        assert np.array_equal(g.lengths(), np.minimum(before + 1, after))
        assert g.status() == 0
    g.close()


def test_qwen7b_full_size():
    _run("qwen7b")


def test_qwen14b_full_size_bench_configuration():
    _run("qwen14b", rebudget_after=True)


def test_llama8b_full_size():
    _run("llama8b")


def test_qwen32b_full_size():
    _run("qwen32b", n_sample=6, n_steps=2, rebudget_after=True)


def test_qwen14b_full_size_one_call_per_layer_with_deferred_bookkeeping():
    """The other launch shape bench.py times: one call per layer with CKV_DEFER_BOOKKEEPING (the scan merges
    the partials of 128 units from about a thousand wavefronts; the bookkeeping of consecutive layers overlaps
    on the context's streams).  Sampled units against the oracle as above; every unit's output against a
    second, identical context stepped with the all-layers call (different kernels, same arithmetic up to
    rounding order); lengths, budgets and time of the two contexts equal after every step."""
    import torch
    import bench
    from oracle import crystal_kv as ok
    from paper_2601_16986_amd import workloads as wl

    cfg = wl.CONFIGS["qwen14b"]
    dev = torch.device("cuda:0")
    g, budgets, (rq, rk, rv) = bench.build_workload(cfg, dev)
    g_ref, _, _ = bench.build_workload(cfg, dev)
    t_now = cfg.prompt + cfg.decode_steps // 2
    flat = budgets.reshape(-1)
    idx = sorted(set([int(np.argmin(flat)), int(np.argmax(flat))] + [int(x) for x in np.linspace(0, flat.size - 1, 6).astype(int)]))
    keys = [tuple(int(v) for v in np.unravel_index(u, budgets.shape)) for u in idx]
    o = ok.CrystalKVOracle(cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, budgets,
                           lam=cfg.lam, top_p=cfg.top_p, t0=t_now, budget_min=cfg.budget_min, budget_max=cfg.budget_max)
    m = wl.mean_query(wl.scaled(cfg, n_layers=1, batch=1))
    for u, key in zip(idx, keys):
        c = wl.steady_unit(cfg, u, int(flat[u]), t_now, m[0, 0, key[2]])
        o.set_unit(key, c.K, c.V, c.pos, c.crf, c.tau)
        parity.sync_unit_to_gpu(g, o, key)
        parity.sync_unit_to_gpu(g_ref, o, key)
    stats = parity.LockstepStats()
    G = cfg.group
    for s in range(3):
        out = torch.stack([g.decode_step(rq[s, l], rk[s, l], rv[s, l], layer=l, defer=True) for l in range(cfg.n_layers)])
        ref = g_ref.decode_step(rq[s], rk[s], rv[s])
        den = torch.maximum(ref.abs(), 1e-2 * ref.abs().amax(dim=-1, keepdim=True))
        err_all = float(((out - ref).abs() / den).max())
        assert err_all <= parity.OUT_TOL, (s, err_all)
        qh, kh, vh = rq[s].float().cpu().numpy(), rk[s].float().cpu().numpy(), rv[s].float().cpu().numpy()
        outh = out.cpu().numpy()
        recs = {}
        for key in keys:
            l, b, h = key
            recs[key] = o.step_unit(key, qh[l, b, h * G:(h + 1) * G], kh[l, b, h], vh[l, b, h])
            assert parity.out_error(outh[l, b, h * G:(h + 1) * G], recs[key].y) <= parity.OUT_TOL, (key, s)
        o.t += 1
        for key in keys:
            parity.compare_unit(g, o, key, recs[key], stats, check_kv=(s == 2))
        assert np.array_equal(g.lengths(), g_ref.lengths()) and np.array_equal(g.lengths(), g.budgets())
        assert g.status() == 0 and g.time() == g_ref.time() == t_now + s + 1
        print(f"step {s}: per-layer deferred vs all-layers call over all units: max err {err_all:.2e}", flush=True)
    assert stats.resynced <= 2, stats.notes
    # and on through the rest of the benchmark's ring of inputs, context against context
    worst = 0.0
    for s in range(3, rq.shape[0]):
        out = torch.stack([g.decode_step(rq[s, l], rk[s, l], rv[s, l], layer=l, defer=True) for l in range(cfg.n_layers)])
        ref = g_ref.decode_step(rq[s], rk[s], rv[s])
        den = torch.maximum(ref.abs(), 1e-2 * ref.abs().amax(dim=-1, keepdim=True))
        worst = max(worst, float(((out - ref).abs() / den).max()))
    assert worst <= parity.OUT_TOL, worst
    assert np.array_equal(g.lengths(), g_ref.lengths()) and g.status() == 0 and g.time() == g_ref.time()
    print(f"steps 3..{rq.shape[0] - 1}: max err {worst:.2e}", flush=True)
    g.close()
    g_ref.close()
