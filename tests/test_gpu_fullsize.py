"""Parity at the full sizes of the benchmark workloads, in the launch configuration bench.py times
(all layers per call, steady-state caches built as in bench.py).

The oracle cannot step thousands of units in test time, so a sample of units is filled from the
host-side generator (the oracle and the GPU get the same arrays) and compared entry by entry for
eight decode steps: 64 units spread over the workload, the units with the smallest and the largest
budget, and (adaptive workloads) units re-sized to sit exactly at and one entry beyond each size
at which the fused kernel changes its code path.  All other units are checked through properties
that hold at any size: caches sit at their budgets after eviction, outputs are finite, no capacity
overflow, time advanced, and Alg. 2 conserves every sequence's total.  Alg. 2 itself is compared
with the oracle at the real number of (layer, head) pairs per sequence on small caches."""
import numpy as np
import pytest

from tests import parity

pytestmark = pytest.mark.gpu

N_SAMPLE = 64
N_STEPS = 8


def _lds_resident_limit(cap, G):
    """Largest entry count whose logits all stay in the fused kernel's LDS tile (4 wavefronts per unit, two
    workgroups per compute unit: 80 KB each less 11 KB of static arrays, the eviction bit mask and two rows of
    the segment table).  The test asserts below that the context reports the tile size assumed here."""
    lds_main = (80 * 1024 - 11 * 1024 - (cap + 31) // 32 * 4 - 2 * ((cap + 255) // 256) * 4) & ~127
    n = 32
    while (n + 32) * G * 4 <= lds_main:
        n += 32
    return n, lds_main


def _sample(cfg, budgets, n_sample, boundaries):
    """Unit indices to compare entry by entry: the smallest and the largest budget, `n_sample` units spread
    over the index range, and units re-sized to sit just under and just over the kernel's internal size
    limits (their budgets are overwritten in `budgets`; a limit n means n entries while attending)."""
    flat = budgets.reshape(-1)
    spread = [int(x) for x in np.linspace(0, flat.size - 1, n_sample).astype(int)]
    taken = set(spread)
    placed = []
    u = 1
    for n_att in boundaries:
        for b in (n_att - 1, n_att):               # budget n - 1 attends over n entries: at the limit, and one over it
            if not (cfg.budget_min <= b <= cfg.budget_max):
                continue
            while u in taken:
                u += 7
            flat[u] = b
            taken.add(u)
            placed.append(u)
    idx = sorted(taken | {int(np.argmin(flat)), int(np.argmax(flat))})
    return idx, placed


def _run(name, n_sample=N_SAMPLE, n_steps=N_STEPS, rebudget_after=None, boundaries=()):
    import torch
    import bench
    from oracle import crystal_kv as ok
    from paper_2601_16986_amd import workloads as wl

    cfg = wl.CONFIGS[name]
    dev = torch.device("cuda:0")
    budgets = wl.draw_budgets(cfg).copy()
    cap = (cfg.budget_max + 1 + 31) // 32 * 32
    n_lds, lds_main = _lds_resident_limit(cap, cfg.group)
    limits = [b for b in boundaries] + ([n_lds] if boundaries else [])
    idx, placed = _sample(cfg, budgets, n_sample, limits)
    g, budgets, (rq, rk, rv) = bench.build_workload(cfg, dev, budgets=budgets)
    waves, lds_ctx = g.path_info()
    assert waves == 4 and lds_ctx == lds_main, (waves, lds_ctx, lds_main)
    t_now = cfg.prompt + cfg.decode_steps // 2
    flat = budgets.reshape(-1)
    keys = [tuple(int(v) for v in np.unravel_index(u, budgets.shape)) for u in idx]
    print(f"{name}: {len(keys)} sampled units, budgets {int(flat[idx].min())}..{int(flat[idx].max())}, "
          f"units at size limits {sorted(int(flat[u]) for u in placed)}", flush=True)
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
            stats.unit_steps += 1
        # properties over every unit
        assert np.isfinite(outh).all()
        assert np.array_equal(g.lengths(), g.budgets())
        assert g.status() == 0 and g.time() == t_now + s + 1
        print(f"  step {s}: {len(keys)} units equal the oracle, max out err so far {stats.max_out_err:.2e}", flush=True)
    print(f"{name}: {len(keys)} sampled units x {n_steps} steps, max out err {stats.max_out_err:.2e}, "
          f"resynced {stats.resynced} {stats.notes}")
    assert stats.resynced <= max(2, stats.unit_steps // 200), stats.notes
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


# entries per unit at which the fused kernel changes its code path: 8, 16 and 32 entries per thread of a
# 256-thread workgroup (the LDS tile's limit is added by _run)
THREAD_LIMITS = (2048, 4096, 8192)


def test_qwen7b_full_size():
    _run("qwen7b")


def test_qwen14b_full_size_bench_configuration():
    _run("qwen14b", rebudget_after=True, boundaries=THREAD_LIMITS)


def test_llama8b_full_size():
    _run("llama8b")


def test_qwen32b_full_size():
    _run("qwen32b", rebudget_after=True, boundaries=THREAD_LIMITS)


@pytest.mark.parametrize("n_layers", [48, 64])
def test_rebudget_at_the_real_head_count_matches_oracle_with_active_bounds(n_layers):
    """Alg. 2 at the problem size of the 14B and 32B shapes, L x H = 384 and 512 (layer, head) pairs per
    sequence (the kernel's per-layer threads and its serial layer-level apportionment at their real
    trip counts), on caches small enough for the oracle to step every unit: budgets bit-equal to the
    oracle's after lock-step decoding, totals conserved, and both a lower and an upper bound active
    in the result (the budget range is narrow, so the utilisations' spread reaches both)."""
    from oracle import crystal_kv as ok
    from paper_2601_16986_amd import ckv, workloads as wl
    cfg = wl.scaled(wl.CONFIGS["qwen14b"], n_layers=n_layers, batch=2, prompt=30, decode_steps=16, budget=24,
                    budget_min=21, budget_max=27, adaptive=True, seed=880 + n_layers)
    st = wl.make_stream(cfg)
    budgets = wl.draw_budgets(cfg)
    assert budgets.min() == 21 and budgets.max() == 27
    o = ok.CrystalKVOracle(cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, budgets, lam=cfg.lam,
                           top_p=cfg.top_p, t0=cfg.prompt, budget_min=cfg.budget_min, budget_max=cfg.budget_max)
    g = ckv.CrystalKV(cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, 64, budgets, lam=cfg.lam,
                      top_p=cfg.top_p, t0=cfg.prompt, budget_min=cfg.budget_min, budget_max=cfg.budget_max)
    for l in range(cfg.n_layers):
        o.load_prompt(l, st.prompt_k[l], st.prompt_v[l])
        g.load_prompt(l, st.prompt_k[l], st.prompt_v[l])
    total0 = budgets.sum(axis=(0, 2))
    step = 0
    for rnd in range(2):
        stats = parity.lockstep(g, o, st_slice(st, step, 8), 8)
        step += 8
        assert stats.resynced == 0, "window sums are only comparable without re-synchronised units"
        nb = o.rebudget()
        g.rebudget()
        gb = g.budgets()
        assert np.array_equal(gb, nb), np.argwhere(gb != nb)[:10]
        assert np.array_equal(gb.sum(axis=(0, 2)), total0)
        for b in range(cfg.batch):
            assert gb[:, b].min() == cfg.budget_min and gb[:, b].max() == cfg.budget_max, (gb[:, b].min(), gb[:, b].max())
        # and the layer level: some layer of every sequence sits at H b_min or H b_max only if its heads all do;
        # what must hold is that layer totals stay inside [H b_min, H b_max]
        lt = gb.sum(axis=2)
        assert lt.min() >= cfg.n_kv_heads * cfg.budget_min and lt.max() <= cfg.n_kv_heads * cfg.budget_max
        print(f"L x H = {n_layers * cfg.n_kv_heads}: round {rnd}, budgets equal the oracle's, "
              f"{int((gb == cfg.budget_min).sum())} at the lower and {int((gb == cfg.budget_max).sum())} at the upper bound", flush=True)
    g.close()


def st_slice(st, first, count):
    """The decode steps [first, first + count) of a stream, as a stream of its own."""
    from dataclasses import replace
    return replace(st, q=st.q[first:first + count], k_new=st.k_new[first:first + count], v_new=st.v_new[first:first + count])


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


def test_seed_prompt_at_the_bench_geometry_sampled_units():
    """ckv_seed_prompt in the configuration `bench.py --seed-prompt 9350,32` times (14B geometry: 48 layers, so
    the replay takes all 11 query tiles of the window in one batch and one pass over the keys; 128 units per
    layer; 9350 entries per unit, i.e. 32 entries per thread of the rewards kernel and a short list of more
    than 64 candidates): eight units of the layer, spread over it, against the oracle entry by entry (CRF bits
    and tau; entries at the edge of a sub-margin top-p decision of the window may differ), every other unit's
    scores finite, non-negative and with tau within the window or at the entry's own position."""
    import math
    import torch
    from oracle import crystal_kv as ok
    from paper_2601_16986_amd import ckv, workloads as wl
    cfg = wl.CONFIGS["qwen14b"]
    dev = torch.device("cuda:0")
    P, W, layer = 9350, 32, 0
    G = cfg.group
    budgets = np.full((cfg.n_layers, cfg.batch, cfg.n_kv_heads), P, dtype=np.int32)
    cap = (P + 64) // 32 * 32
    g = ckv.CrystalKV(cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cap, budgets,
                      lam=cfg.lam, top_p=cfg.top_p, t0=P, budget_min=1, budget_max=cap - 1, device=dev)
    m = wl.torch_mean_query(cfg, dev)
    gen = wl.torch_generator(cfg, 9, dev)
    r_now = math.sqrt(wl.DRIFT_VAR) * torch.randn(m.shape, generator=gen, device=dev)
    k, v, *_ = wl.torch_steady_layer(cfg, layer, budgets[layer], P, m[layer], r_now[layer], dev)
    g.load_prompt(layer, k, v)
    q_obs = (torch.randn((W, cfg.batch, cfg.n_q_heads, cfg.head_dim), generator=gen, device=dev)
             + m[layer].repeat_interleave(G, dim=1)[None]).to(torch.bfloat16)
    g.seed_prompt(layer, q_obs)
    torch.cuda.synchronize()
    assert g.status() == 0 and g.time() == P
    # the sampled units in an oracle of their own: one sequence whose KV heads are the sampled units
    units = [(int(u) // cfg.n_kv_heads, int(u) % cfg.n_kv_heads) for u in np.linspace(0, cfg.batch * cfg.n_kv_heads - 1, 8).astype(int)]
    S = len(units)
    o = ok.CrystalKVOracle(1, 1, S * G, S, cfg.head_dim, np.full((1, 1, S), P, dtype=np.int32), lam=cfg.lam, top_p=cfg.top_p,
                           t0=P, budget_min=1, budget_max=cap - 1)
    kh, vh, qh = k.float().cpu().numpy(), v.float().cpu().numpy(), q_obs.float().cpu().numpy()
    q_o = np.zeros((W, 1, S * G, cfg.head_dim), dtype=np.float32)
    for i, (b, h) in enumerate(units):
        o.set_unit((0, 0, i), kh[b, h], vh[b, h], np.arange(P), np.ones(P, np.float32), np.full(P, P - 1))
        q_o[:, 0, i * G:(i + 1) * G] = qh[:, b, h * G:(h + 1) * G]
    decs = o.seed_prompt(0, q_o)
    n_sub = 0
    for i, (b, h) in enumerate(units):
        u, e = o.units[(0, 0, i)], g.export_unit(layer, b, h, with_kv=False)
        assert e["n"] == P and np.array_equal(e["pos"], u.pos)
        if np.array_equal(e["crf"].view(np.uint32), u.crf.view(np.uint32)) and np.array_equal(e["tau"], u.tau):
            continue
        sub = [d for d in decs[(0, 0, i)] if min(d.sum_margin, d.edge_gap) < parity.MARGIN_TOL]
        may = set(j for d in sub for j in parity.edge_entries(d))
        differ = set(np.nonzero((e["crf"].view(np.uint32) != u.crf.view(np.uint32)) | (e["tau"] != u.tau))[0].tolist())
        assert sub and differ <= may, ((b, h), sorted(differ)[:20], sorted(may)[:20])
        n_sub += 1
    print(f"seed at the bench geometry: {S} units equal the oracle ({n_sub} through a sub-margin decision)")
    assert n_sub <= 2
    for b in range(cfg.batch):
        for h in range(cfg.n_kv_heads):
            e = g.export_unit(layer, b, h, with_kv=False)
            assert e["n"] == P and np.isfinite(e["crf"]).all() and (e["crf"] >= 0).all()
            assert np.all((e["tau"] == np.arange(P)) | ((e["tau"] >= P - W) & (e["tau"] <= P - 1)))
    g.close()
