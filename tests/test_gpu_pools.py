"""Shared pools (headroom >= 1): units own the 256-slot segments that budget + headroom entries need, Alg. 2 and
prompts move segments between units through the spare list.  Everything is checked against the oracle in lock
step, exactly as with pools that give every unit room for `cap` entries; the segment table itself is checked
for consistency (no segment owned twice, none lost)."""
import numpy as np
import pytest

from tests import parity
from tests.test_gpu_parity import _mods, _pair, _small

pytestmark = pytest.mark.gpu

SEG = 256


def _table(g):
    """(owned [units], rows [units][max_seg], spare list) read straight from the context's workspace."""
    units, max_seg = g.units, (g.cap + SEG - 1) // SEG
    info = g.segment_table()
    owned, rows, spare = info["owned"], info["rows"], info["spare"]
    assert owned.shape == (units,) and rows.shape == (units, max_seg)
    return owned, rows, spare


def _check_table(g):
    owned, rows, spare = _table(g)
    pool_segs = g.pool_slots // SEG
    held = [int(rows[u, j]) for u in range(g.units) for j in range(int(owned[u]))]
    every = held + [int(x) for x in spare]
    assert len(set(every)) == len(every), "a segment is owned twice"
    assert sorted(every) == list(range(pool_segs)), "a segment was lost"
    for u in range(g.units):
        assert np.all(rows[u, int(owned[u]):] == 0)
    n, b = g.lengths().reshape(-1), g.budgets().reshape(-1)
    assert np.all(owned * SEG >= n), "a unit holds more entries than its segments"
    return owned, n, b


@pytest.mark.parametrize("path", [1, 3])
def test_rebudget_moves_segments_between_units_and_steps_stay_in_lock_step(path):
    """Budgets around the segment size, Alg. 2 every 8 steps: units grow and shrink across the 256-entry boundary
    (asserted), the segments follow after the eviction that brings the shrunken units down, and every step
    matches the oracle, outputs, scores, evictions and budgets alike.  The pools hold what ckv_pool_slots says,
    far less than units * cap."""
    cfg = _small("qwen14b", n_layers=2, batch=2, n_q_heads=10, n_kv_heads=2, prompt=230, decode_steps=60,
                 budget=250, budget_min=40, budget_max=1023, adaptive=True, seed=91)
    budgets = np.array([[[250, 262], [240, 250]], [[258, 230], [300, 210]]], dtype=np.int32)
    st, o, g = _pair(cfg, cap=1024, budgets=budgets, path=path, headroom=1)
    assert g.pool_slots <= g.units * 1024 // 2
    owned0, _, _ = _check_table(g)
    assert owned0.tolist() == [1, 2, 1, 1, 2, 1, 2, 1]
    stats = parity.LockstepStats()
    crossed_up = crossed_down = 0
    for s in range(cfg.decode_steps):
        ref, recs = o.decode_step(st.q[s], st.k_new[s], st.v_new[s])
        out = g.decode_step(st.q[s], st.k_new[s], st.v_new[s]).cpu().numpy()
        assert parity.out_error(out, ref) <= parity.OUT_TOL
        for key, rec in recs.items():
            parity.compare_unit(g, o, key, rec, stats, check_kv=(s % 16 == 15))
        if s % 8 == 7:
            before = g.budgets().reshape(-1)
            o.rebudget()
            g.rebudget()
            after = g.budgets().reshape(-1)
            assert np.array_equal(after, o.budgets().reshape(-1))
            crossed_up += int(np.sum((before + 1 <= SEG) & (after + 1 > SEG)))
            crossed_down += int(np.sum((before + 1 > SEG) & (after + 1 <= SEG)))
        owned, n, b = _check_table(g)
        if s % 8 not in (7, 0):                     # two steps after a re-allocation everything has been handed over
            assert np.array_equal(owned, (b + 1 + SEG - 1) // SEG), (s, owned, b)
    assert crossed_up > 0 and crossed_down > 0, (crossed_up, crossed_down)
    assert stats.resynced <= 2, stats.notes
    assert g.status() == 0
    g.close()


def test_a_prompt_longer_than_the_budget_passes_through_the_spare_list():
    """Prefill layer by layer into shared pools: each layer's units borrow segments for the whole prompt, get
    their scores from the prompt's last queries, are cut to their budgets and give the segments back before
    the next layer loads.  The pools never hold more than the budgets plus one layer's prompt.  Scores,
    evictions and the decode steps that follow equal the oracle's."""
    ok, ckv, wl = _mods()
    cfg = _small("tiny", n_layers=3, batch=2, n_q_heads=8, n_kv_heads=2, prompt=700, decode_steps=12,
                 budget=200, budget_min=50, budget_max=1023, seed=93)
    budgets = np.full((3, 2, 2), 200, dtype=np.int32)
    budgets[1, 0, 1] = 300
    st = wl.make_stream(cfg)
    W = 16
    o = ok.CrystalKVOracle(cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, budgets, lam=cfg.lam,
                           top_p=cfg.top_p, t0=cfg.prompt, budget_min=cfg.budget_min, budget_max=cfg.budget_max)
    g = ckv.CrystalKV(cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, 1024, budgets, lam=cfg.lam,
                      top_p=cfg.top_p, t0=cfg.prompt, budget_min=cfg.budget_min, budget_max=cfg.budget_max,
                      headroom=1, prompt_len=cfg.prompt)
    # budgets: 12 units x 1..2 segments, + 12 spare for rounding, + 4 units x 3 segments for the prompt in flight
    assert g.pool_slots == ((200 * 11 + 300 + 12 + SEG - 1) // SEG + 12 + 4 * 3) * SEG
    rng = np.random.default_rng(5)
    for l in range(cfg.n_layers):
        q_obs = wl.bf16_round(rng.standard_normal((W, cfg.batch, cfg.n_q_heads, cfg.head_dim)).astype(np.float32))
        o.load_prompt(l, st.prompt_k[l], st.prompt_v[l])
        g.load_prompt(l, st.prompt_k[l], st.prompt_v[l])
        owned, n, b = _check_table(g)
        upl = cfg.batch * cfg.n_kv_heads
        assert np.all(owned[l * upl:(l + 1) * upl] == 3) and np.all(n[l * upl:(l + 1) * upl] == cfg.prompt)
        o.seed_prompt(l, q_obs)
        g.seed_prompt(l, q_obs)
        o.evict([(l, b_, h) for b_ in range(cfg.batch) for h in range(cfg.n_kv_heads)])
        g.evict(l)
        for b_ in range(cfg.batch):
            for h in range(cfg.n_kv_heads):
                e, u = g.export_unit(l, b_, h), o.units[(l, b_, h)]
                order = np.argsort(e["pos"][:e["n"]])
                assert e["n"] == u.n and np.array_equal(e["pos"][:e["n"]][order], np.sort(u.pos))
                uo = np.argsort(u.pos)
                assert np.array_equal(e["crf"][:e["n"]][order], u.crf[uo]) and np.array_equal(e["tau"][:e["n"]][order], u.tau[uo])
    # the last layer's surplus goes back with the first evicting step
    stats = parity.lockstep(g, o, st, cfg.decode_steps, check_kv_every=6)
    owned, n, b = _check_table(g)
    assert np.array_equal(owned, (b + 1 + SEG - 1) // SEG)
    assert stats.resynced <= 1 and g.status() == 0
    g.close()


def test_pools_too_small_are_refused_and_a_short_spare_list_is_reported():
    _, ckv, wl = _mods()
    cfg = _small("tiny", n_layers=1, batch=1, n_q_heads=4, n_kv_heads=2, prompt=100, decode_steps=4, budget=300,
                 budget_min=10, budget_max=1023, seed=7)
    budgets = np.array([[[300, 300]]], dtype=np.int32)
    with pytest.raises(ckv.CkvError) as e:
        ckv.CrystalKV(1, 1, 4, 2, 128, 1024, budgets, t0=100, budget_min=10, budget_max=1023, headroom=1, pool_slots=3 * SEG)
    assert e.value.code == ckv.EINVAL
    g = ckv.CrystalKV(1, 1, 4, 2, 128, 1024, budgets, t0=100, budget_min=10, budget_max=1023, headroom=1, pool_slots=4 * SEG)
    st = wl.make_stream(cfg)
    g.load_prompt(0, st.prompt_k[0], st.prompt_v[0])
    assert g.status() == 0
    # budgets that need six segments when the pools have four: nobody is given anything, the status says so,
    # and the units keep working within what they own
    g.set_budgets(np.array([[[700, 600]]], dtype=np.int32))
    g.rebalance()
    assert g.status() == ckv.ECAPACITY and g.status() == 0        # reported once
    owned, _, _ = _check_table(g)
    assert owned.tolist() == [2, 2]
    g.decode_step(st.q[0], st.k_new[0], st.v_new[0])
    assert g.status() == 0 and g.lengths().reshape(-1).tolist() == [101, 101]
    g.close()


def test_full_size_32b_shape_runs_in_pools_proportional_to_the_budgets():
    """The 32B-shaped workload (16384 units, budgets 512..16384, mean 4096) in shared pools: both pools together
    stay below 1.25 x the bytes of the budgeted entries (uniform capacity needs 4 x), Alg. 2 re-allocates
    nearly every budget, the segments follow, and sampled units stay in lock step with the oracle across it."""
    import torch
    import bench
    from oracle import crystal_kv as ok
    from paper_2601_16986_amd import workloads as wl
    cfg = wl.CONFIGS["qwen32b"]
    dev = torch.device("cuda:0")
    g, budgets, (rq, rk, rv) = bench.build_workload(cfg, dev)
    assert g.headroom == 1
    live = int((budgets.astype(np.int64) + 1).sum())
    assert g.pool_slots * 512 <= 1.25 * live * 512, (g.pool_slots, live)
    print(f"pools: {2 * g.pool_slots * 256 / 1e9:.1f} GB for {live * 512 / 1e9:.1f} GB of budgeted entries "
          f"(uniform capacity: {2 * g.units * ((cfg.budget_max + 256) // 256 * 256) * 256 / 1e9:.1f} GB)", flush=True)
    t_now = cfg.prompt + cfg.decode_steps // 2
    flat = budgets.reshape(-1)
    idx = [int(x) for x in np.linspace(0, flat.size - 1, 24).astype(int)]
    # whole sequences are needed for Alg. 2 on the oracle's side: take the budgets from the GPU after the
    # re-allocation instead (bit-equality of Alg. 2 at this size has its own test), and follow the sampled units
    keys = [tuple(int(v) for v in np.unravel_index(u, budgets.shape)) for u in idx]
    o = ok.CrystalKVOracle(cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, budgets, lam=cfg.lam,
                           top_p=cfg.top_p, t0=t_now, budget_min=cfg.budget_min, budget_max=cfg.budget_max)
    m = wl.mean_query(wl.scaled(cfg, n_layers=1, batch=1))
    for u, key in zip(idx, keys):
        c = wl.steady_unit(cfg, u, int(flat[u]), t_now, m[0, 0, key[2]])
        o.set_unit(key, c.K, c.V, c.pos, c.crf, c.tau)
        g.import_unit(*key, c.K, c.V, c.crf, c.tau, c.pos, t_now - 1)
    stats = parity.LockstepStats()
    G = cfg.group

    def step(s):
        out = g.decode_step(rq[s], rk[s], rv[s])
        q, kn, vn = rq[s].float().cpu().numpy(), rk[s].float().cpu().numpy(), rv[s].float().cpu().numpy()
        out = out.cpu().numpy()
        recs = {}
        for key in keys:
            l, b, h = key
            recs[key] = o.step_unit(key, q[l, b, h * G:(h + 1) * G], kn[l, b, h], vn[l, b, h])
            assert parity.out_error(out[l, b, h * G:(h + 1) * G], recs[key].y) <= parity.OUT_TOL
        o.t += 1
        for key in keys:
            parity.compare_unit(g, o, key, recs[key], stats, check_kv=False)

    for s in range(3):
        step(s)
    g.rebudget()
    new_b = g.budgets()
    assert int((new_b != budgets).sum()) > budgets.size // 2
    for key in keys:
        o.units[key].budget = int(new_b[key])
    for s in range(3, 6):
        step(s)
    owned, n, b = _check_table(g)
    assert np.array_equal(owned, (b + 1 + SEG - 1) // SEG)
    assert int((owned != (flat + 1 + SEG - 1) // SEG).sum()) > 1000          # segments did move
    assert g.status() == 0 and stats.resynced <= 3, stats.notes
    g.close()


def test_caller_owned_pools_and_a_single_arena_give_the_same_results():
    """The binding can carve all seven device buffers from one caller-owned tensor (`arena=`) or take the K and V
    pools from the caller (`pools=`): same steps, same bits as with buffers of its own."""
    import torch
    _, ckv, wl = _mods()
    cfg = _small("tiny", n_layers=2, batch=2, n_q_heads=8, n_kv_heads=2, prompt=300, decode_steps=10, budget=280,
                 budget_min=20, budget_max=511, seed=17)
    st = wl.make_stream(cfg)
    budgets = wl.draw_budgets(cfg)
    geom = (cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, 512, budgets)
    kw = dict(lam=cfg.lam, top_p=cfg.top_p, t0=cfg.prompt, budget_min=cfg.budget_min, budget_max=cfg.budget_max, headroom=1)
    dev = torch.device("cuda:0")
    need = ckv.arena_bytes(*geom, **kw)
    arena = torch.empty(need + 4096, dtype=torch.uint8, device=dev)[4096:]            # not even 2 MiB aligned
    plain = ckv.CrystalKV(*geom, **kw)
    slots = plain.pool_slots
    pools = tuple(torch.empty(slots * 128, dtype=torch.bfloat16, device=dev) for _ in range(2))
    ctxs = [plain, ckv.CrystalKV(*geom, arena=arena, **kw), ckv.CrystalKV(*geom, pools=pools, **kw)]
    assert ctxs[1].k_pool.data_ptr() >= arena.data_ptr() and ctxs[1].workspace.data_ptr() < arena.data_ptr() + arena.numel()
    assert ctxs[2].k_pool.data_ptr() == pools[0].data_ptr()
    with pytest.raises(ckv.CkvError):
        ckv.CrystalKV(*geom, arena=arena[:need // 2], **kw)
    for g in ctxs:
        for l in range(cfg.n_layers):
            g.load_prompt(l, st.prompt_k[l], st.prompt_v[l])
    for s in range(cfg.decode_steps):
        outs = [g.decode_step(st.q[s], st.k_new[s], st.v_new[s]) for g in ctxs]
        assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])
    for key in [(0, 0, 0), (1, 1, 1)]:
        es = [g.export_unit(*key, with_kv=False) for g in ctxs]
        for f in ("pos", "crf", "tau"):
            assert np.array_equal(es[0][f], es[1][f]) and np.array_equal(es[0][f], es[2][f])
    for g in ctxs:
        assert g.status() == 0
        g.close()


def test_place_pools_returns_usable_buffers_and_a_report():
    """The start-up calibration: buffers of the requested sizes come back (K and V pools, and memory for the other
    five buffers), the report says what was tried in both stages, and a context built on them gives the bits of a
    context with buffers of its own.  Pools too small to matter are simply allocated."""
    import torch
    _, ckv, wl = _mods()
    k, v, rest, rep = ckv.place_pools(8 << 20, rest_bytes=1 << 20)
    assert rep["candidates"] == 0 and k.numel() * 2 >= 8 << 20 and rest.numel() >= 1 << 20
    cfg = _small("qwen7b", n_layers=2, batch=64, n_q_heads=8, n_kv_heads=8, prompt=300, decode_steps=4, budget=2040,
                 budget_min=100, budget_max=2047, seed=21)
    st = wl.make_stream(cfg)
    budgets = wl.draw_budgets(cfg)
    geom = (cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, 2048, budgets)
    kw = dict(lam=cfg.lam, top_p=cfg.top_p, t0=cfg.prompt, budget_min=cfg.budget_min, budget_max=cfg.budget_max, headroom=1)
    plain = ckv.CrystalKV(*geom, **kw)
    ps = plain.pool_slots
    rest_bytes = ckv.arena_bytes(*geom, **kw) - 2 * ps * 256
    k, v, rest, rep = ckv.place_pools(ps * 256, rest_bytes=rest_bytes, max_fraction=0.4)
    assert 2 <= rep["candidates"] <= 48 and rep["step_ms_min"] <= rep["step_ms_chosen"] <= rep["step_ms_max"]
    assert k.numel() >= ps * 128 and v.numel() >= ps * 128 and rest.numel() >= rest_bytes
    # second stage: whole steps over pairs (pools, other buffers); the fastest pair is the one returned
    pairs = rep["whole_step_ms"]
    assert len(pairs) >= 2 and rep["rest_in"] is not None and rep["rest_in"] != rep["chosen"]
    assert pairs[f"{rep['chosen']}+{rep['rest_in']}"] == min(pairs.values())
    placed = ckv.CrystalKV(*geom, pools=(k[:ps * 128], v[:ps * 128]), arena=rest, **kw)
    for g in (plain, placed):
        for l in range(cfg.n_layers):
            g.load_prompt(l, st.prompt_k[l], st.prompt_v[l])
    for s in range(cfg.decode_steps):
        a = plain.decode_step(st.q[s], st.k_new[s], st.v_new[s])
        b = placed.decode_step(st.q[s], st.k_new[s], st.v_new[s])
        assert torch.equal(a, b)
    assert plain.status() == 0 and placed.status() == 0
    plain.close(); placed.close()
