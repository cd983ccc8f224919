"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests re-types the oracle's own formulas: each compares it with
a hand-computed fixture, a closed form, a library routine, brute force on tiny
inputs, or an invariant.
"""
import itertools
import json
import math
import os

import numpy as np
import pytest

from oracle import crystal_kv as ok
from paper_2601_16986_amd import workloads as wl


# ------------------------------------------------------------------ attention
def test_attention_equals_library_sdpa_when_nothing_is_evicted():
    """Sec. 2.2: with a budget above the token count the path is ordinary softmax
    attention over all tokens; torch's SDPA (float64, KV heads repeated for GQA)
    is the library routine."""
    import torch
    import torch.nn.functional as F
    cfg = wl.scaled(wl.CONFIGS["tiny"], prompt=9, decode_steps=7, budget=1000, budget_min=1, budget_max=1000)
    st = wl.make_stream(cfg, tiny_heavy=False)
    o = ok.CrystalKVOracle(1, 1, 8, 2, 128, np.full((1, 1, 2), 1000), lam=0.5, top_p=0.9, t0=9)
    o.load_prompt(0, st.prompt_k[0], st.prompt_v[0])
    for s in range(7):
        out, _ = o.decode_step(st.q[s], st.k_new[s], st.v_new[s])
        K = np.concatenate([st.prompt_k[0, 0], np.moveaxis(st.k_new[:s + 1, 0, 0], 0, 1)], axis=1)  # [Hkv][n][d]
        V = np.concatenate([st.prompt_v[0, 0], np.moveaxis(st.v_new[:s + 1, 0, 0], 0, 1)], axis=1)
        Kt = torch.from_numpy(K.astype(np.float64)).repeat_interleave(4, dim=0)[None]      # [1][Hq][n][d]
        Vt = torch.from_numpy(V.astype(np.float64)).repeat_interleave(4, dim=0)[None]
        qt = torch.from_numpy(st.q[s, 0, 0].astype(np.float64))[None, :, None, :]          # [1][Hq][1][d]
        ref = F.scaled_dot_product_attention(qt, Kt, Vt, scale=o.scale)[0, :, 0, :].numpy()
        assert np.allclose(out[0, 0], ref, rtol=1e-12, atol=1e-13)
    assert o.lengths()[0, 0, 0] == 9 + 7


def test_softmax_rows_sum_to_one_and_slot_order_is_irrelevant():
    g = np.random.default_rng(1)
    q, K, V = g.standard_normal((5, 128)), g.standard_normal((300, 128)), g.standard_normal((300, 128))
    y, a = ok.attention(q, K, V, 0.0884)
    assert np.all(np.abs(a.sum(axis=1) - 1.0) < 1e-12)
    assert np.all(a >= 0)
    perm = g.permutation(300)
    y2, a2 = ok.attention(q, K[perm], V[perm], 0.0884)
    assert np.allclose(y, y2, rtol=1e-12, atol=1e-14)
    assert np.allclose(a[:, perm], a2, rtol=1e-12, atol=1e-300)


def test_attention_single_entry_returns_its_value():
    q, K, V = np.ones((3, 4)), np.array([[1.0, 2, 3, 4]]), np.array([[9.0, 8, 7, 6]])
    y, a = ok.attention(q, K, V, 0.5)
    assert np.array_equal(a, np.ones((3, 1)))
    assert np.array_equal(y, np.tile(V, (3, 1)))


def test_attention_two_entries_closed_form():
    # logits 0 and ln 3 -> weights 1/4 and 3/4
    q = np.array([[1.0, 0.0]])
    K = np.array([[0.0, 5.0], [math.log(3.0), -2.0]])
    V = np.array([[4.0, 0.0], [0.0, 8.0]])
    y, a = ok.attention(q, K, V, 1.0)
    assert np.allclose(a, [[0.25, 0.75]], rtol=1e-15)
    assert np.allclose(y, [[1.0, 6.0]], rtol=1e-15)


# -------------------------------------------------------------------- top-p
def brute_force_nucleus(abar, pos, p):
    """Smallest prefix of the (weight desc, pos asc) order whose sum exceeds p,
    found by trying every subset size and every subset (tiny n only)."""
    n = len(abar)
    best = None
    for size in range(1, n + 1):
        cands = [s for s in itertools.combinations(range(n), size) if sum(abar[i] for i in s) > p]
        if cands:
            # among subsets of minimal size take the one the ordering prefers:
            # largest weights first, lower position on equal weight
            key = lambda s: sorted((-abar[i], pos[i]) for i in s)
            best = min(cands, key=key)
            break
    return set(range(n)) if best is None else set(best)


@pytest.mark.parametrize("seed", range(20))
def test_hit_mask_matches_subset_brute_force(seed):
    g = np.random.default_rng(seed)
    n = int(g.integers(1, 10))
    abar = g.random(n) ** 3
    if seed % 3 == 0 and n > 2:            # force exact ties
        abar[1] = abar[0]
    abar = abar / abar.sum()
    pos = g.permutation(50)[:n]
    p = float(g.choice([0.3, 0.5, 0.6, 0.9, 0.99]))
    d = ok.hit_mask(abar, pos, p)
    assert set(np.nonzero(d.hit)[0]) == brute_force_nucleus(list(abar), list(pos), p)


def test_hit_mask_minimality_and_limits():
    g = np.random.default_rng(7)
    abar = g.random(500) ** 4
    abar /= abar.sum()
    pos = np.arange(500)
    for p in (0.5, 0.9):
        d = ok.hit_mask(abar, pos, p)
        s = abar[d.hit].sum()
        assert s > p
        assert s - abar[d.hit].min() <= p          # dropping the smallest hit falls to <= p
        assert abar[d.hit].min() >= abar[~d.hit].max()
    # p -> 0+: only the arg-max (plus the new entry); p >= 1: everything
    d = ok.hit_mask(abar, pos, 1e-12, new_index=499)
    assert set(np.nonzero(d.hit)[0]) == {int(np.argmax(abar)), 499}
    assert ok.hit_mask(abar, pos, 1.0).hit.all()
    assert ok.hit_mask(abar, pos, 1.5).hit.all()


def test_hit_mask_strict_threshold_and_position_tie_break():
    # cumulative weight equal to p does not "exceed" it
    d = ok.hit_mask(np.array([0.5, 0.25, 0.25]), np.array([0, 1, 2]), 0.5)
    assert d.hit.tolist() == [True, True, False]
    # equal weights: the lower position comes first whatever the slot order
    d = ok.hit_mask(np.array([0.25, 0.5, 0.25]), np.array([9, 5, 3]), 0.5)
    assert d.hit.tolist() == [False, True, True]


# ---------------------------------------------------------------------- CRF
@pytest.mark.parametrize("lam", [0.0, 0.3, 0.5, 0.7, 0.95, 1.0])
def test_incremental_crf_equals_closed_form_from_hit_history(lam):
    """Sec. 5.2: the incremental rule must reproduce CRF = sum_j lambda^(t - t_j)."""
    g = np.random.default_rng(11)
    n, T = 40, 120
    tab = ok.decay_table(lam)
    crf = np.zeros(n, np.float32)
    birth = g.integers(0, 20, size=n)
    tau = birth.copy()
    history = [[] for _ in range(n)]
    for t in range(T):
        alive = birth <= t
        hit = (g.random(n) < 0.15) & alive
        hit |= birth == t                         # arrival is a reference
        for i in np.nonzero(hit)[0]:
            history[i].append(t)
        tmp, crf2, tau2 = ok.crf_update(np.where(alive, crf, 0), np.where(alive, tau, t), t,
                                        hit.astype(np.float32), hit, tab)
        crf = np.where(alive, crf2, crf).astype(np.float32)
        tau = np.where(alive, tau2, tau)
        for i in np.nonzero(alive)[0]:
            ref = ok.crf_closed_form(history[i], t, lam)
            assert abs(float(tmp[i]) - ref) <= 1e-5 * max(ref, 1e-30) + 1e-37
        if lam < 1.0:
            assert float(tmp.max()) <= 1.0 / (1.0 - lam) * (1 + 1e-5)
        assert float(tmp.min()) >= 0.0


def test_unaccessed_entry_decays_geometrically():
    tab = ok.decay_table(0.7)
    for dt in (0, 1, 5, 40):
        tmp, crf, tau = ok.crf_update(np.array([2.5], np.float32), np.array([10]), 10 + dt,
                                      np.zeros(1, np.float32), np.zeros(1, bool), tab)
        assert tmp[0] == pytest.approx(2.5 * float(np.float32(0.7)) ** dt, rel=2e-7)
        assert crf[0] == np.float32(2.5) and tau[0] == 10       # a miss records nothing


def test_lambda_one_is_lfu_and_lambda_zero_is_lru():
    """Sec. 5.2: lambda = 1 counts hits exactly; lambda = 0 scores only the current hits."""
    g = np.random.default_rng(5)
    n, T = 30, 200
    for lam in (1.0, 0.0):
        tab = ok.decay_table(lam)
        crf, tau = np.zeros(n, np.float32), np.zeros(n, np.int64)
        count = np.zeros(n, np.int64)
        for t in range(T):
            hit = g.random(n) < 0.3
            count += hit
            tmp, crf, tau = ok.crf_update(crf, tau, t, hit.astype(np.float32), hit, tab)
            if lam == 1.0:
                assert np.array_equal(tmp, count.astype(np.float32))
            else:
                assert np.array_equal(tmp, hit.astype(np.float32))
        if lam == 1.0:
            # eviction with lambda = 1 drops the least frequently hit entries
            retain, evicted = ok.evict_select(tmp, np.arange(n), 20)
            assert count[evicted].max() <= count[retain].min()


def test_decay_table_shape():
    t = ok.decay_table(0.5)
    assert t[0] == 1 and t[1] == 0.5 and t[126] == np.float32(2.0 ** -126) and t[-1] == 0 and len(t) == 128
    assert ok.decay_table(1.0).tolist() == [1.0]
    assert ok.decay_table(0.0).tolist() == [1.0, 0.0]
    t = ok.decay_table(0.9)
    assert np.all(np.diff(t) < 0) and t[-1] == 0 and t[-2] >= ok.FLT_MIN


# ----------------------------------------------------------------- eviction
@pytest.mark.parametrize("seed", range(10))
def test_evict_select_against_full_sort(seed):
    g = np.random.default_rng(100 + seed)
    n = int(g.integers(2, 12))
    B = int(g.integers(1, n))
    tmp = g.choice([0.0, 0.25, 0.5, 1.0, 1.5], size=n).astype(np.float32)     # many ties
    pos = g.permutation(100)[:n]
    retain, evicted = ok.evict_select(tmp, pos, B)
    assert len(retain) == B and len(evicted) == n - B
    # brute force: every evicted key must not beat any kept key under (score, -position)
    for i in retain:
        for j in evicted:
            assert (tmp[i], -pos[i]) > (tmp[j], -pos[j])
    # python's own sort as the textbook routine
    ranked = sorted(range(n), key=lambda i: (-float(tmp[i]), int(pos[i])))
    assert sorted(ranked[:B]) == retain.tolist()


def test_evict_tie_keeps_lower_position_and_noop_within_budget():
    retain, evicted = ok.evict_select(np.array([1, 1, 1], np.float32), np.array([7, 3, 5]), 2)
    assert retain.tolist() == [1, 2] and evicted.tolist() == [0]
    retain, evicted = ok.evict_select(np.array([1, 2], np.float32), np.array([0, 1]), 2)
    assert retain.tolist() == [0, 1] and evicted.size == 0


# -------------------------------------------------------- whole Alg. 1 trace
def test_alg1_hand_worked_trace(golden_dir):
    fx = json.load(open(os.path.join(golden_dir, "alg1_trace_8tok.json")))
    lam, p, B = fx["lambda"], fx["top_p"], fx["budget"]
    tab = ok.decay_table(lam)
    pos = np.zeros(0, np.int64)
    crf = np.zeros(0, np.float32)
    tau = np.zeros(0, np.int64)
    for st in fx["steps"]:
        t = st["t"]
        pos, crf, tau = np.append(pos, t), np.append(crf, np.float32(0)), np.append(tau, t)
        assert pos.tolist() == st["live"]
        d = ok.hit_mask(np.array(st["abar"]), pos, p, new_index=len(pos) - 1)
        assert sorted(pos[d.hit].tolist()) == st["hit"]
        tmp, crf, tau = ok.crf_update(crf, tau, t, d.hit.astype(np.float32), d.hit, tab)
        for k, (c, tt) in st["stored"].items():
            i = int(np.nonzero(pos == int(k))[0][0])
            assert float(crf[i]) == c and int(tau[i]) == tt and float(tmp[i]) == c
        for k, c in st["tmp_miss"].items():
            i = int(np.nonzero(pos == int(k))[0][0])
            assert float(tmp[i]) == c
            assert float(crf[i]) != c or int(tau[i]) == t or c == 0    # a miss does not record
        retain, evicted = ok.evict_select(tmp, pos, B)
        assert sorted(pos[evicted].tolist()) == st["evict"]
        pos, crf, tau = pos[retain], crf[retain], tau[retain]
    assert pos.tolist() == fx["final_retained"]
    # the survivors carry their stored score, not the temporary one (Alg. 1 gathers CRF)
    assert crf.tolist() == [1.140625, 1.5, 1.0, 1.0] and tau.tolist() == [7, 6, 6, 7]


def test_oracle_class_runs_the_same_trace_through_real_attention():
    """The class drives append -> attend -> Alg. 1.  With d = 8 one-hot keys
    and a query whose logits are the logs of the fixture's weights, attention
    reproduces the fixture's weights, so the class must reproduce its evictions."""
    fx = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "alg1_trace_8tok.json")))
    o = ok.CrystalKVOracle(1, 1, 1, 1, 8, np.full((1, 1, 1), fx["budget"]), lam=fx["lambda"],
                           top_p=fx["top_p"], softmax_scale=1.0, t0=0)
    for st in fx["steps"]:
        t = st["t"]
        k_new = np.zeros(8)
        k_new[t] = 1.0                      # entry of position t answers on coordinate t
        q = np.full(8, -1e4)
        for ppos, w in zip(st["live"], st["abar"]):
            q[ppos] = math.log(w)
        rec = o.step_unit((0, 0, 0), q[None, :], k_new, np.arange(8.0) + t)
        assert np.allclose(rec.abar, st["abar"], rtol=1e-12)
        assert rec.evicted_pos.tolist() == st["evict"]
        o.t += 1
    assert o.units[(0, 0, 0)].pos.tolist() == fx["final_retained"]


# -------------------------------------------------------------------- Alg. 2
def test_alg2_hand_example(golden_dir):
    fx = json.load(open(os.path.join(golden_dir, "alg2_example.json")))
    Bl, Bh = ok.budget_shares(fx["CRF"], fx["B"], fx["B_total"])
    assert np.allclose(Bl, fx["B_layer"], rtol=1e-14)
    assert np.allclose(Bh, fx["B_new"], rtol=1e-14)
    newB = ok.rebudget(np.array(fx["CRF"], float), np.array(fx["B"]), fx["B_total"], 1, 400)
    assert newB.tolist() == fx["B_new"]


@pytest.mark.parametrize("seed", range(8))
def test_alg2_invariants(seed):
    g = np.random.default_rng(seed)
    L, H = int(g.integers(1, 7)), int(g.integers(1, 9))
    B = g.integers(50, 500, size=(L, H))
    C = g.random((L, H)) * 100
    tot = int(B.sum())
    Bl, Bh = ok.budget_shares(C, B, tot)
    assert abs(Bh.sum() - tot) < 1e-9 * tot and np.allclose(Bh.sum(axis=1), Bl)
    Bl2, Bh2 = ok.budget_shares(C * 37.0, B, tot)                      # scale invariance
    assert np.allclose(Bh, Bh2, rtol=1e-12)
    newB = ok.rebudget(C, B, tot, 10, 5000)
    assert int(newB.sum()) == tot and newB.min() >= 10 and newB.max() <= 5000
    # with no bound active the integers are the real shares rounded down or up
    if Bh.min() > 11 and Bh.max() < 4999:
        assert np.all(np.abs(newB - Bh) < 1.0 + 1e-9 + L)     # layer rounding moves heads by < 1 + L/H
    # equal utilisation everywhere -> budgets proportional to... themselves being uniform
    U = np.full((L, H), 123)
    same = ok.rebudget(np.full((L, H), 5.0), U, int(U.sum()), 1, 10 ** 6)
    assert np.array_equal(same, U)


def test_alg2_degenerate_inputs_keep_budgets():
    B = np.array([[100, 200], [300, 400]])
    assert np.array_equal(ok.rebudget(np.zeros((2, 2)), B, 1000, 1, 1000), B)


def test_apportion_properties():
    assert ok.apportion([1, 1, 1], 10, [0] * 3, [10] * 3) == [4, 3, 3]       # remainder to the lowest index
    assert ok.apportion([3, 1], 8, [0, 0], [8, 8]) == [6, 2]
    assert ok.apportion([100, 1, 1], 10, [2] * 3, [5] * 3) == [5, 3, 2]       # water-filling under an upper bound
    assert ok.apportion([0, 0], 7, [0, 0], [9, 9]) == [4, 3]                 # no weight: equal shares
    assert ok.apportion([5, 0], 10, [2, 2], [9, 9]) == [8, 2]                # lower bound
    g = np.random.default_rng(3)
    for _ in range(200):
        m = int(g.integers(1, 12))
        lo = g.integers(0, 5, size=m)
        hi = lo + g.integers(0, 50, size=m)
        tot = int(g.integers(lo.sum(), hi.sum() + 1))
        x = g.random(m) * (g.random(m) < 0.8)
        v = ok.apportion(list(x), tot, lo, hi)
        assert sum(v) == tot and all(lo[k] <= v[k] <= hi[k] for k in range(m))
    with pytest.raises(ValueError):
        ok.apportion([1, 1], 100, [0, 0], [10, 10])


# -------------------------------------------------------------- probe classes
def test_probe_classes_counts_and_order():
    g = np.random.default_rng(9)
    for n in (1, 3, 10, 57):
        abar = g.random(n)
        pos = g.permutation(1000)[:n]
        cls = ok.probe_classes(abar, pos)
        k = (3 * n) // 10
        assert (cls == ok.CLASS_CRYSTAL).sum() == k and (cls == ok.CLASS_SLIP).sum() == k
        ranked = sorted(range(n), key=lambda i: (-abar[i], pos[i]))
        assert all(cls[i] == ok.CLASS_CRYSTAL for i in ranked[:k])
        assert all(cls[i] == ok.CLASS_SLIP for i in ranked[n - k:] if k)


# ------------------------------------------------------------ end to end tiny
def test_tiny_workload_invariants_and_heavy_survival(golden_dir):
    """Tiny workload, all 512 steps: per-head kept count == budget once full,
    scores within [0, 1/(1-lambda)], and the 4 heavy positions per head, which
    draw attention throughout, are never evicted.  The final cache size
    reproduces Table 1's 'HBM saving' closed form 1 - budget/length."""
    cfg = wl.CONFIGS["tiny"]
    st = wl.make_stream(cfg)
    o = ok.CrystalKVOracle(cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                           wl.draw_budgets(cfg), lam=cfg.lam, top_p=cfg.top_p, t0=cfg.prompt)
    o.load_prompt(0, st.prompt_k[0], st.prompt_v[0])
    for s in range(cfg.decode_steps):
        out, recs = o.decode_step(st.q[s], st.k_new[s], st.v_new[s])
        for key, r in recs.items():
            u = o.units[key]
            assert u.n == min(cfg.prompt + s + 1, cfg.budget)
            assert len(r.evicted_pos) == max(0, cfg.prompt + s + 1 - cfg.budget) - max(0, cfg.prompt + s - cfg.budget)
            assert float(r.tmp.max()) <= 2.0 + 1e-6 and float(r.tmp.min()) >= 0.0
            assert abs(r.abar.sum() - 1.0) < 1e-12
    for (l, b, h), u in o.units.items():
        heavy_pos = np.nonzero(st.heavy[l, b, h])[0]
        assert set(heavy_pos.tolist()) <= set(u.pos.tolist())
    total = cfg.prompt + cfg.decode_steps
    saving = 100.0 * (1.0 - o.lengths()[0, 0, 0] / total)
    assert saving == pytest.approx(100.0 * (1 - 128 / 576))
    fx = json.load(open(os.path.join(golden_dir, "table1_hbm_saving.json")))
    for row in fx["rows"]:
        assert round(100.0 * (1.0 - row["budget"] / row["gen_len"]), 2) == pytest.approx(row["saving_percent"], abs=0.006)


# ------------------------------------------------------------------ prompt scores
def _seed_case(seed, P=37, W=9, lam=0.6, top_p=0.9, hq=8, hkv=2):
    cfg = wl.scaled(wl.CONFIGS["tiny"], n_layers=1, batch=2, n_q_heads=hq, n_kv_heads=hkv, prompt=P, decode_steps=W,
                    budget=1000, budget_min=1, budget_max=1000, seed=seed)
    st = wl.make_stream(cfg)
    q_obs = st.q[:W, 0]                                   # any W queries: [W][Bz][Hq][d]
    return cfg, st, q_obs


@pytest.mark.parametrize("seed,lam", [(3, 0.6), (4, 0.0), (5, 1.0), (6, 0.93)])
def test_seed_prompt_equals_decoding_the_window_without_eviction(seed, lam):
    """The reading behind `seed_prompt`: the prompt's last W positions are W decode steps that already
    happened.  Loading only the first P - W tokens (each referenced once, on arrival) and decoding the
    other W tokens with the same queries, nothing evicted, must leave the same scores.  The two routes
    share `attention`, `hit_mask` and `crf_update` but not the bookkeeping around them (append and time
    there, prefix views here)."""
    P, W = 37, 9
    cfg, st, q_obs = _seed_case(seed, P, W, lam)
    big = np.full((1, 2, 2), 1000)
    a = ok.CrystalKVOracle(1, 2, 8, 2, 128, big, lam=lam, top_p=0.9, t0=P)
    a.load_prompt(0, st.prompt_k[0], st.prompt_v[0])
    a.seed_prompt(0, q_obs)
    b = ok.CrystalKVOracle(1, 2, 8, 2, 128, big, lam=lam, top_p=0.9, t0=P - W)
    head = np.arange(P - W)
    b.load_prompt(0, st.prompt_k[0][:, :, :P - W], st.prompt_v[0][:, :, :P - W],
                  crf0=np.ones((2, 2, P - W), np.float32), tau0=np.broadcast_to(head, (2, 2, P - W)))
    for j in range(W):
        k_new = st.prompt_k[:, :, :, P - W + j]           # [L][Bz][Hkv][d]
        v_new = st.prompt_v[:, :, :, P - W + j]
        b.decode_step(q_obs[j][None], k_new, v_new, evict=False)
    assert b.t == P
    for key in a.units:
        ua, ub = a.units[key], b.units[key]
        assert np.array_equal(ua.pos, ub.pos)
        assert np.array_equal(ua.crf.view(np.uint32), ub.crf.view(np.uint32)) and np.array_equal(ua.tau, ub.tau)
        assert ua.crf_window == 0                          # nothing of the replay reaches Alg. 2's window


def test_seed_prompt_scores_are_the_closed_form_over_the_hit_times():
    """Sec. 5.2: CRF = sum_j lambda^(t - t_j) over the entry's reference times, here its arrival (entries
    of the window and before alike) plus every window query that hit it, evaluated at the last of them."""
    P, W, lam = 41, 12, 0.7
    cfg, st, q_obs = _seed_case(11, P, W, lam)
    o = ok.CrystalKVOracle(1, 2, 8, 2, 128, np.full((1, 2, 2), 1000), lam=lam, top_p=0.9, t0=P)
    o.load_prompt(0, st.prompt_k[0], st.prompt_v[0])
    decs = o.seed_prompt(0, q_obs)
    for key, u in o.units.items():
        for i in range(P):
            times = [i] + [P - W + j for j, dcs in enumerate(decs[key])
                           if i < len(dcs.hit) and dcs.hit[i] and P - W + j != i]
            assert u.tau[i] == max(times)
            want = sum(lam ** (max(times) - tj) for tj in times)
            assert abs(float(u.crf[i]) - want) <= 1e-5 * want


def test_seed_prompt_limits_lru_lfu_and_single_query():
    """lambda = 0: only the last reference counts (CRF = 1, tau = last hit); lambda = 1: CRF = number of
    references; W = 1: the last query's nucleus and the last token itself are the only entries touched."""
    P, W = 33, 8
    cfg, st, q_obs = _seed_case(21, P, W)
    for lam in (0.0, 1.0):
        o = ok.CrystalKVOracle(1, 2, 8, 2, 128, np.full((1, 2, 2), 1000), lam=lam, top_p=0.9, t0=P)
        o.load_prompt(0, st.prompt_k[0], st.prompt_v[0])
        decs = o.seed_prompt(0, q_obs)
        for key, u in o.units.items():
            nhits = np.ones(P, np.int64)
            for j, dcs in enumerate(decs[key]):
                h = np.zeros(P, bool)
                h[:len(dcs.hit)] = dcs.hit
                h[P - W + j] = False                       # the arrival is already counted
                nhits += h
            assert np.array_equal(u.crf, np.ones(P, np.float32) if lam == 0.0 else nhits.astype(np.float32))
    o = ok.CrystalKVOracle(1, 2, 8, 2, 128, np.full((1, 2, 2), 1000), lam=0.5, top_p=0.9, t0=P)
    o.load_prompt(0, st.prompt_k[0], st.prompt_v[0])
    decs = o.seed_prompt(0, q_obs[-1:])
    for key, u in o.units.items():
        hit = decs[key][0].hit
        assert hit[P - 1] and np.array_equal(u.tau, np.where(hit, P - 1, np.arange(P)))
        assert np.array_equal(u.crf, np.where(hit & (np.arange(P) < P - 1), np.float32(1.0) + np.float32(0.5) ** (P - 1 - np.arange(P)).astype(np.float32), np.float32(1.0)).astype(np.float32))


# ------------------------------------------------------------------ sink + recent window (comparison policy)
def test_window_select_closed_form_and_brute_force():
    """Sec. 2.3's initial-plus-recent baseline.  With positions 0..n-1 the survivors are the first
    n_sink and the last B - n_sink positions; in any order of the entries the same set of positions
    survives; and on tiny inputs the survivors are the best subset under "sinks first, then the newer
    the better", found by brute force over all subsets."""
    rng = np.random.default_rng(5)
    for n, B, s in [(40, 12, 4), (40, 12, 0), (9, 8, 3), (17, 5, 5), (10, 10, 2), (6, 9, 1)]:
        pos = rng.permutation(n)
        retain, evicted = ok.window_select(pos, B, s)
        want = set(range(n)) if n <= B else set(range(s)) | set(range(n - (B - s), n))
        assert set(pos[retain].tolist()) == want
        assert sorted(retain.tolist() + evicted.tolist()) == list(range(n))
        assert np.all(np.diff(retain) > 0)
    # more sinks than budget: the lowest positions stay
    retain, _ = ok.window_select(np.array([7, 0, 3, 1, 2, 9]), 2, 4)
    assert retain.tolist() == [1, 3]
    # brute force with gaps in the positions (some already evicted)
    for trial in range(20):
        n, B, s = 7, int(rng.integers(1, 7)), int(rng.integers(0, 5))
        pos = np.sort(rng.choice(30, size=n, replace=False))
        rng.shuffle(pos)
        def goodness(sub):
            p = sorted(pos[list(sub)].tolist())
            sinks = [x for x in p if x < s]
            # every kept sink outranks any number of recent entries; among sinks the lower the better
            return (len(sinks), [-x for x in sinks], sorted([x for x in p if x >= s], reverse=True))
        best = max(itertools.combinations(range(n), B), key=goodness)
        retain, _ = ok.window_select(pos, B, s)
        assert retain.tolist() == sorted(best)


def test_window_policy_keeps_a_sliding_window_through_decoding():
    """Decoding with the window policy after every step: each cache holds exactly the sink positions and
    the latest budget - n_sink positions at every time, the attention output is plain softmax attention
    over those entries, and the stored scores of survivors are untouched by the policy."""
    cfg = wl.scaled(wl.CONFIGS["tiny"], prompt=30, decode_steps=25, budget=16, budget_min=1, budget_max=64)
    st = wl.make_stream(cfg, tiny_heavy=False)
    B, s = 16, 4
    o = ok.CrystalKVOracle(1, 1, 8, 2, 128, np.full((1, 1, 2), B), lam=0.5, top_p=0.9, t0=30)
    o.load_prompt(0, st.prompt_k[0], st.prompt_v[0])
    o.evict_window(s)
    for step in range(25):
        out, recs = o.decode_step(st.q[step], st.k_new[step], st.v_new[step], evict=False)
        for key, u in o.units.items():
            # attention over [sinks, window, new]: compare with softmax attention written out here
            h = key[2]
            K, V = u.K, u.V
            for g in range(4):
                lg = (K @ st.q[step, 0, 0, 4 * h + g].astype(np.float64)) * o.scale
                w = np.exp(lg - lg.max())
                assert np.allclose(out[0, 0, 4 * h + g], (w / w.sum()) @ V, rtol=1e-11, atol=1e-13)
        crf_after_step = {k: dict(zip(u.pos.tolist(), u.crf.tolist())) for k, u in o.units.items()}
        ev = o.evict_window(s)
        t = 30 + step
        for key, u in o.units.items():
            assert sorted(u.pos.tolist()) == list(range(s)) + list(range(t - (B - s) + 1, t + 1))
            assert ev[key].tolist() == [t - (B - s)]
            assert all(crf_after_step[key][p] == c for p, c in zip(u.pos.tolist(), u.crf.tolist()))


# ------------------------------------------------------------------ margins of the decisions
def _frac(x):
    return math.inf if x is None else x[0] / x[1]


def test_hit_decision_margins_of_the_hand_worked_trace(golden_dir):
    """`sum_margin` and `edge_gap` decide which GPU/oracle differences the parity tests may accept, so they
    are pinned like any other output: the fixture lists, per step, the nucleus size, the distance of the cut
    to p and the relative weight gap at the edge, all computed by hand."""
    fx = json.load(open(os.path.join(golden_dir, "alg1_trace_8tok.json")))
    for st in fx["steps"]:
        d = ok.hit_mask(np.array(st["abar"]), np.array(st["live"]), fx["top_p"], new_index=len(st["live"]) - 1)
        assert d.m_star == st["m_star"]
        assert d.sum_margin == pytest.approx(st["sum_margin"], rel=1e-12, abs=1e-15)
        want = _frac(st["edge_gap_fraction"])
        assert d.edge_gap == (want if math.isinf(want) else pytest.approx(want, rel=1e-12, abs=1e-15))
        # the order the margins refer to: weight descending, position ascending
        ranked = sorted(range(len(st["live"])), key=lambda i: (-st["abar"][i], st["live"][i]))
        assert d.order.tolist() == ranked


def test_hit_decision_margins_on_constructed_edge_cases():
    pos = np.arange(4)
    # the cut lands 1e-7 above p: the margin is that distance, not the (large) distance below
    d = ok.hit_mask(np.array([0.5, 0.3 + 1e-7, 0.1, 0.1 - 1e-7]), pos, 0.8)
    assert d.m_star == 2 and d.sum_margin == pytest.approx(1e-7, rel=1e-6)
    assert d.edge_gap == pytest.approx((0.3 + 1e-7 - 0.1) / (0.3 + 1e-7), rel=1e-12)
    # the sum before the cut lies 2e-8 below p: that side is the margin
    d = ok.hit_mask(np.array([0.8 - 2e-8, 0.1, 0.05 + 2e-8, 0.05]), pos, 0.8)
    assert d.m_star == 2 and d.sum_margin == pytest.approx(2e-8, rel=1e-6)
    # two weights 3e-7 apart (relative) at the edge
    a_in = 0.2
    a_out = a_in * (1 - 3e-7)
    d = ok.hit_mask(np.array([0.5, a_in, a_out, 1 - 0.5 - a_in - a_out]), pos, 0.6)
    assert d.m_star == 2 and d.edge_gap == pytest.approx(3e-7, rel=1e-6) and d.sum_margin == pytest.approx(0.1, rel=1e-9)
    # exact tie at the edge: gap 0 (the position decides); no entry outside: gap infinite
    assert ok.hit_mask(np.array([0.4, 0.3, 0.3]), np.array([5, 9, 2]), 0.6).edge_gap == 0.0
    d = ok.hit_mask(np.array([0.5, 0.3, 0.2]), np.arange(3), 1.0)
    assert d.m_star == 3 and math.isinf(d.edge_gap) and d.sum_margin == pytest.approx(1.0 - 0.8, rel=1e-12)
    # a margin must never be negative and never exceed p or the last included weight
    g = np.random.default_rng(17)
    for _ in range(200):
        n = int(g.integers(1, 30))
        a = g.random(n) ** 3
        a /= a.sum()
        p = float(g.choice([0.3, 0.6, 0.9]))
        d = ok.hit_mask(a, g.permutation(100)[:n], p)
        assert 0.0 <= d.sum_margin <= max(p, 1 - p) + 1e-12 and d.edge_gap >= 0.0
        srt = np.sort(a)[::-1]
        c = np.cumsum(srt)
        assert d.sum_margin <= srt[d.m_star - 1] + 1e-15       # both sides of the cut are within one weight of p
        if d.m_star < n:
            assert d.edge_gap == pytest.approx((srt[d.m_star - 1] - srt[d.m_star]) / srt[d.m_star - 1], abs=1e-12)


def test_evict_gap_and_step_record_of_the_hand_worked_trace(golden_dir):
    """The class's record of a step: evict_gap as computed by hand, and the pre-update state it keeps for
    parity checks is the state the step started from (after the append)."""
    fx = json.load(open(os.path.join(golden_dir, "alg1_trace_8tok.json")))
    o = ok.CrystalKVOracle(1, 1, 1, 1, 8, np.full((1, 1, 1), fx["budget"]), lam=fx["lambda"],
                           top_p=fx["top_p"], softmax_scale=1.0, t0=0)
    prev = {}
    for st in fx["steps"]:
        t = st["t"]
        k_new = np.zeros(8)
        k_new[t] = 1.0
        q = np.full(8, -1e4)
        for ppos, w in zip(st["live"], st["abar"]):
            q[ppos] = math.log(w)
        rec = o.step_unit((0, 0, 0), q[None, :], k_new, np.zeros(8))
        want = _frac(st["evict_gap_fraction"])
        assert rec.evict_gap == (want if math.isinf(want) else pytest.approx(want, rel=1e-12))
        assert rec.t == t and rec.budget == fx["budget"] and rec.pre_pos.tolist() == st["live"]
        for p_, c_, tt in zip(rec.pre_pos.tolist(), rec.pre_crf.tolist(), rec.pre_tau.tolist()):
            assert (c_, tt) == prev.get(p_, (0.0, t))           # stored state of the previous step; new entry: (0, t)
        u = o.units[(0, 0, 0)]
        prev = {p_: (c_, tt) for p_, c_, tt in zip(u.pos.tolist(), u.crf.tolist(), u.tau.tolist())}
        o.t += 1


# ------------------------------------------------------------------ aggregated CRF (Alg. 2 input)
def test_crf_sum_fixed_hand_case_and_bound():
    """Aggregated CRF of a head in 2^-20 fixed point.  Dyadic scores make floor(x 2^20) exact by hand:
    1.5 -> 1572864, 0.25 -> 262144, 3 * 2^-22 -> 0 (floor, where rounding would give 1), 0.75 + 2^-20 + 2^-21
    -> 786433, 2^-20 -> 1; total 2621442.  In general the fixed-point sum lies at most n * 2^-20 below the
    plain float64 sum and never above it."""
    tmp = np.array([1.5, 0.25, 3 * 2.0 ** -22, 0.75 + 2.0 ** -20 + 2.0 ** -21, 2.0 ** -20], np.float32)
    assert ok.crf_sum_fixed(tmp) == 1572864 + 262144 + 0 + 786433 + 1 == 2621442
    assert ok.crf_sum_fixed(np.zeros(0, np.float32)) == 0
    assert ok.FIXED_POINT_ONE == 2 ** 20
    g = np.random.default_rng(23)
    for n in (1, 7, 300, 5000):
        tmp = (g.random(n) * g.choice([1e-7, 1e-3, 1.0, 2.0], size=n)).astype(np.float32)
        plain = float(np.sum(tmp.astype(np.float64)))
        fixed = ok.crf_sum_fixed(tmp) / 2.0 ** 20
        assert plain - n * 2.0 ** -20 <= fixed <= plain + 1e-12 * plain
        assert isinstance(ok.crf_sum_fixed(tmp), int)


def _dictated_step(o, key, t, live, weights, d=16):
    """One decode step of unit `key` whose attention weights are dictated: one-hot keys (position i answers
    on coordinate i) and a query whose logits are the logs of the wanted weights."""
    k_new = np.zeros(d)
    k_new[t] = 1.0
    q = np.full(d, -1e4)
    for p_, w in zip(live, weights):
        q[p_] = math.log(w)
    return o.step_unit(key, q[None, :], k_new, np.zeros(d))


def test_rebudget_window_mean_equals_alg2_on_the_plain_mean_hand_case():
    """Sec. 5.3 / Alg. 2 through the class: two layers x two heads start empty with budget 60 each and take
    two decode steps with dictated weights.  Step t = 0: the lone new entry scores 1.  Step t = 1 (lambda
    = 0.5, p = 0.6): in units A the old entry gets weight 0.9 (hit: 0.5 * 1 + 1 = 1.5, plus the new entry's 1
    -> 2.5), in unit B the new entry gets 0.9 (old entry missed: 0.5, plus 1 -> 1.5).  Window means of the
    aggregated CRF: A = (1 + 2.5) / 2 = 1.75, B = (1 + 1.5) / 2 = 1.25.  Layer 0 = (A, B), layer 1 = (A, A).
    Alg. 2 by hand: eta_0 = 3 / 120, eta_1 = 3.5 / 120; B'_0 = 240 * 3 / 6.5 = 110.77, B'_1 = 129.23 ->
    integers 111, 129 (floor, the unit left over to the larger fraction); heads of layer 0: 111 * 1.75 / 3 =
    64.75 and 46.25 -> 65, 46; heads of layer 1: 64.5 each -> 65, 64 (tie: lower index).  The scores are
    dyadic, so the 2^-20 fixed-point accumulator is exact and the class must agree with Alg. 2 applied to
    the plain float64 means."""
    o = ok.CrystalKVOracle(2, 1, 2, 2, 16, np.full((2, 1, 2), 60), lam=0.5, top_p=0.6, softmax_scale=1.0, t0=0,
                           budget_min=10, budget_max=100)
    unit_b = (0, 0, 1)
    sums = {key: [] for key in o.units}
    for t in range(2):
        for key in o.units:
            if t == 0:
                rec = _dictated_step(o, key, 0, [0], [1.0])
            elif key == unit_b:
                rec = _dictated_step(o, key, 1, [0, 1], [0.1, 0.9])
            else:
                rec = _dictated_step(o, key, 1, [0, 1], [0.9, 0.1])
            sums[key].append(float(np.sum(rec.tmp.astype(np.float64))))     # plain sum of this step's CRF_temp
            assert rec.crf_sum == int(round(sums[key][-1] * 2 ** 20))       # dyadic: the fixed point is exact
        o.t += 1
        o.window_steps += 1
    assert sums[unit_b] == [1.0, 1.5] and sums[(0, 0, 0)] == [1.0, 2.5]
    C_plain = np.array([[np.mean(sums[(l, 0, h)]) for h in range(2)] for l in range(2)])
    assert C_plain.tolist() == [[1.75, 1.25], [1.75, 1.75]]
    want = ok.rebudget(C_plain, np.full((2, 2), 60), 240, 10, 100)
    got = o.rebudget()
    assert got[:, 0, :].tolist() == want.tolist() == [[65, 46], [65, 64]]
    # the real-valued shares of Alg. 2 Steps 1-4 that these integers round
    Bl, Bh = ok.budget_shares(C_plain, np.full((2, 2), 60), 240)
    assert np.allclose(Bl, [240 * 3 / 6.5, 240 * 3.5 / 6.5], rtol=1e-14)
    assert np.allclose(Bh, [[Bl[0] * 1.75 / 3, Bl[0] * 1.25 / 3], [Bl[1] / 2, Bl[1] / 2]], rtol=1e-14)
    # the window restarts: a second call without steps in between changes nothing
    assert o.window_steps == 0 and all(u.crf_window == 0 for u in o.units.values())
    assert np.array_equal(o.rebudget(), got)


def test_rebudget_window_mean_is_a_mean_over_steps_not_a_sum_or_last_value():
    """Units whose per-step aggregated CRF differ between steps: the class's budgets must equal Alg. 2 on the
    mean over the window's steps of the plain float64 sums (to within the fixed point's 2^-20 per entry, which
    cannot move these budgets: the test checks that), for windows of 1, 3 and 5 steps, random geometry."""
    g = np.random.default_rng(31)
    for n_steps in (1, 3, 5):
        L, H = 3, 2
        budgets = g.integers(20, 60, size=(L, 1, H))
        cfg = wl.scaled(wl.CONFIGS["tiny"], n_layers=L, batch=1, n_q_heads=2 * H, n_kv_heads=H, prompt=12, decode_steps=n_steps,
                        budget=40, budget_min=5, budget_max=100, seed=400 + n_steps)
        st = wl.make_stream(cfg, tiny_heavy=False)
        o = ok.CrystalKVOracle(L, 1, 2 * H, H, 128, budgets, lam=0.7, top_p=0.9, t0=12, budget_min=5, budget_max=100)
        for l in range(L):
            o.load_prompt(l, st.prompt_k[l], st.prompt_v[l])
        acc = np.zeros((L, H))
        for s in range(n_steps):
            _, recs = o.decode_step(st.q[s], st.k_new[s], st.v_new[s], evict=False)
            for (l, b, h), r in recs.items():
                acc[l, h] += float(np.sum(r.tmp.astype(np.float64)))
        C_plain = acc / n_steps
        n_max = 12 + n_steps
        want = ok.rebudget(C_plain, budgets[:, 0, :], int(budgets.sum()), 5, 100)
        # the fixed point lowers every mean by at most n 2^-20: budgets computed from the lowered means
        lowered = ok.rebudget(C_plain - n_max * 2.0 ** -20, budgets[:, 0, :], int(budgets.sum()), 5, 100)
        got = o.rebudget()[:, 0, :]
        assert np.array_equal(want, lowered), "pick another seed: this case sits on a rounding edge"
        assert np.array_equal(got, want)
        if n_steps > 1:
            # the case has the power to tell the window mean from the last step's value alone (Alg. 2 is scale
            # invariant, so a sum and a mean over the same steps are the same input by construction)
            last = np.array([[float(np.sum(recs[(l, 0, h)].tmp.astype(np.float64))) for h in range(H)] for l in range(L)])
            assert not np.array_equal(ok.rebudget(last, budgets[:, 0, :], int(budgets.sum()), 5, 100), want)


# ------------------------------------------------------------------ Alg. 1 Step 4 on its own
def test_standalone_evict_uses_scores_decayed_to_the_last_step():
    """`current_tmp` / `evict()`: Step 4 called between steps ranks entries by CRF_temp at the time of the
    last completed step.  Pins: (i) the closed form of Sec. 5.2 for an entry not accessed since tau,
    lambda^(t_last - tau) CRF(tau), and the full closed form sum_j lambda^(t_last - t_j) over the logged hit
    times; (ii) a step without eviction followed by evict() leaves what the same step with eviction
    leaves; (iii) brute force: the evicted entries are the lowest under (closed-form score, higher
    position first)."""
    lam = 0.5
    cfg = wl.scaled(wl.CONFIGS["tiny"], prompt=20, decode_steps=30, budget=24, budget_min=1, budget_max=64, seed=77)
    st = wl.make_stream(cfg)
    mk = lambda: ok.CrystalKVOracle(1, 1, 8, 2, 128, np.full((1, 1, 2), 24), lam=lam, top_p=0.9, t0=20)
    a, b = mk(), mk()
    for o in (a, b):
        o.load_prompt(0, st.prompt_k[0], st.prompt_v[0])
    hits = {key: {p_: [19] for p_ in range(20)} for key in a.units}       # prompt entries: referenced at P - 1
    for s in range(30):
        lazy = s % 4 != 3                                       # `a` evicts only every fourth step, on its own
        _, recs = a.decode_step(st.q[s], st.k_new[s], st.v_new[s], evict=False)
        t_last = a.t - 1
        for key, r in recs.items():
            u = a.units[key]
            hits[key][t_last] = []
            for p_, h in zip(u.pos.tolist(), r.decision.hit.tolist()):
                if h:
                    hits[key][p_].append(t_last)
            tmp = a.current_tmp(u)
            for i, p_ in enumerate(u.pos.tolist()):
                closed = sum(lam ** (t_last - tj) for tj in hits[key][p_])
                assert float(tmp[i]) == pytest.approx(closed, rel=1e-6)
                assert float(tmp[i]) == pytest.approx(float(u.crf[i]) * lam ** (t_last - int(u.tau[i])), rel=1e-6)
            assert np.array_equal(tmp, r.tmp)                   # the step's own CRF_temp, recomputed from the stored state
        if lazy:
            continue
        # catch `b` up with fused evictions only on the same steps: both must agree after a.evict()
        before = {key: (u.pos.copy(), a.current_tmp(u)) for key, u in a.units.items()}
        ev = a.evict()
        for key, (pos0, tmp0) in before.items():
            ranked = sorted(range(len(pos0)), key=lambda i: (float(tmp0[i]), -int(pos0[i])))
            k = len(pos0) - 24
            assert sorted(pos0[ranked[:k]].tolist()) == ev[key].tolist() and len(ev[key]) == k == (0 if s == 3 else 4)
            for p_ in ev[key].tolist():
                del hits[key][p_]
        for s2 in range(s - 3, s + 1):
            b.decode_step(st.q[s2], st.k_new[s2], st.v_new[s2], evict=(s2 == s))
        for key in a.units:
            ua, ub = a.units[key], b.units[key]
            assert np.array_equal(ua.pos, ub.pos) and np.array_equal(ua.crf, ub.crf) and np.array_equal(ua.tau, ub.tau)
