"""ckv_probe_noalloc (the entry point that allocates nothing: its scan scratch is the library's static device
array) against ckv_probe, through the C ABI: classes identical byte for byte, on two calls in a row, the second
on a smaller input, with decode steps of the contexts before and after; and a layer too large for the static
scratch is refused."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _context(cfg, cap, budgets, steps):
    from oracle import crystal_kv as ok
    from paper_2601_16986_amd import ckv, workloads as wl
    st = wl.make_stream(cfg, tiny_heavy=False)
    o = ok.CrystalKVOracle(cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, budgets, lam=cfg.lam,
                           top_p=cfg.top_p, t0=cfg.prompt, budget_min=cfg.budget_min, budget_max=cfg.budget_max)
    g = ckv.CrystalKV(cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cap, budgets, lam=cfg.lam,
                      top_p=cfg.top_p, t0=cfg.prompt, budget_min=cfg.budget_min, budget_max=cfg.budget_max)
    for l in range(cfg.n_layers):
        o.load_prompt(l, st.prompt_k[l], st.prompt_v[l])
        g.load_prompt(l, st.prompt_k[l], st.prompt_v[l])
    for s in range(steps):
        o.decode_step(st.q[s], st.k_new[s], st.v_new[s])
        g.decode_step(st.q[s], st.k_new[s], st.v_new[s])
    return st, o, g


def _check_against_both(g, o, st, layer):
    import torch
    q = torch.from_numpy(np.ascontiguousarray(st.probe_q[layer])).to(g.device).to(torch.bfloat16)
    ref = g.probe(layer, q)                                       # the existing entry point (context's workspace)
    got = torch.full_like(ref, 255)
    g.probe_noalloc(layer, q, got)                                # static scratch
    torch.cuda.synchronize()
    assert torch.equal(ref, got), int((ref != got).sum())
    # and the oracle's classes, as for ckv_probe (entries within rounding of a class boundary may fall either way)
    cls = got.cpu().numpy()
    for (l, b, h), u in o.units.items():
        if l != layer:
            continue
        want, abar = o.probe((l, b, h), st.probe_q[l, b, h * o.G:(h + 1) * o.G])
        e = g.export_unit(l, b, h, with_kv=False)
        mine = dict(zip(e["pos"].tolist(), cls[b, h, :e["n"]].tolist()))
        k = (3 * u.n) // 10
        srt = np.sort(abar)
        edges = [srt[k - 1], srt[k], srt[u.n - k - 1], srt[u.n - k]] if k else []
        for p_, c_, a in zip(u.pos.tolist(), want.tolist(), abar.tolist()):
            if mine[p_] != c_:
                assert min(abs(a - x) / x for x in edges) < 1e-5, (l, b, h, p_)
        assert (cls[b, h, :e["n"]] == 2).sum() == k and (cls[b, h, e["n"]:] == 255).all()


def test_probe_noalloc_equals_probe_on_two_calls_the_second_smaller():
    from paper_2601_16986_amd import ckv, workloads as wl
    big = wl.scaled(wl.CONFIGS["qwen7b"], n_layers=2, batch=3, n_q_heads=14, n_kv_heads=2, prompt=333, decode_steps=6,
                    budget=500, budget_min=300, budget_max=735, adaptive=False, rebudget_interval=0, seed=5)
    budgets = np.array([[[300, 700], [513, 333], [641, 352]], [[352, 641], [333, 513], [700, 300]]], dtype=np.int32)
    st1, o1, g1 = _context(big, 736, budgets, 6)
    small = wl.scaled(wl.CONFIGS["tiny"], n_layers=1, batch=1, n_q_heads=8, n_kv_heads=2, prompt=45, decode_steps=9,
                      budget=40, budget_min=1, budget_max=95, adaptive=False, rebudget_interval=0, seed=9)
    st2, o2, g2 = _context(small, 96, np.full((1, 1, 2), 40, np.int32), 9)
    _check_against_both(g1, o1, st1, 1)                          # first call: units of several chunks
    _check_against_both(g2, o2, st2, 0)                          # second call, smaller: stale partials of the first stay in the array
    _check_against_both(g1, o1, st1, 0)                          # and back, on another layer of the first context
    # the contexts' own workspaces were left alone: decoding goes on as if nothing happened
    for g, o, st, s in ((g1, o1, st1, 6), (g2, o2, st2, 9)):
        assert g.status() == 0
    g1.close()
    g2.close()


def test_probe_noalloc_refuses_a_layer_beyond_the_static_scratch():
    import torch
    from paper_2601_16986_amd import ckv
    # 128 units of 32768 slots with 8 query heads each: 6 G cap bytes = 1.6 MB of scan scratch per unit, 200 MB per layer
    L, Bz, Hq, Hkv, cap = 1, 64, 16, 2, 32768
    g = ckv.CrystalKV(L, Bz, Hq, Hkv, 128, cap, np.full((L, Bz, Hkv), 64, np.int32), t0=0, budget_min=1, budget_max=cap - 1)
    q = torch.zeros((Bz, Hq, 128), dtype=torch.bfloat16, device=g.device)
    cls = torch.zeros((Bz, Hkv, cap), dtype=torch.uint8, device=g.device)
    with pytest.raises(ckv.CkvError) as e:
        g.probe_noalloc(0, q, cls)
    assert e.value.code == ckv.EWORKSPACE and "static scratch" in str(e.value)
    assert g.status() == 0                                        # refused before anything was launched
    g.close()
