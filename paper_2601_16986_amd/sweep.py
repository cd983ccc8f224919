"""lambda x top-p sweep on a synthetic workload (a model-free analogue of the paper's hyper-parameter study,
Sec. 6.4 / Fig. 4): which (lambda, p) keep the entries that matter under a fixed budget?

    python -m paper_2601_16986_amd.sweep [--tokens 2048] [--prompt 256] [--budget 256]

Runs on the GPU through the library's binding only.  The workload is the synthetic recipe of
`workloads.make_stream` (1 % heavy keys aligned with the head's mean query, AR(1) drift shared by keys and
queries, everything else noise), 2 layers x 4 sequences x 2 KV heads with 5 query heads each.  Per setting
the whole sequence is decoded with eviction every step, then two recalls are taken per unit and averaged:

* heavy recall: share of the heavy positions that are still cached;
* Crystal recall: share of the reference Crystal set that is still cached, the reference being Sec. 3's
  labelling (top 30 % by the answer query's attention) over ALL positions, obtained from a second context
  whose budget holds the whole sequence (nothing evicted) and `ckv_probe`; the answer query is the held-out
  query of the step after the last one.  Normalised by min(|Crystal|, budget).

Three reference rows on the same skeleton (the policies Sec. 2.3 names): "recent" keeps the newest B entries
(a sliding window: `ckv_evict_window` with no sinks after every step), "sink + recent" keeps the first 4
positions and the newest B - 4 (the same call with 4 sinks), "accumulated attention" scores every entry by
the plain sum of its attention weights (the attention-weighted reward with
lambda = 1: the accumulation policy of heavy-hitter eviction schemes).  Policies only: no accuracy claim.
Prints one markdown table and one JSON line.
"""
import argparse
import json

import numpy as np


def run(cfg, st, lam, top_p, budget, torch, ckv, device, answer_q, reward_mode=0, n_sink=None):
    T = cfg.decode_steps
    N = cfg.prompt + T
    budgets = np.full((cfg.n_layers, cfg.batch, cfg.n_kv_heads), budget, dtype=np.int32)
    cap = (max(budget, cfg.prompt) + 64) // 32 * 32
    g = ckv.CrystalKV(cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cap, budgets, lam=lam,
                      top_p=top_p, reward_mode=reward_mode, t0=cfg.prompt, budget_min=1, budget_max=cap - 1, device=device)
    for l in range(cfg.n_layers):
        g.load_prompt(l, st["pk"][l], st["pv"][l])
    evict = g.evict if n_sink is None else (lambda: g.evict_window(n_sink))
    if budget < cfg.prompt:
        evict()
    out = torch.empty((cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.head_dim), dtype=torch.float32, device=device)
    for s in range(T):
        g.decode_step(st["q"][s], st["k"][s], st["v"][s], out=out, evict=n_sink is None)
        if n_sink is not None:
            evict()
    assert g.status() == 0
    kept = {}
    for l in range(cfg.n_layers):
        for b in range(cfg.batch):
            for h in range(cfg.n_kv_heads):
                kept[(l, b, h)] = g.export_unit(l, b, h, with_kv=False)["pos"]
    classes = None
    if budget >= N:                                     # the reference context: label every position
        classes = {}
        for l in range(cfg.n_layers):
            cls = g.probe(l, answer_q[l]).cpu().numpy()
            for b in range(cfg.batch):
                for h in range(cfg.n_kv_heads):
                    pos = kept[(l, b, h)]
                    classes[(l, b, h)] = set(pos[cls[b, h, :len(pos)] == 2].tolist())       # 2 = Crystal
    g.close()
    return kept, classes


def recalls(kept, heavy, crystal, budget):
    """Mean over the units of the share of heavy positions, and of the reference Crystal set, still cached.
    kept: {unit: positions}, heavy: bool [L][Bz][Hkv][N], crystal: {unit: set of positions}."""
    hr, cr = [], []
    for key, pos in kept.items():
        have = set(np.asarray(pos).tolist())
        hp = set(np.nonzero(heavy[key])[0].tolist())
        if hp:
            hr.append(len(hp & have) / min(len(hp), budget))
        cr.append(len(crystal[key] & have) / min(len(crystal[key]), budget))
    return float(np.mean(hr)), float(np.mean(cr))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--tokens", type=int, default=2048)
    ap.add_argument("--prompt", type=int, default=256)
    ap.add_argument("--budget", type=int, default=256)
    ap.add_argument("--seed", type=int, default=5)
    args = ap.parse_args()
    import torch
    from paper_2601_16986_amd import ckv, workloads as wl

    device = torch.device("cuda:0")
    T = args.tokens - args.prompt
    cfg = wl.scaled(wl.CONFIGS["qwen14b"], n_layers=2, batch=4, n_q_heads=10, n_kv_heads=2, prompt=args.prompt,
                    decode_steps=T + 1, budget=args.budget, budget_min=1, budget_max=args.tokens + 64, adaptive=False,
                    rebudget_interval=0, seed=args.seed)
    host = wl.make_stream(cfg)                          # T + 1 steps: the last query is the held-out answer query
    cfg = wl.scaled(cfg, decode_steps=T)
    dev = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to(device).to(torch.bfloat16)
    st = {"pk": dev(host.prompt_k), "pv": dev(host.prompt_v), "q": dev(host.q[:T]), "k": dev(host.k_new[:T]),
          "v": dev(host.v_new[:T])}
    answer_q = dev(host.q[T])
    heavy = host.heavy[..., :args.tokens]

    _, crystal = run(cfg, st, 0.5, 0.9, args.tokens + 32, torch, ckv, device, answer_q)
    lams = [0.0, 0.3, 0.5, 0.7, 0.9, 1.0]
    ps = [0.5, 0.7, 0.9, 0.95]
    rows, results = [], []
    settings = ([("recent", 0.5, 0.9), ("accumulated", 1.0, 0.9), ("sink + recent", 0.5, 0.9)]
                + [(None, lam, p) for p in ps for lam in lams])
    for name, lam, p in settings:
        kept, _ = run(cfg, st, lam, p, args.budget, torch, ckv, device, answer_q,
                      reward_mode=ckv.REWARD_ATTN_WEIGHTED if name == "accumulated" else ckv.REWARD_TOPP_HIT,
                      n_sink={"recent": 0, "sink + recent": 4}.get(name))
        hr, cr = recalls(kept, heavy, crystal, args.budget)
        results.append({"lambda": lam, "top_p": p, "name": name, "heavy_recall": hr, "crystal_recall": cr})
    print(f"tokens {args.tokens} (prompt {args.prompt}), budget {args.budget} per unit, {len(crystal)} units, "
          f"heavy positions per unit {heavy.sum() / len(crystal):.1f}, reference Crystal set {np.mean([len(c) for c in crystal.values()]):.0f} positions")
    print("| top-p \\ lambda | " + " | ".join(f"{x:g}" for x in lams) + " |")
    print("|---|" + "---|" * len(lams))
    for p in ps:
        cells = [r for r in results if r["name"] is None and r["top_p"] == p]
        print(f"| {p:g} | " + " | ".join(f"{r['heavy_recall']:.2f} / {r['crystal_recall']:.2f}" for r in cells) + " |")
    r0, r1, r2 = results[0], results[1], results[2]
    print(f"| newest {args.budget} only | {r0['heavy_recall']:.2f} / {r0['crystal_recall']:.2f} |" + " |" * (len(lams) - 1))
    print(f"| 4 sinks + newest {args.budget - 4} | {r2['heavy_recall']:.2f} / {r2['crystal_recall']:.2f} |" + " |" * (len(lams) - 1))
    print(f"| accumulated attention | {r1['heavy_recall']:.2f} / {r1['crystal_recall']:.2f} |" + " |" * (len(lams) - 1))
    print(json.dumps({"tokens": args.tokens, "prompt": args.prompt, "budget": args.budget, "cells": "heavy recall / Crystal recall",
                      "results": results}))


if __name__ == "__main__":
    main()
