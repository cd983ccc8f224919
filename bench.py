#!/usr/bin/env python3
"""Benchmark of the Crystal-KV decode hot path on one MI355X.

A "step" is one decode step over ALL layers x sequences x KV heads of the
workload: append, GQA attention over the budgeted caches, top-p hit mask, CRF
update, eviction + compaction (every step), and, for workloads that re-allocate
budgets, Alg. 2 at its interval.  Inputs are synthetic and resident in HBM
before the timed region.  Prints ONE JSON line.

  value        decode steps/s from HIP-graph replays of the all-layers call
  roofline     the dominant kernel (the fused per-unit kernel, or the scan kernel
               when the separate kernels are used): algorithmic bytes per launch
               over its average duration, measured with HIP events around each
               launch in a separate eager pass
  cpu_baseline the numpy oracle timed on the host on a bounded sample
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
RING = 32                     # distinct synthetic step inputs held at a time (and steps per HIP graph).  The timed
                              # regions refill them with fresh draws between repeats: a replayed input inserts keys
                              # that are exact duplicates of cached ones, identical keys tie in the top-p and
                              # eviction orders, and a cache that fills up with copies drifts into the (slow,
                              # unrealistic) tie-breaking paths


def build_workload(cfg, device, budgets=None, headroom=1, pool_factor=1.0, pools=None):
    """Steady-state caches of the workload on the device (every unit full at its budget), plus the ring of
    step inputs.  budgets: override of the workload's own draw (tests place units at chosen sizes)."""
    import numpy as np
    import torch
    from paper_2601_16986_amd import ckv, workloads as wl

    if budgets is None:
        budgets = wl.draw_budgets(cfg)
    cap = (cfg.budget_max + 1 + 31) // 32 * 32
    t_now = cfg.prompt + cfg.decode_steps // 2
    pool_slots = None
    if pool_factor != 1.0:
        import ctypes as C
        lay = ckv.Layout(cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cap, ckv.F32, headroom, 0)
        b32 = np.ascontiguousarray(np.asarray(budgets, dtype=np.int32))
        pool_slots = int(ckv.load().ckv_pool_slots(C.byref(lay), b32.ctypes.data_as(C.c_void_p), 0) * pool_factor) // 256 * 256
    kwargs = dict(lam=cfg.lam, top_p=cfg.top_p, t0=t_now, budget_min=cfg.budget_min, budget_max=cfg.budget_max,
                  headroom=headroom, pool_slots=pool_slots)     # headroom 1: shared pools, memory follows the budgets
    placement = None
    if pools == "place":
        # Where the pools lie in physical memory moves the step by a tenth on this hardware: once, at start-up,
        # try allocations across the device's memory and keep the one decode steps run fastest on.
        import ctypes as C
        lay = ckv.Layout(cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cap, ckv.F32, headroom, 0)
        b32 = np.ascontiguousarray(np.asarray(budgets, dtype=np.int32))
        ps = pool_slots or int(ckv.load().ckv_pool_slots(C.byref(lay), b32.ctypes.data_as(C.c_void_p), 0))
        kwargs["pool_slots"] = ps
        rest_bytes = ckv.arena_bytes(cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cap, budgets, **kwargs) - 2 * ps * 256
        kp, vp, rest, placement = ckv.place_pools(ps * 256, device, rest_bytes=rest_bytes)
        pools = (kp[:ps * 128], vp[:ps * 128])
        kwargs["arena"] = rest
    g = ckv.CrystalKV(cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cap, budgets,
                      device=device, pools=pools, **kwargs)
    g.placement = placement
    m = wl.torch_mean_query(cfg, device)
    gen = wl.torch_generator(cfg, 9, device)
    r_now = math.sqrt(wl.DRIFT_VAR) * torch.randn(m.shape, generator=gen, device=device)
    for layer in range(cfg.n_layers):
        k, v, n, crf, tau, pos = wl.torch_steady_layer(cfg, layer, budgets[layer], t_now, m[layer], r_now[layer], device)
        g.load_cache(layer, k, v, n, crf, tau, pos)
        torch.cuda.synchronize()
        del k, v, n, crf, tau, pos
    ring, r_end = wl.torch_step_ring(cfg, RING, m, r_now, device, return_state=True)
    g.refill = _refiller(cfg, ring, m, r_end, device)
    return g, budgets, ring


def _refiller(cfg, ring, m, r_state, device):
    """refill(): overwrite the ring's tensors in place (HIP graphs that read them stay valid) with the next
    RING steps' inputs, drawn fresh, the drift continuing where the last batch ended."""
    from paper_2601_16986_amd import workloads as wl
    state = {"r": r_state, "epoch": 0}

    def refill():
        state["epoch"] += 1
        fresh, state["r"] = wl.torch_step_ring(cfg, RING, m, state["r"], device, epoch=state["epoch"], return_state=True)
        for dst, src in zip(ring, fresh):
            dst.copy_(src)
    return refill


def build_fullkv(cfg, device, tokens, total_steps):
    """The FullKV baseline of Table 1 on the same geometry: every unit holds all `tokens` positions and
    nothing is ever evicted (room for `total_steps` appended entries)."""
    import numpy as np
    import torch
    from paper_2601_16986_amd import ckv, workloads as wl

    budgets = np.full((cfg.n_layers, cfg.batch, cfg.n_kv_heads), tokens, dtype=np.int32)
    cap = (tokens + total_steps + 1 + 31) // 32 * 32
    g = ckv.CrystalKV(cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cap, budgets,
                      lam=cfg.lam, top_p=cfg.top_p, t0=tokens, budget_min=1, budget_max=cap - 1, device=device)
    m = wl.torch_mean_query(cfg, device)
    gen = wl.torch_generator(cfg, 9, device)
    r_now = math.sqrt(wl.DRIFT_VAR) * torch.randn(m.shape, generator=gen, device=device)
    for layer in range(cfg.n_layers):
        k, v, n, crf, tau, pos = wl.torch_steady_layer(cfg, layer, budgets[layer], tokens, m[layer], r_now[layer], device)
        g.load_cache(layer, k, v, n, crf, tau, pos)
        torch.cuda.synchronize()
        del k, v, n, crf, tau, pos
    ring = wl.torch_step_ring(cfg, RING, m, r_now, device)
    return g, budgets, ring


def seed_prompt_bench(cfg, device, P, W):
    """Prompt-side seeding on the workload's geometry: every layer holds a P-token prompt; ckv_seed_prompt
    replays its last W queries (one pass over the keys per batch of query tiles, the queries' rewards, the score
    recurrence).  Timed with events over all layers after one untimed layer; bytes: as built, the least possible,
    and what W decode steps over the visible prefixes would move."""
    import numpy as np
    import torch
    from paper_2601_16986_amd import ckv, workloads as wl

    budgets = np.full((cfg.n_layers, cfg.batch, cfg.n_kv_heads), P, dtype=np.int32)
    cap = (P + 64) // 32 * 32
    g = ckv.CrystalKV(cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cap, budgets,
                      lam=cfg.lam, top_p=cfg.top_p, t0=P, budget_min=1, budget_max=cap - 1, device=device)
    m = wl.torch_mean_query(cfg, device)
    gen = wl.torch_generator(cfg, 9, device)
    r_now = math.sqrt(wl.DRIFT_VAR) * torch.randn(m.shape, generator=gen, device=device)
    for layer in range(cfg.n_layers):
        k, v, *_ = wl.torch_steady_layer(cfg, layer, budgets[layer], P, m[layer], r_now[layer], device)
        g.load_prompt(layer, k, v)
        torch.cuda.synchronize()
        del k, v
    q_obs = (torch.randn((W, cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.head_dim), generator=gen, device=device)
             + m.repeat_interleave(cfg.group, dim=2)[None]).to(torch.bfloat16)
    g.seed_prompt(0, q_obs[:, 0].contiguous())
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    qs = [q_obs[:, l].contiguous() for l in range(cfg.n_layers)]
    e0.record()
    for l in range(cfg.n_layers):
        g.seed_prompt(l, qs[l])
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1)
    upl = cfg.batch * cfg.n_kv_heads
    entries = sum(P - W + j + 1 for j in range(W)) * upl             # per layer, query by query
    bytes_layer = entries * 512
    # what the replay needs at the least: every key row once (weights only, so no values), the queries, and the
    # scores read and written once per query
    # as built: a tile of 16 query columns holds Q = 16 // G queries; a batch of tiles (as many as the decode
    # workspace holds, at most 16) makes two passes over the keys (softmax partials, then mean weights: 4 B per
    # entry and query written); the rewards kernel reads the weights and writes the rewards in their place, the
    # recurrence reads them; the scores are read and written once per batch
    Q = max(1, 16 // cfg.group)
    tiles = (W + Q - 1) // Q
    fit = min(cfg.n_layers * cfg.group // Q, 16)
    per_batch = fit if fit >= 2 else 1
    passes = (tiles + per_batch - 1) // per_batch
    min_bytes = upl * (P * 256 + W * cfg.group * 256 + W * P * 16)
    pass_bytes = upl * (passes * P * (2 * 256 + 16) + 2 * W * cfg.group * 256 + W * P * 16)
    sec = ms / cfg.n_layers * 1e-3
    assert g.status() == 0
    g.close()
    return {"metric": "prompt seeding (ckv_seed_prompt), layers/s", "value": cfg.n_layers / (ms * 1e-3), "unit": "layers/s",
            "n_gpus": 1, "ms_per_layer": ms / cfg.n_layers, "higher_is_better": True, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": f"{cfg.name} geometry: {cfg.n_layers} layers, batch {cfg.batch}, {cfg.n_q_heads}/{cfg.n_kv_heads} heads, "
                                   f"prompt of {P} tokens, window of {W} queries", "units_per_layer": upl,
                       "entries_scanned_per_layer": entries, "queries_per_tile": Q, "tiles": tiles, "batches": passes, "passes_over_the_keys": 2 * passes},
            # K and V of the W visible prefixes, the bytes a query-by-query replay of decode steps moves (the figure of
            # the first version, kept for comparison; the replay as built reads far less, so this can exceed 1)
            "decode_replay_equivalent_gbps": bytes_layer / sec / 1e9,
            "decode_replay_equivalent_frac": bytes_layer / sec / 1e9 / HBM_PEAK_GBPS,
            "bytes_as_built": pass_bytes, "hbm_frac_as_built": pass_bytes / sec / 1e9 / HBM_PEAK_GBPS,
            "bytes_minimum": min_bytes, "hbm_frac_of_minimum": min_bytes / sec / 1e9 / HBM_PEAK_GBPS}


def algorithmic_bytes(cfg, budgets):
    """Per decode step.  Scan kernel: K and V rows of every cached entry once
    (512 B) plus the query group; whole step: 524 B per entry (K, V, CRF and
    tau reads) plus per-unit q, out (fp32), new k/v and one evicted row move."""
    import numpy as np
    n = np.asarray(budgets, dtype=np.int64) + 1          # entries attended: budget + the new one
    U, G = n.size, cfg.group
    scan = int(n.sum()) * 512 + U * G * 256
    step = int(n.sum()) * 524 + U * (G * 256 + G * 512 + 512 + 2 * 524)
    fused = step                                         # the fused kernel does the whole step, the append included
    return scan, step, int(n.sum()), fused


def measured_traffic(kernel_name, workload):
    """HBM bytes per launch of the dominant kernel as counted by the profiler (FETCH_SIZE + WRITE_SIZE,
    calibrated against plain read/copy kernels): a figure taken from the committed counter summary of
    this kernel and workload, or None if there is none (the counters cannot be read from inside a run)."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "hbm_traffic.txt")
    try:
        for line in open(path):
            f = line.split()
            if len(f) >= 3 and f[0] == kernel_name and f[1] == workload:
                return int(f[2])
    except OSError:
        pass
    return None


def _cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.lower().startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def _oracle_worker(job):
    """Steps the oracle over this worker's units (their own caches and the workload's own step inputs,
    cycled) until the deadline; one BLAS thread.  Returns (cached entries attended, wall seconds)."""
    import numpy as np
    from threadpoolctl import threadpool_limits
    from oracle import crystal_kv as ok
    cfg, t_now, caches, inputs, seconds = job
    o = ok.CrystalKVOracle(1, 1, cfg.group * len(caches), len(caches), cfg.head_dim,
                           np.asarray([c[1] for c in caches]).reshape(1, 1, -1), lam=cfg.lam, top_p=cfg.top_p, t0=t_now)
    for i, (c, _) in enumerate(caches):
        o.set_unit((0, 0, i), c.K, c.V, c.pos, c.crf, c.tau)
    entries = 0
    with threadpool_limits(limits=1):
        t0 = time.perf_counter()
        s = 0
        while time.perf_counter() - t0 < seconds:
            for i in range(len(caches)):
                q, k, v = inputs[i][s % len(inputs[i])]
                o.step_unit((0, 0, i), q, k, v)
                entries += o.units[(0, 0, i)].n + 1
            o.t += 1
            s += 1
        dt = time.perf_counter() - t0
    return entries, dt


def cpu_baseline(cfg, budgets, seconds=8.0, n_inputs=8):
    """The numpy oracle, as it stands, on the host: units spread over the workload, each with its steady-state
    cache and the rows the workload's own step generator gives it; one thread, then one process per host core
    over independent units.  Scaled by cached entries to the whole workload.  Runs before anything touches the
    GPU (the worker processes are forked)."""
    import multiprocessing as mp
    import numpy as np
    from paper_2601_16986_amd import workloads as wl

    cores = max(1, min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "16") or 16), 16))
    flat = np.asarray(budgets).reshape(-1)
    shape = np.asarray(budgets).shape
    t_now = cfg.prompt + cfg.decode_steps // 2
    m = wl.mean_query(cfg)
    n_units = 2 * cores
    sample = sorted(set(int(u) for u in np.linspace(0, flat.size - 1, n_units).astype(int)))
    keys = [tuple(int(v) for v in np.unravel_index(u, shape)) for u in sample]
    G = cfg.group
    steps_in, r = [], None
    for s in range(n_inputs):                                   # the workload's own decode-step inputs (all layers), untimed
        q, k, v, r = wl.decode_inputs(cfg, s, m, r)
        steps_in.append([(q[l, b, h * G:(h + 1) * G].copy(), k[l, b, h].copy(), v[l, b, h].copy()) for (l, b, h) in keys])
    caches = [(wl.steady_unit(cfg, u, int(flat[u]), t_now, m[key]), int(flat[u])) for u, key in zip(sample, keys)]
    inputs = [[steps_in[s][i] for s in range(n_inputs)] for i in range(len(sample))]
    total_entries = int((flat.astype(np.int64) + 1).sum())
    # one thread: every other sampled unit
    one = list(range(0, len(sample), max(1, len(sample) // 6)))[:6]
    e1, dt1 = _oracle_worker((cfg, t_now, [caches[i] for i in one], [inputs[i] for i in one], seconds))
    single = (e1 / dt1) / total_entries
    # all host cores: one process per core, each with its own units
    jobs = [(cfg, t_now, caches[w::cores], inputs[w::cores], seconds) for w in range(cores) if caches[w::cores]]
    with mp.get_context("fork").Pool(len(jobs)) as pool:
        res = pool.map(_oracle_worker, jobs)
    rate = sum(e / dt for e, dt in res)
    return {"value": rate / total_entries, "unit": "steps/s", "cores": len(jobs), "kind": "oracle",
            "host_cpus": os.cpu_count(), "cpu_model": _cpu_model(),
            "single_thread": {"value": single, "unit": "steps/s", "cores": 1},
            "sample": f"{len(sample)} units spread over the workload with their steady-state caches and the workload's own "
                      f"step inputs ({n_inputs} steps, cycled): one thread over {len(one)} of them for {dt1:.1f} s "
                      f"({e1} cached entries), then {len(jobs)} processes (one BLAS thread each) over all of them for "
                      f"{max(dt for _, dt in res):.1f} s ({sum(e for e, _ in res)} cached entries); "
                      f"scaled by entries to all {flat.size} units ({total_entries} entries per step)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=128)
    ap.add_argument("--warmup", type=int, default=256)
    ap.add_argument("--repeats", type=int, default=5, help="the K timed steps are run this many times; the median is reported")
    ap.add_argument("--config", default="qwen14b")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-layer", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="time eager launches instead of graph replays")
    ap.add_argument("--headroom", type=int, default=1,
                    help="1 (default): shared pools, a unit owns the 256-slot segments its budget + 1 entries need; "
                         "0: every unit owns room for the largest budget")
    ap.add_argument("--no-placement", action="store_true",
                    help="take the buffers wherever the allocator puts them instead of choosing their place by the start-up "
                         "calibration (ckv.place_pools)")
    ap.add_argument("--pool-factor", type=float, default=1.0, help="pools this many times what ckv_pool_slots asks for (measurement aid)")
    ap.add_argument("--path", type=int, default=0,
                    help="kernels of the all-layers step: 0 default, 1 separate scan/finish, 3 / 4 fused with 4 / 2 wavefronts per unit")
    ap.add_argument("--fullkv", type=int, default=0, metavar="TOKENS",
                    help="FullKV baseline instead: every unit holds TOKENS positions, attention-only steps, no eviction")
    ap.add_argument("--seed-prompt", default="", metavar="P,W",
                    help="instead: time ckv_seed_prompt (scores of a P-token prompt from its last W queries) over all layers")
    ap.add_argument("--probe-only", action="store_true",
                    help="only run the plain streaming-read and copy kernels (4 GiB each): counter calibration")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (units are independent; nothing is sharded); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    from paper_2601_16986_amd import workloads as wl

    cfg = wl.CONFIGS[args.config]
    fullkv = args.fullkv > 0
    plain = not (fullkv or args.seed_prompt or args.probe_only)
    # the host leg first: its worker processes are forked, which must happen before the GPU is initialised
    cpu = None
    if plain and not args.no_cpu_baseline:
        cpu = cpu_baseline(cfg, wl.draw_budgets(cfg))

    import torch
    device = torch.device("cuda:0")
    torch.cuda.set_device(device)
    from paper_2601_16986_amd import ckv
    read_gbps = ckv.bandwidth_probe(4 << 30, copy=False)
    copy_gbps = ckv.bandwidth_probe(4 << 30, copy=True)
    if args.probe_only:
        print(json.dumps({"stream_read_gbps": read_gbps, "copy_gbps": copy_gbps, "bytes": 4 << 30}))
        return
    if args.seed_prompt:
        print(json.dumps(seed_prompt_bench(cfg, device, *[int(x) for x in args.seed_prompt.split(",")])))
        return
    steps = max(1, args.steps)
    warm = max(1, args.warmup)
    repeats = max(1, args.repeats)
    if fullkv:
        g, budgets, (rq, rk, rv) = build_fullkv(cfg, device, args.fullkv, warm + (repeats + 2) * steps + 4 * RING)
    else:
        g, budgets, (rq, rk, rv) = build_workload(cfg, device, headroom=args.headroom, pool_factor=args.pool_factor,
                                                      pools=None if (args.no_placement or fullkv) else "place")
    if args.path:
        g.set_path(args.path)
    out = torch.empty(rq.shape[1:], dtype=torch.float32, device=device)
    R = 0 if fullkv else cfg.rebudget_interval

    def eager_steps(k):
        for i in range(k):
            g.decode_step(rq[i % RING], rk[i % RING], rv[i % RING], out=out, evict=not fullkv, attention_only=fullkv)

    # warm-up, with fresh inputs every RING steps like the timed region (replayed inputs fill the caches with
    # duplicate keys, see RING)
    done = 0
    while done < warm:
        if done and getattr(g, "refill", None) is not None:
            g.refill()
        k = min(RING, warm - done)
        eager_steps(k)
        done += k
    torch.cuda.synchronize()
    assert g.status() == 0, "a unit overflowed during warm-up"

    # ---- timed region: exactly `steps` decode steps (HIP-graph replays of up to RING consecutive steps, then a
    # shorter graph for what is left), synchronised on both sides; `repeats` such regions, the median is reported
    n_full, n_tail = divmod(steps, RING)
    g_full = g_tail = None
    if not args.no_graph:
        if n_full:
            g_full = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_full):
                eager_steps(RING)
        if n_tail:
            g_tail = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_tail):
                eager_steps(n_tail)
        torch.cuda.synchronize()
    # Every RING steps the ring is refilled with fresh inputs; the refills (input generation, not part of the
    # path) are kept out of the clock: the K steps are timed in pieces of up to RING steps, each piece
    # synchronised on both sides, and a repeat's time is the sum of its pieces.
    refill = getattr(g, "refill", None)
    times = []
    for _ in range(repeats):
        total = 0.0
        pieces = [RING] * n_full + ([n_tail] if n_tail else [])
        for k in pieces:
            if refill is not None:
                refill()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            if args.no_graph:
                eager_steps(k)
            else:
                (g_full if k == RING else g_tail).replay()
            torch.cuda.synchronize()
            total += time.perf_counter() - t0
        times.append(total * 1e3 / steps)
    ms_steps_only = float(np.median(times))
    assert g.status() == 0

    # ---- roofline pass: eager, HIP events around every launch of the dominant kernel
    if refill is not None:
        refill()
    g.profile_enable(True)
    eager_steps(RING)
    scan_ms, launches = g.profile_read()
    g.profile_enable(False)
    lengths = g.lengths()
    if not fullkv:
        assert np.array_equal(lengths, g.budgets()), "caches are not at their budgets after the run"
    scan_bytes, step_bytes, entries, fused_bytes = algorithmic_bytes(cfg, lengths - 1 if fullkv else g.budgets())
    if fullkv:                                           # attention only: K, V, q, out
        fused_bytes = step_bytes = scan_bytes + int(cfg.n_units) * cfg.group * 512
    fused_waves, _ = g.path_info()
    # dominant kernel of an all-layers step: the fused per-unit kernel if the context uses it, else the scan kernel
    kernel_name = f"unit_kernel<{fused_waves}>" if fused_waves else "scan_kernel<false>"
    kernel_bytes = fused_bytes if fused_waves else scan_bytes
    scan_avg_ms = scan_ms / max(launches, 1)
    achieved = kernel_bytes / (scan_avg_ms * 1e-3) / 1e9
    traffic = None if fullkv else measured_traffic(kernel_name, cfg.name)

    # ---- secondary: the shape a real model imposes, one call per layer
    per_layer = per_layer_deferred = None
    if not args.no_per_layer and not args.no_graph and not fullkv:
        outl = out[0]

        def layer_steps(k, defer):
            for i in range(k):
                for l in range(cfg.n_layers):
                    g.decode_step(rq[i % RING, l], rk[i % RING, l], rv[i % RING, l], layer=l, out=outl, defer=defer)

        res_pl = []
        for defer in (False, True):          # plain, then with the layers' bookkeeping on the context's own streams
            layer_steps(1, defer)
            g.join()
            torch.cuda.synchronize()
            gl = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gl):
                layer_steps(RING, defer)
                g.join()
            torch.cuda.synchronize()
            tl = []
            for _ in range(3):
                if refill is not None:
                    refill()
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                gl.replay()
                torch.cuda.synchronize()
                tl.append((time.perf_counter() - t1) * 1e3 / RING)
            res_pl.append(float(np.median(tl)))
            del gl
        per_layer, per_layer_deferred = res_pl

    # ---- Alg. 2 at its interval.  A re-allocation moves the caches away from the steady state the workload
    # defines (shrunken units drop thousands of entries at once, grown ones refill one entry per step), so it is
    # measured last and charged per step: what ckv_rebudget plus the step after it (which evicts down to the
    # new budgets) take beyond an ordinary step, divided by the interval.
    rebudget = None
    ms_per_step = ms_steps_only
    if R:
        def timed(fn):
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t1) * 1e3
        plain_ms = float(np.median([timed(lambda: eager_steps(1)) for _ in range(5)]))
        with_ms = timed(lambda: (g.rebudget(), eager_steps(1)))
        extra = max(0.0, with_ms - plain_ms)
        after = g.budgets()
        assert np.array_equal(after.sum(axis=(0, 2)), np.asarray(budgets).sum(axis=(0, 2))) and g.status() == 0
        ms_per_step = ms_steps_only + extra / R
        rebudget = {"interval": R, "rebudget_plus_next_step_ms": with_ms, "ordinary_eager_step_ms": plain_ms,
                    "amortised_ms_per_step": extra / R, "budgets_changed": int((after != np.asarray(budgets)).sum())}

    res = {
        "metric": "decode steps/s (attention + LRFU + evict, all layers per step)" if not fullkv
                  else "decode steps/s (FullKV baseline: attention only, nothing evicted)",
        "value": 1e3 / ms_per_step,
        "unit": "steps/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warm,
        "repeats": repeats,
        "ms_per_step": ms_per_step,
        "ms_per_step_repeats": times,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": (f"{cfg.name}: {cfg.n_layers} layers, {cfg.n_q_heads}/{cfg.n_kv_heads} heads, d=128, "
                                f"batch {cfg.batch}, mean budget {cfg.budget} "
                                f"({cfg.budget_min}..{cfg.budget_max}), evict every step, steady state at t={cfg.prompt + cfg.decode_steps // 2}"
                                + (f", Alg. 2 every {R} steps (amortised)" if R else ""))
                   if not fullkv else
                   (f"{cfg.name} FullKV: {cfg.n_layers} layers, {cfg.n_q_heads}/{cfg.n_kv_heads} heads, d=128, batch {cfg.batch}, "
                    f"every cache holds all {args.fullkv} positions and grows by one per step"),
                   "units": int(cfg.n_units), "entries_per_step": entries,
                   "launch": ("all layers per call, eager" if args.no_graph else
                              f"all layers per call, HIP graphs of up to {RING} steps, fresh inputs every {RING} steps, median of {repeats} timed regions of {steps} steps"),
                   "memory": (None if fullkv else
                              {"pool_slots": int(g.pool_slots), "kv_pool_bytes": int(2 * g.pool_slots * 256),
                               "budgeted_entry_bytes": int((np.asarray(budgets, dtype=np.int64) + 1).sum() * 512),
                               "headroom": int(g.headroom), "placement": getattr(g, "placement", None)})},
        "rebudget": rebudget,
        "kv_gbps": step_bytes / (ms_per_step * 1e-3) / 1e9,
        "hbm_frac": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "per_layer_graph_ms_per_step": per_layer,
        "per_layer_deferred_graph_ms_per_step": per_layer_deferred,   # same, CKV_DEFER_BOOKKEEPING on every call
        "stream_read_gbps": read_gbps,          # plain non-temporal streaming read measured on this machine
        "copy_gbps": copy_gbps,
        "roofline": {"bound": "hbm", "kernel": kernel_name, "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic,
                     "traffic_source": "profiles/hbm_traffic.txt (rocprofv3 --pmc summary of this kernel and workload, committed)"
                     if traffic is not None else None,
                     "bytes_per_launch": kernel_bytes, "avg_launch_ms": scan_avg_ms, "launches": launches,
                     "frac_of_stream_read": achieved / read_gbps},
    }
    if cpu is not None:
        res["cpu_baseline"] = cpu
    g.close()
    print(json.dumps(res))


if __name__ == "__main__":
    main()
