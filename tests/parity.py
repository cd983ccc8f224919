"""Lock-step comparison of the HIP path with the CPU oracle (test helper).

Both sides consume the same seeded inputs.  Information flows from the oracle
to the GPU only.  When a hit decision lies within rounding distance of its
threshold (the oracle's own margins say so, and they are pinned by the CPU
tests) the GPU may have decided the other way for the entries at the edge of
the nucleus, and for those alone: the oracle replays Alg. 1 Steps 2-4 of that
unit under every admissible alternative decision, the GPU's whole state must
equal one of the outcomes bit for bit, the event is counted and the GPU unit is
re-imported from the oracle's own state.  Any other difference fails the test.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

# Output tolerance (bf16 inputs, fp32 accumulation): |gpu - ref| <= OUT_TOL * max(|ref|, 1e-2 * max|ref row|).
OUT_TOL = 2e-3
# A top-p cut closer than this to p (absolute, p ~ 1) or two edge weights closer than
# this (relative) may legitimately fall either way: the GPU's weights carry ~1e-6
# relative error from fp32 accumulation and the hardware exp2.
MARGIN_TOL = 1e-5


def out_error(out_gpu, out_ref):
    out_gpu = np.asarray(out_gpu, np.float64)
    den = np.maximum(np.abs(out_ref), 1e-2 * np.abs(out_ref).max(axis=-1, keepdims=True))
    return float((np.abs(out_gpu - out_ref) / den).max())


@dataclass
class LockstepStats:
    steps: int = 0
    unit_steps: int = 0
    resynced: int = 0                 # unit-steps re-imported after a sub-margin decision
    max_out_err: float = 0.0
    notes: list = field(default_factory=list)


def sync_unit_to_gpu(g, o, key):
    u = o.units[key]
    g.import_unit(*key, u.K.astype(np.float32), u.V.astype(np.float32), u.crf, u.tau, u.pos, o.t - 1)


def edge_entries(rec, tol=MARGIN_TOL):
    """Indices (into the step's pre-update arrays) of the entries a sub-margin decision may flip: the last
    entry inside the nucleus and the first outside when the cut's sum lies within `tol` of p, and every
    entry whose weight lies within `tol` (relative) of the weight at the cut.  `rec`: a StepRecord, or a
    HitDecision whose last entry is the one that arrived in its step."""
    d = getattr(rec, "decision", rec)
    abar = d.abar
    n = len(abar)
    edge = set()
    if d.m_star >= 1:
        a_cut = abar[d.order[d.m_star - 1]]
        if d.sum_margin < tol:
            edge.add(int(d.order[d.m_star - 1]))
            if d.m_star < n:
                edge.add(int(d.order[d.m_star]))
        if d.edge_gap < tol:
            edge.update(int(i) for i in np.nonzero(np.abs(abar - a_cut) <= tol * a_cut)[0])
    edge.discard(n - 1)                     # the entry appended this step is a hit whatever its weight
    return sorted(edge)


def admissible_outcomes(o, rec, max_edge=6):
    """States the unit may be in after the step if the hit bits of the edge entries fall either way:
    Steps 2-4 of Alg. 1 replayed by the oracle's own functions from the recorded pre-update state.
    Yields dicts of pos, crf, tau, hit (position-sorted) and evicted_pos."""
    from itertools import product
    from oracle import crystal_kv as ok
    edge = edge_entries(rec)
    assert 0 < len(edge) <= max_edge, f"{len(edge)} entries at the edge of the nucleus"
    base = rec.decision.hit
    for bits in product((False, True), repeat=len(edge)):
        hit = base.copy()
        hit[edge] = bits
        if np.array_equal(hit, base):
            continue
        tmp, crf, tau = ok.crf_update(rec.pre_crf, rec.pre_tau, rec.t, hit.astype(np.float32), hit, o.tab)
        retain, evicted = ok.evict_select(tmp, rec.pre_pos, rec.budget)
        srt = retain[np.argsort(rec.pre_pos[retain])]
        yield dict(pos=rec.pre_pos[srt], crf=crf[srt], tau=tau[srt], hit=hit[srt], evicted_pos=np.sort(rec.pre_pos[evicted]))


def compare_unit(g, o, key, rec, stats, *, check_kv=False, allow_resync=True, evicting=True):
    """Compare one unit after a step.  Returns True if the unit was re-imported."""
    u = o.units[key]
    e = g.export_unit(*key, with_kv=check_kv)
    gp = e["pos"]
    order_g = np.argsort(gp)
    order_o = np.argsort(u.pos)
    same = (e["n"] == u.n and np.array_equal(gp[order_g], u.pos[order_o])
            and np.array_equal(e["crf"][order_g].view(np.uint32), u.crf[order_o].view(np.uint32))
            and np.array_equal(e["tau"][order_g], u.tau[order_o])
            and np.array_equal((e["flags"][order_g] & 1).astype(bool), u.hit[order_o])
            and np.array_equal(e["evicted_pos"], rec.evicted_pos if rec is not None else e["evicted_pos"]))
    if same and check_kv:
        same = (np.array_equal(e["K"][order_g], u.K[order_o].astype(np.float32))
                and np.array_equal(e["V"][order_g], u.V[order_o].astype(np.float32)))
        assert same, f"unit {key}: K/V rows differ after compaction"
    if same:
        return False
    d = rec.decision if rec is not None else None
    sub_margin = d is not None and (d.sum_margin < MARGIN_TOL or d.edge_gap < MARGIN_TOL)
    if not (allow_resync and sub_margin):
        msg = [f"unit {key} differs at t={o.t - 1}: n gpu {e['n']} oracle {u.n}"]
        if d is not None:
            msg.append(f"sum_margin {d.sum_margin:.3e} edge_gap {d.edge_gap:.3e} m* {d.m_star}")
        sg, so = set(gp.tolist()), set(u.pos.tolist())
        msg.append(f"only gpu {sorted(sg - so)[:10]} only oracle {sorted(so - sg)[:10]}")
        if sg == so:
            bad = np.nonzero(e["crf"][order_g] != u.crf[order_o])[0][:10]
            msg.append(f"crf differs at pos {gp[order_g][bad].tolist()} gpu {e['crf'][order_g][bad].tolist()} "
                       f"oracle {u.crf[order_o][bad].tolist()}")
            badt = np.nonzero(e["tau"][order_g] != u.tau[order_o])[0][:10]
            msg.append(f"tau differs at pos {gp[order_g][badt].tolist()}")
            badh = np.nonzero((e["flags"][order_g] & 1).astype(bool) != u.hit[order_o])[0][:10]
            msg.append(f"hit differs at pos {gp[order_g][badh].tolist()}")
            if rec is not None:
                msg.append(f"evicted gpu {np.asarray(e['evicted_pos']).tolist()[:20]} oracle {np.asarray(rec.evicted_pos).tolist()[:20]}")
        raise AssertionError("\n".join(msg))
    # sub-margin: the GPU's state must be what Alg. 1 gives when only edge entries' hit bits differ
    gs = dict(pos=gp[order_g], crf=e["crf"][order_g].view(np.uint32), tau=e["tau"][order_g],
              hit=(e["flags"][order_g] & 1).astype(bool), evicted_pos=e["evicted_pos"])
    if not evicting:
        rec = _without_eviction(rec)
    matched = any(len(c["pos"]) == len(gs["pos"]) and np.array_equal(c["pos"], gs["pos"])
                  and np.array_equal(c["crf"].view(np.uint32), gs["crf"]) and np.array_equal(c["tau"], gs["tau"])
                  and np.array_equal(c["hit"], gs["hit"]) and np.array_equal(c["evicted_pos"], gs["evicted_pos"])
                  for c in admissible_outcomes(o, rec))
    assert matched, (f"unit {key} at t={o.t - 1}: the decision is sub-margin (sum_margin {d.sum_margin:.3e}, edge_gap "
                     f"{d.edge_gap:.3e}) but the GPU's state is none of the outcomes that flipping the edge entries "
                     f"{rec.pre_pos[edge_entries(rec)].tolist()} allows")
    stats.resynced += 1
    stats.notes.append((o.t - 1, key, d.sum_margin, d.edge_gap))
    sync_unit_to_gpu(g, o, key)
    return True


def _without_eviction(rec):
    """The record of a step that ran without Step 4: the replay must not evict either."""
    from dataclasses import replace
    return replace(rec, budget=len(rec.pre_pos))


def lockstep(g, o, stream, n_steps, *, evict=True, check_kv_every=0, on_step=None):
    """Run n_steps decode steps on both sides (all layers per call)."""
    stats = LockstepStats()
    for s in range(n_steps):
        ref, recs = o.decode_step(stream.q[s], stream.k_new[s], stream.v_new[s], evict=evict)
        out = g.decode_step(stream.q[s], stream.k_new[s], stream.v_new[s], evict=evict).cpu().numpy()
        stats.max_out_err = max(stats.max_out_err, out_error(out, ref))
        assert stats.max_out_err <= OUT_TOL, f"step {s}: attention output off by {stats.max_out_err}"
        ck = bool(check_kv_every) and (s % check_kv_every == check_kv_every - 1)
        for key, rec in recs.items():
            compare_unit(g, o, key, rec, stats, check_kv=ck, evicting=evict)
            stats.unit_steps += 1
        stats.steps += 1
        if on_step is not None:
            on_step(s)
    return stats
