"""The parity helper's own logic, on the CPU: which GPU/oracle differences `compare_unit` accepts.

A stand-in for the GPU context returns states built by hand from the oracle's recorded step; the helper
must accept the oracle's own state, accept (and count) a state in which only entries at the edge of a
sub-margin top-p decision were decided the other way, and reject everything else: any difference when
the decision is not sub-margin, and, when it is, a flipped entry away from the edge, a wrong score on an
entry the flip does not reach, a wrong eviction."""
import math

import numpy as np
import pytest

from oracle import crystal_kv as ok
from tests import parity


class FakeGpu:
    """Holds one unit's state the way ckv.CrystalKV.export_unit reports it."""

    def __init__(self):
        self.state = None
        self.imported = 0

    def export_unit(self, l, b, h, with_kv=True):
        return self.state

    def import_unit(self, l, b, h, K, V, crf, tau, pos, t_unit):
        self.imported += 1


def _state(pos, crf, tau, hit, evicted_pos, shuffle_seed=0):
    perm = np.random.default_rng(shuffle_seed).permutation(len(pos))          # slot order is unspecified
    return dict(n=len(pos), pos=np.asarray(pos, np.int32)[perm], crf=np.asarray(crf, np.float32)[perm],
                tau=np.asarray(tau, np.int32)[perm], flags=np.asarray(hit, np.uint8)[perm],
                evicted_pos=np.sort(np.asarray(evicted_pos, np.int32)))


def _step(weights, budget=4, p=0.6):
    """One unit with 5 old entries (positions 0..4, distinct stored scores) takes a step at t = 5 with the
    given attention weights over positions 0..5."""
    d = 8
    o = ok.CrystalKVOracle(1, 1, 1, 1, d, np.full((1, 1, 1), budget), lam=0.5, top_p=p, softmax_scale=1.0, t0=5)
    K = np.eye(d)[:5]
    o.load_prompt(0, K[None, None], np.zeros((1, 1, 5, d)), crf0=np.array([[[1.0, 1.5, 1.25, 1.75, 1.125]]], np.float32),
                  tau0=np.array([[[4, 4, 3, 4, 2]]]))
    k_new = np.eye(d)[5]
    q = np.log(np.concatenate([np.asarray(weights, np.float64), np.full(d - 6, 1e-300)]))
    rec = o.step_unit((0, 0, 0), q[None, :], k_new, np.zeros(d))
    o.t += 1
    return o, rec


def _oracle_state(o):
    u = o.units[(0, 0, 0)]
    return _state(u.pos, u.crf, u.tau, u.hit, u.last_evicted)


def test_identical_state_passes_and_clear_decisions_admit_no_difference():
    o, rec = _step([0.05, 0.4, 0.1, 0.3, 0.05, 0.1])
    assert rec.decision.sum_margin > 1e-3 and rec.decision.edge_gap > 1e-3
    g, stats = FakeGpu(), parity.LockstepStats()
    g.state = _oracle_state(o)
    assert parity.compare_unit(g, o, (0, 0, 0), rec, stats) is False and stats.resynced == 0
    bad = _oracle_state(o)
    bad["crf"] = bad["crf"].copy()
    bad["crf"][0] = np.nextafter(bad["crf"][0], np.float32(9))             # one ulp on one score
    g.state = bad
    with pytest.raises(AssertionError):
        parity.compare_unit(g, o, (0, 0, 0), rec, stats)
    assert g.imported == 0


def _alternative(o, rec, flip_pos):
    """The state Alg. 1 leaves if the entries at positions `flip_pos` are decided the other way (built
    here step by step, not through the helper under test)."""
    hit = rec.decision.hit.copy()
    for p_ in flip_pos:
        i = int(np.nonzero(rec.pre_pos == p_)[0][0])
        hit[i] = not hit[i]
    dec = np.float32(0.5) ** (rec.t - rec.pre_tau).astype(np.float32)
    tmp = (dec * rec.pre_crf).astype(np.float32) + hit.astype(np.float32)
    crf = np.where(hit, tmp, rec.pre_crf)
    tau = np.where(hit, rec.t, rec.pre_tau)
    order = sorted(range(len(hit)), key=lambda i: (-float(tmp[i]), int(rec.pre_pos[i])))
    keep, gone = sorted(order[:rec.budget]), sorted(order[rec.budget:])
    return _state(rec.pre_pos[keep], crf[keep], tau[keep], hit[keep], rec.pre_pos[gone], shuffle_seed=3)


def test_sub_margin_cut_accepts_only_flips_of_the_edge_entries():
    # cumulative weight of the first two lands 4e-7 above p = 0.6: the GPU may need a third entry
    o, rec = _step([0.05, 0.35 + 4e-7, 0.1, 0.25, 0.05 - 4e-7, 0.2])
    d = rec.decision
    assert d.m_star == 2 and d.sum_margin == pytest.approx(4e-7 - (float(np.float32(0.6)) - 0.6), rel=1e-3) and d.edge_gap > 1e-2
    assert rec.pre_pos[parity.edge_entries(rec)].tolist() == [3]            # position 5 is the new entry: always a hit
    g, stats = FakeGpu(), parity.LockstepStats()
    g.state = _alternative(o, rec, [3])                                       # position 3 (0.25) falls out of the nucleus
    assert parity.compare_unit(g, o, (0, 0, 0), rec, stats) is True
    assert stats.resynced == 1 and g.imported == 1 and stats.notes[0][1] == (0, 0, 0)
    # a flip away from the edge is not excused by the small margin
    g.state = _alternative(o, rec, [2])
    with pytest.raises(AssertionError):
        parity.compare_unit(g, o, (0, 0, 0), rec, stats)
    # nor is an edge flip combined with a wrong score elsewhere
    bad = _alternative(o, rec, [3])
    i1 = int(np.nonzero(bad["pos"] == 1)[0][0])
    bad["crf"] = bad["crf"].copy()
    bad["crf"][i1] += np.float32(0.5)
    g.state = bad
    with pytest.raises(AssertionError):
        parity.compare_unit(g, o, (0, 0, 0), rec, stats)
    # nor an edge flip with another victim than Alg. 1 Step 4 picks for it
    bad = _alternative(o, rec, [3])
    good_victims = bad["evicted_pos"].tolist()
    survivor = int(bad["pos"][0])
    bad["evicted_pos"] = np.array(sorted(good_victims[:-1] + [survivor]), np.int32)
    g.state = bad
    with pytest.raises(AssertionError):
        parity.compare_unit(g, o, (0, 0, 0), rec, stats)
    assert stats.resynced == 1
    # with resynchronisation switched off even the admissible alternative fails
    g.state = _alternative(o, rec, [3])
    with pytest.raises(AssertionError):
        parity.compare_unit(g, o, (0, 0, 0), rec, stats, allow_resync=False)


def test_near_tie_at_the_edge_accepts_the_swap():
    a_in = 0.2
    a_out = a_in * (1 - 2e-7)
    o, rec = _step([0.02, 0.45, a_in, a_out, 0.03, 1 - 0.5 - a_in - a_out], p=0.6)
    d = rec.decision
    assert d.m_star == 2 and d.edge_gap == pytest.approx(2e-7, rel=1e-3) and d.sum_margin > 1e-2
    assert rec.pre_pos[parity.edge_entries(rec)].tolist() == [2, 3]
    g, stats = FakeGpu(), parity.LockstepStats()
    g.state = _alternative(o, rec, [2, 3])                                    # the GPU ranks position 3 above position 2
    assert parity.compare_unit(g, o, (0, 0, 0), rec, stats) is True and stats.resynced == 1
    g.state = _alternative(o, rec, [1])
    with pytest.raises(AssertionError):
        parity.compare_unit(g, o, (0, 0, 0), rec, stats)


def test_steps_without_eviction_replay_without_eviction():
    o, rec = _step([0.05, 0.35 + 4e-7, 0.1, 0.25, 0.05 - 4e-7, 0.2], budget=4)
    # undo the oracle's eviction for this check: a step run with evict=False keeps all six entries
    o2 = ok.CrystalKVOracle(1, 1, 1, 1, 8, np.full((1, 1, 1), 4), lam=0.5, top_p=0.6, softmax_scale=1.0, t0=5)
    o2.load_prompt(0, np.eye(8)[:5][None, None], np.zeros((1, 1, 5, 8)), crf0=np.array([[[1.0, 1.5, 1.25, 1.75, 1.125]]], np.float32),
                   tau0=np.array([[[4, 4, 3, 4, 2]]]))
    q = np.log(np.concatenate([[0.05, 0.35 + 4e-7, 0.1, 0.25, 0.05 - 4e-7, 0.2], np.full(2, 1e-300)]))
    rec2 = o2.step_unit((0, 0, 0), q[None, :], np.eye(8)[5], np.zeros(8), evict=False)
    o2.t += 1
    assert o2.units[(0, 0, 0)].n == 6
    from dataclasses import replace
    alt = _alternative(o2, replace(rec2, budget=6), [3])
    g, stats = FakeGpu(), parity.LockstepStats()
    g.state = alt
    assert parity.compare_unit(g, o2, (0, 0, 0), rec2, stats, evicting=False) is True
    with pytest.raises(AssertionError):                                       # as an evicting step the same state is wrong
        parity.compare_unit(g, o2, (0, 0, 0), rec2, stats, evicting=True)
    assert math.isinf(rec2.evict_gap)
