"""CPU oracle for the Crystal-KV decode hot path.

TEST INFRASTRUCTURE ONLY.  This module is a plain, slow, by-eye-checkable numpy
implementation of what the method computes per decode step.  Nothing on the
product path may import it: only tests, the smoke check and the benchmark's
`cpu_baseline` leg do.  It shares no code, table or constant generator with
the HIP library and never reads anything the HIP library produced.

What follows which passage of the paper (arxiv 2601.16986):

* `attention`            - Sec. 2.2: AttnScore = softmax(q K^T), y = AttnScore V,
                           the new (k, v) appended before attending.
* `hit_mask`             - Sec. 5.2 and Alg. 1 Step 1: top-p nucleus over the
                           attention weights = smallest set whose cumulative
                           weight exceeds p.
* `crf_closed_form`      - Sec. 5.2, CRF definition: sum_j lambda^(t - t_j).
* `decay_table`,
  `crf_update`           - Sec. 5.2 incremental CRF and Alg. 1 Steps 2-3: hits
                           store (lambda^(t-tau) CRF + 1, tau = t); misses only
                           get a temporary decayed score.
* `evict_select`         - Alg. 1 Step 4: Retain = TopK(CRF_temp, B), then gather
                           of CRF, tau, K, V.
* `budget_shares`        - Alg. 2 Steps 1-4 (real-valued), utilisation eta of
                           Sec. 5.3.
* `apportion`,
  `rebudget`             - integer budgets from Alg. 2's real ones (the paper is
                           silent on this; reading stated below).
* `probe_classes`        - Sec. 3: rank entries by the answer query's attention,
                           top 30 % = CrystalKV, bottom 30 % = SlipKV.
* `window_select`        - Sec. 2.3, the baseline that assumes attention goes to
                           the initial and the most recent tokens: keep the
                           sink positions and the newest entries (a comparison
                           policy on the same caches, not part of the method).
* `CrystalKVOracle`      - the per-step control flow of Sec. 4 / Alg. 1 over all
                           (layer, sequence, KV head) units.
* `CrystalKVOracle.seed_prompt`
                         - Alg. 1 Steps 1-3 replayed over the prompt's last
                           queries (the paper leaves the prompt's scores open;
                           reading stated below).

Readings where the paper is silent (each is a named parameter or stated here):

* softmax scale: the paper's formula has none; `softmax_scale` is a parameter
  (1/sqrt(d) in every workload here).
* GQA: one KV head serves G query heads; the per-entry weight used for the hit
  mask is the mean over those G softmax rows (still sums to 1).
* a new entry counts as referenced at its arrival step (classic LRFU insertion):
  it is appended with CRF = 0, tau = t and is always in that step's hit set, so
  it ends the step with CRF = 1 and the closed form holds with t_1 = arrival.
* "exceed p" is strict (>); entries with equal weight are ordered by lower
  position first; p >= 1 (or a total that never exceeds p) marks every entry.
* TopK ties: among equal CRF_temp the lower position is retained.
* the score update runs on every step; only Step 4 is gated, and it acts when
  the cache holds more entries than the budget.
* survivors keep their stored (CRF, tau), not CRF_temp (Alg. 1 gathers CRF).
* arithmetic of the score: fp32.  lambda^delta comes from a table
  TAB[delta] = float32(pow(double(lambda), delta)), values below FLT_MIN flushed
  to 0, TAB[0] = 1 (also for lambda = 0); delta is clamped to the last table
  index, which is the first delta whose entry is 0 (or 2^20 if none is; a table
  of one entry when lambda = 1).  CRF_temp = fl32(fl32(TAB[delta] * CRF) + r)
  with r = 1 for a hit and 0 for a miss (two roundings, no fused multiply-add),
  flushed to 0 below FLT_MIN.
* aggregated CRF of a head (Alg. 2 input): the sum of CRF_temp over the head's
  entries at the current step, accumulated in 2^-20 fixed point
  (floor(CRF_temp * 2^20) as an integer), averaged over the steps since the
  last re-allocation.
* integer budgets: see `apportion` and `rebudget`.
* prompt scores (`seed_prompt`): the paper starts Alg. 1 at decode time and
  says nothing about the scores the prompt's entries start with.  Reading: the
  last W prompt positions P-W .. P-1 are treated as W decode steps that have
  already happened, without eviction: the query of position t sees the entries
  of positions <= t (causal), Steps 1-3 run at time t, and position t's own
  entry, arriving at that step, is in its hit set (the insertion rule above).
  Entries before the window count as referenced once, on arrival (CRF = 1,
  tau = position).  Nothing of this enters the aggregated-CRF window of Alg. 2.
* reward_mode 1 ("attention weighted", a labelled variant, not the paper's
  Alg. 1): the reward is the entry's mean attention weight instead of 0/1, and
  every entry stores its score and tau each step.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

FLT_MIN = np.float32(1.17549435e-38)
TABLE_CAP = 1 << 20
FIXED_POINT_ONE = 1 << 20  # resolution of the aggregated-CRF accumulator

REWARD_TOPP_HIT = 0
REWARD_ATTN_WEIGHTED = 1

CLASS_SLIP = 0
CLASS_POTENTIAL = 1
CLASS_CRYSTAL = 2


# ----------------------------------------------------------------------------
# Sec. 2.2: attention
# ----------------------------------------------------------------------------
def attention(q, K, V, scale):
    """softmax(scale * q K^T) V in float64.

    q: [G, d] (the G query heads that share this KV head), K, V: [n, d].
    Returns (y [G, d], a [G, n]); each row of `a` sums to 1.
    """
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    s = float(scale) * (q @ K.T)
    s = s - s.max(axis=1, keepdims=True)
    e = np.exp(s)
    a = e / e.sum(axis=1, keepdims=True)
    return a @ V, a


# ----------------------------------------------------------------------------
# Sec. 5.2 / Alg. 1 Step 1: top-p hit mask
# ----------------------------------------------------------------------------
@dataclass
class HitDecision:
    hit: np.ndarray            # bool [n]
    m_star: int                # size of the nucleus (before forcing the new entry)
    order: np.ndarray          # entry indices, by (weight desc, position asc)
    sum_margin: float          # min(c_m* - p, p - c_(m*-1)): distance of the cut to p
    edge_gap: float            # relative weight gap between last-in and first-out
    abar: np.ndarray = None    # the weights the decision was taken on (record keeping)


def hit_mask(abar, pos, p, new_index=None):
    """Smallest set of entries, by descending weight, whose cumulative weight
    exceeds p; the entry at `new_index` (appended this step) is always a hit."""
    abar = np.asarray(abar, dtype=np.float64)
    pos = np.asarray(pos)
    n = abar.shape[0]
    order = np.lexsort((pos, -abar))           # weight desc, then position asc
    c = np.cumsum(abar[order])                 # sequential float64 running sum
    over = np.nonzero(c > p)[0]
    m_star = int(over[0]) + 1 if over.size else n
    hit = np.zeros(n, dtype=bool)
    hit[order[:m_star]] = True
    if new_index is not None:
        hit[new_index] = True
    # margins of the decision (used by parity tests to tell a real mismatch
    # from a cut that lies within rounding distance of p)
    if n == 0:
        return HitDecision(hit, 0, order, math.inf, math.inf)
    upper = c[m_star - 1] - p if over.size else math.inf
    lower = p - (c[m_star - 2] if m_star >= 2 else 0.0)
    if m_star < n:
        a_in, a_out = abar[order[m_star - 1]], abar[order[m_star]]
        edge = (a_in - a_out) / a_in if a_in > 0 else 0.0
    else:
        edge = math.inf
    return HitDecision(hit, m_star, order, float(min(upper, lower)), float(edge), abar)


# ----------------------------------------------------------------------------
# Sec. 5.2: CRF, closed form and incremental
# ----------------------------------------------------------------------------
def crf_closed_form(hit_times, t, lam):
    """CRF(e) = sum_j lambda^(t - t_j) in float64 (0^0 = 1)."""
    return float(sum(math.pow(float(lam), t - tj) for tj in hit_times))


def decay_table(lam):
    """TAB[delta] = float32(pow(double(float32(lambda)), delta)), flushed to 0
    below FLT_MIN; ends at the first 0 entry (or at TABLE_CAP)."""
    lam64 = float(np.float32(lam))
    if lam64 == 1.0:
        return np.ones(1, dtype=np.float32)
    tab = [np.float32(1.0)]
    for delta in range(1, TABLE_CAP + 1):
        v = np.float32(math.pow(lam64, delta))
        if v < FLT_MIN:
            v = np.float32(0.0)
        tab.append(v)
        if v == 0.0:
            break
    return np.asarray(tab, dtype=np.float32)


def crf_update(crf, tau, t, reward, store, tab):
    """One step of the incremental CRF for every entry of one head.

    crf float32 [n], tau int [n] (time the stored CRF refers to), `reward`
    float32 [n] (1/0 for hit/miss in the paper's Alg. 1), `store` bool [n]
    (which entries record the new score and time: the hits).
    Returns (crf_temp float32 [n], new_crf, new_tau).
    """
    crf = np.asarray(crf, dtype=np.float32)
    tau = np.asarray(tau, dtype=np.int64)
    delta = np.int64(t) - tau
    if np.any(delta < 0):
        raise ValueError("entry updated in the future")
    dec = tab[np.minimum(delta, tab.shape[0] - 1)]
    prod = (dec * crf).astype(np.float32)               # rounding 1
    tmp = (prod + np.asarray(reward, np.float32)).astype(np.float32)  # rounding 2
    tmp = np.where(tmp < FLT_MIN, np.float32(0.0), tmp).astype(np.float32)
    store = np.asarray(store, dtype=bool)
    new_crf = np.where(store, tmp, crf).astype(np.float32)
    new_tau = np.where(store, np.int64(t), tau)
    return tmp, new_crf, new_tau


def crf_sum_fixed(tmp):
    """Aggregated CRF of a head at this step, in 2^-20 fixed point (Python int)."""
    return int(np.floor(np.asarray(tmp, np.float64) * FIXED_POINT_ONE).astype(np.int64).sum())


# ----------------------------------------------------------------------------
# Alg. 1 Step 4: eviction
# ----------------------------------------------------------------------------
def evict_select(tmp, pos, budget):
    """Indices retained and evicted.  Retain = the `budget` entries that come
    first by (CRF_temp desc, position asc); returned in ascending index order."""
    tmp = np.asarray(tmp, dtype=np.float32)
    pos = np.asarray(pos)
    n = tmp.shape[0]
    if n <= budget:
        return np.arange(n), np.zeros(0, dtype=np.int64)
    order = np.lexsort((pos, -tmp.astype(np.float64)))
    retain = np.sort(order[:budget])
    evicted = np.sort(order[budget:])
    return retain, evicted


def window_select(pos, budget, n_sink):
    """Sink-plus-recent-window retention (Sec. 2.3: the baseline that keeps the
    initial and the most recent tokens).  Sinks are the entries whose position
    is below `n_sink`; they are kept first (lowest position first if even they
    exceed the budget), the rest of the budget goes to the highest positions.
    Returns (retain, evicted) as ascending index arrays."""
    pos = np.asarray(pos)
    n = pos.shape[0]
    if n <= budget:
        return np.arange(n), np.zeros(0, dtype=np.int64)
    idx = np.arange(n)
    sinks = sorted(idx[pos < n_sink], key=lambda i: pos[i])
    others = sorted(idx[pos >= n_sink], key=lambda i: -pos[i])
    keep = (sinks + others)[:budget]
    retain = np.sort(np.asarray(keep, dtype=np.int64))
    evicted = np.setdiff1d(idx, retain)
    return retain, evicted


# ----------------------------------------------------------------------------
# Sec. 3: answer-probe classes
# ----------------------------------------------------------------------------
def probe_classes(abar, pos):
    """Top floor(0.3 n) entries by (weight desc, position asc) are Crystal (2),
    the last floor(0.3 n) are Slip (0), the rest Potential (1)."""
    abar = np.asarray(abar, dtype=np.float64)
    n = abar.shape[0]
    k = (3 * n) // 10
    order = np.lexsort((np.asarray(pos), -abar))
    cls = np.full(n, CLASS_POTENTIAL, dtype=np.uint8)
    cls[order[:k]] = CLASS_CRYSTAL
    if k:
        cls[order[n - k:]] = CLASS_SLIP
    return cls


# ----------------------------------------------------------------------------
# Alg. 2: adaptive budget allocation
# ----------------------------------------------------------------------------
def budget_shares(C, B, B_total):
    """Alg. 2 in real numbers.  C, B: [L, H] aggregated CRF and current budgets.
    Returns (B_layer [L], B_head [L, H]) as float64."""
    C = np.asarray(C, dtype=np.float64)
    B = np.asarray(B, dtype=np.float64)
    L, H = C.shape
    eta_layer = np.zeros(L)
    for i in range(L):
        sc = 0.0
        sb = 0.0
        for j in range(H):
            sc += C[i, j]
            sb += B[i, j]
        eta_layer[i] = sc / sb                                    # Step 1
    sum_eta = 0.0
    for i in range(L):
        sum_eta += eta_layer[i]
    B_layer = np.zeros(L)
    B_head = np.zeros((L, H))
    for i in range(L):
        B_layer[i] = B_total * (eta_layer[i] / sum_eta)           # Step 2
        eta_head = np.zeros(H)
        s = 0.0
        for j in range(H):
            eta_head[j] = C[i, j] / B[i, j]                       # Step 3
            s += eta_head[j]
        for j in range(H):
            B_head[i, j] = B_layer[i] * (eta_head[j] / s)         # Step 4
    return B_layer, B_head


def apportion(x, total, lo, hi):
    """Integers v_k in [lo_k, hi_k] summing to `total`, proportional to the
    weights x_k >= 0 as far as the bounds allow.

    1. Water-filling in float64: y_k = R * (x_k / X) over the still-free
       entries (R = what the fixed entries leave of `total`, X = the free
       weights' sum; equal shares if X is 0).  While some y_k leaves its
       bounds: if the overshoot above the upper bounds is at least the
       shortfall below the lower ones, fix every entry above its upper bound
       there, otherwise fix every entry below its lower bound there; repeat.
    2. Free entries take floor(y_k); the remaining units go one each to the
       largest fractional parts (ties: lower index), never beyond a bound.
    3. Any difference still left (bounds in the way) is spread one unit at a
       time over all entries in index order, within the bounds.
    Requires sum(lo) <= total <= sum(hi).
    """
    m = len(x)
    lo = [int(v) for v in lo]
    hi = [int(v) for v in hi]
    total = int(total)
    if not (sum(lo) <= total <= sum(hi)):
        raise ValueError("apportion: total outside the bounds")
    fixed = [False] * m
    val = [0] * m
    y = [0.0] * m
    for _ in range(m + 1):
        R = total
        n_free = 0
        X = 0.0
        for k in range(m):
            if fixed[k]:
                R -= val[k]
            else:
                n_free += 1
                X += float(x[k])
        if n_free == 0:
            break
        over = 0.0
        under = 0.0
        for k in range(m):
            if fixed[k]:
                continue
            y[k] = float(R) * (float(x[k]) / X) if X > 0.0 else float(R) / float(n_free)
            if y[k] > hi[k]:
                over += y[k] - hi[k]
            if y[k] < lo[k]:
                under += lo[k] - y[k]
        if over == 0.0 and under == 0.0:
            break
        if over >= under:
            for k in range(m):
                if not fixed[k] and y[k] > hi[k]:
                    fixed[k] = True
                    val[k] = hi[k]
        else:
            for k in range(m):
                if not fixed[k] and y[k] < lo[k]:
                    fixed[k] = True
                    val[k] = lo[k]
    free = [k for k in range(m) if not fixed[k]]
    frac = [0.0] * m
    for k in free:
        f = math.floor(y[k])
        f = min(max(int(f), lo[k]), hi[k])
        val[k] = f
        frac[k] = y[k] - math.floor(y[k])
    rem = total - sum(val)
    order = sorted(free, key=lambda k: (-frac[k], k))
    if rem > 0:
        for k in order:
            if rem == 0:
                break
            if val[k] < hi[k]:
                val[k] += 1
                rem -= 1
    elif rem < 0:
        for k in reversed(order):
            if rem == 0:
                break
            if val[k] > lo[k]:
                val[k] -= 1
                rem += 1
    while rem != 0:
        moved = False
        for k in range(m):
            if rem > 0 and val[k] < hi[k]:
                val[k] += 1
                rem -= 1
                moved = True
            elif rem < 0 and val[k] > lo[k]:
                val[k] -= 1
                rem += 1
                moved = True
            if rem == 0:
                break
        if not moved:
            raise RuntimeError("apportion: cannot place the remainder")
    return val


def rebudget(C, B, B_total, b_min, b_max):
    """Integer budgets B'[L][H] for one sequence from Alg. 2.

    Two levels, as in Alg. 2: layers get integer totals apportioned to the
    layer utilisations eta_i with bounds [H b_min, H b_max] and sum B_total;
    inside layer i the heads get integers apportioned to eta_ij with bounds
    [b_min, b_max] and sum = that layer's integer total.  If the utilisations
    of all layers sum to 0 (or are not finite) the budgets stay as they are; a
    layer whose head utilisations sum to 0 splits its total equally.
    """
    C = np.asarray(C, dtype=np.float64)
    B = np.asarray(B, dtype=np.int64)
    L, H = C.shape
    eta_layer = [0.0] * L
    sum_eta = 0.0
    for i in range(L):
        sc = 0.0
        sb = 0.0
        for j in range(H):
            sc += float(C[i, j])
            sb += float(B[i, j])
        eta_layer[i] = sc / sb
        sum_eta += eta_layer[i]
    if not (sum_eta > 0.0) or not math.isfinite(sum_eta):
        return B.copy()
    layer_tot = apportion(eta_layer, B_total, [H * b_min] * L, [H * b_max] * L)
    out = np.zeros((L, H), dtype=np.int64)
    for i in range(L):
        eta_head = [float(C[i, j]) / float(B[i, j]) for j in range(H)]
        out[i] = apportion(eta_head, layer_tot[i], [b_min] * H, [b_max] * H)
    return out


# ----------------------------------------------------------------------------
# Whole path, all units
# ----------------------------------------------------------------------------
@dataclass
class Unit:
    """One (layer, sequence, KV head) cache."""
    K: np.ndarray        # [n, d] float64 (bf16 values held exactly)
    V: np.ndarray
    pos: np.ndarray      # [n] int64, position of the token each entry came from
    crf: np.ndarray      # [n] float32
    tau: np.ndarray      # [n] int64
    budget: int
    hit: np.ndarray = field(default_factory=lambda: np.zeros(0, dtype=bool))
    crf_window: int = 0  # fixed-point sum of per-step aggregated CRF
    last_evicted: np.ndarray = field(default_factory=lambda: np.zeros(0, dtype=np.int64))

    @property
    def n(self):
        return int(self.pos.shape[0])


@dataclass
class StepRecord:
    """What one unit did in one decode step (for parity checks)."""
    y: np.ndarray              # [G, d] float64 attention output
    abar: np.ndarray           # [n] float64 mean attention weight
    decision: HitDecision
    tmp: np.ndarray            # [n] float32 CRF_temp
    crf_sum: int               # fixed-point aggregated CRF
    evicted_pos: np.ndarray    # positions evicted in this step (sorted)
    evict_gap: float           # relative gap between the last kept and first evicted score
    # the unit as it stood after the append and before Alg. 1 ran (record keeping for parity checks that
    # replay Steps 2-4 under another admissible hit decision; no arithmetic)
    t: int = 0
    budget: int = 0
    pre_pos: np.ndarray = None
    pre_crf: np.ndarray = None
    pre_tau: np.ndarray = None


class CrystalKVOracle:
    """Caches of all (layer, sequence, KV head) units and the per-step flow.

    Geometry: n_layers, batch, n_q_heads, n_kv_heads, head_dim.  `budgets` is
    an int array [L][Bz][Hkv].  Time t starts at `t0` (the prompt length) and
    advances by one per decode step; the token decoded at step t has position t.
    """

    def __init__(self, n_layers, batch, n_q_heads, n_kv_heads, head_dim, budgets, *,
                 lam=0.5, top_p=0.9, softmax_scale=None, reward_mode=REWARD_TOPP_HIT,
                 t0=0, budget_min=1, budget_max=1 << 30):
        assert n_q_heads % n_kv_heads == 0
        self.L, self.Bz, self.Hq, self.Hkv, self.d = n_layers, batch, n_q_heads, n_kv_heads, head_dim
        self.G = n_q_heads // n_kv_heads
        self.lam = float(np.float32(lam))
        self.top_p = float(np.float32(top_p))
        if softmax_scale is None:
            softmax_scale = 1.0 / math.sqrt(head_dim)
        self.scale = float(np.float32(softmax_scale))
        self.reward_mode = reward_mode
        self.t = int(t0)
        self.budget_min, self.budget_max = int(budget_min), int(budget_max)
        self.tab = decay_table(self.lam)
        budgets = np.asarray(budgets, dtype=np.int64).reshape(n_layers, batch, n_kv_heads)
        self.budget_total = budgets.sum(axis=(0, 2))          # per sequence, conserved
        self.window_steps = 0
        self.units = {}
        for l in range(n_layers):
            for b in range(batch):
                for h in range(n_kv_heads):
                    self.units[(l, b, h)] = Unit(
                        K=np.zeros((0, head_dim)), V=np.zeros((0, head_dim)),
                        pos=np.zeros(0, dtype=np.int64), crf=np.zeros(0, dtype=np.float32),
                        tau=np.zeros(0, dtype=np.int64), budget=int(budgets[l, b, h]))

    # -- state in ------------------------------------------------------------
    def load_prompt(self, layer, K, V, crf0=None, tau0=None):
        """K, V: [Bz][Hkv][P][d].  Prompt entries get positions 0..P-1 and,
        unless given, CRF = 1 and tau = P - 1 (referenced once, at the end of
        the prompt)."""
        P = K.shape[2]
        for b in range(self.Bz):
            for h in range(self.Hkv):
                u = self.units[(layer, b, h)]
                u.K = np.asarray(K[b, h], dtype=np.float64).copy()
                u.V = np.asarray(V[b, h], dtype=np.float64).copy()
                u.pos = np.arange(P, dtype=np.int64)
                u.crf = (np.ones(P, np.float32) if crf0 is None
                         else np.asarray(crf0[b, h], np.float32).copy())
                u.tau = (np.full(P, P - 1, np.int64) if tau0 is None
                         else np.asarray(tau0[b, h], np.int64).copy())
                u.hit = np.zeros(P, dtype=bool)

    def seed_prompt(self, layer, q_obs):
        """Scores of a freshly loaded prompt from its last W queries (reading
        in the header).  q_obs: [W][Bz][Hq][d], the queries of positions
        P-W .. P-1 in order.  Replaces the CRF and tau the prompt was loaded
        with.  Returns {unit key: [HitDecision of position P-W, ..., P-1]}."""
        q_obs = np.asarray(q_obs, dtype=np.float64)
        W = q_obs.shape[0]
        decisions = {}
        for b in range(self.Bz):
            for h in range(self.Hkv):
                u = self.units[(layer, b, h)]
                P = u.n
                assert 1 <= W <= P and np.array_equal(u.pos, np.arange(P)), "needs a freshly loaded prompt"
                u.crf = np.where(u.pos < P - W, np.float32(1.0), np.float32(0.0)).astype(np.float32)
                u.tau = u.pos.astype(np.int64).copy()
                decs = []
                for j in range(W):
                    t = P - W + j                       # time of this query = its position
                    nv = t + 1                          # entries of positions 0 .. t are visible
                    q = q_obs[j, b, h * self.G:(h + 1) * self.G]
                    _, a = attention(q, u.K[:nv], u.V[:nv], self.scale)
                    abar = a.sum(axis=0) / float(self.G)
                    if self.reward_mode == REWARD_TOPP_HIT:
                        dec = hit_mask(abar, u.pos[:nv], self.top_p, new_index=nv - 1)
                        reward, store = dec.hit.astype(np.float32), dec.hit
                    else:
                        dec = HitDecision(np.ones(nv, bool), nv, np.arange(nv), math.inf, math.inf)
                        reward, store = abar.astype(np.float32), np.ones(nv, dtype=bool)
                    _, u.crf[:nv], u.tau[:nv] = crf_update(u.crf[:nv], u.tau[:nv], t, reward, store, self.tab)
                    decs.append(dec)
                u.hit = np.zeros(P, dtype=bool)
                u.hit[:len(decs[-1].hit)] = decs[-1].hit
                decisions[(layer, b, h)] = decs
        return decisions

    def set_unit(self, key, K, V, pos, crf, tau):
        u = self.units[key]
        u.K = np.asarray(K, np.float64).copy()
        u.V = np.asarray(V, np.float64).copy()
        u.pos = np.asarray(pos, np.int64).copy()
        u.crf = np.asarray(crf, np.float32).copy()
        u.tau = np.asarray(tau, np.int64).copy()
        u.hit = np.zeros(u.n, dtype=bool)

    # -- one decode step -------------------------------------------------------
    def step_unit(self, key, q, k_new, v_new, evict=True):
        """Sec. 2.2 append + attend, then Alg. 1 Steps 1-3 and, if `evict` and
        the cache exceeds its budget, Step 4.  q: [G, d], k_new, v_new: [d]."""
        u = self.units[key]
        t = self.t
        # append before attending
        u.K = np.vstack([u.K, np.asarray(k_new, np.float64)[None, :]])
        u.V = np.vstack([u.V, np.asarray(v_new, np.float64)[None, :]])
        u.pos = np.append(u.pos, np.int64(t))
        u.crf = np.append(u.crf, np.float32(0.0))
        u.tau = np.append(u.tau, np.int64(t))
        n = u.n
        pre = (u.pos.copy(), u.crf.copy(), u.tau.copy())
        y, a = attention(q, u.K, u.V, self.scale)
        abar = a.sum(axis=0) / float(self.G)
        if self.reward_mode == REWARD_TOPP_HIT:
            dec = hit_mask(abar, u.pos, self.top_p, new_index=n - 1)
            reward = dec.hit.astype(np.float32)
            store = dec.hit
        else:
            dec = HitDecision(np.ones(n, bool), n, np.arange(n), math.inf, math.inf)
            reward = abar.astype(np.float32)
            store = np.ones(n, dtype=bool)
        tmp, u.crf, u.tau = crf_update(u.crf, u.tau, t, reward, store, self.tab)
        u.hit = dec.hit.copy()
        s_fixed = crf_sum_fixed(tmp)
        u.crf_window += s_fixed
        evicted_pos, gap = np.zeros(0, np.int64), math.inf
        if evict:
            evicted_pos, gap = self._evict_unit(u, tmp)
        return StepRecord(y, abar, dec, tmp, s_fixed, evicted_pos, gap, t, u.budget, *pre)

    def _evict_unit(self, u, tmp, n_sink=None):
        if u.n <= u.budget:
            u.last_evicted = np.zeros(0, np.int64)
            return u.last_evicted, math.inf
        if n_sink is None:
            retain, evicted = evict_select(tmp, u.pos, u.budget)
        else:
            retain, evicted = window_select(u.pos, u.budget, n_sink)
        kept_min = float(tmp[retain].min())
        ev_max = float(tmp[evicted].max())
        gap = (kept_min - ev_max) / kept_min if kept_min > 0 else 0.0
        evicted_pos = np.sort(u.pos[evicted])
        u.K, u.V = u.K[retain], u.V[retain]
        u.pos, u.crf, u.tau, u.hit = u.pos[retain], u.crf[retain], u.tau[retain], u.hit[retain]
        u.last_evicted = evicted_pos
        return evicted_pos, gap

    def decode_step(self, q, k_new, v_new, evict=True):
        """q: [L][Bz][Hq][d]; k_new, v_new: [L][Bz][Hkv][d].  Returns
        (out [L][Bz][Hq][d] float64, {unit key: StepRecord}).  Advances t."""
        out = np.zeros((self.L, self.Bz, self.Hq, self.d))
        recs = {}
        for (l, b, h) in self.units:
            g0 = h * self.G
            r = self.step_unit((l, b, h), q[l, b, g0:g0 + self.G], k_new[l, b, h], v_new[l, b, h], evict)
            out[l, b, g0:g0 + self.G] = r.y
            recs[(l, b, h)] = r
        self.t += 1
        self.window_steps += 1
        return out, recs

    # -- Alg. 1 Step 4 on its own ---------------------------------------------
    def current_tmp(self, u):
        """CRF_temp of every entry at the time of the last completed step."""
        n = u.n
        tmp, _, _ = crf_update(u.crf, u.tau, self.t - 1, np.zeros(n, np.float32),
                               np.zeros(n, bool), self.tab)
        return tmp

    def evict(self, keys=None):
        res = {}
        for key in (self.units if keys is None else keys):
            u = self.units[key]
            res[key] = self._evict_unit(u, self.current_tmp(u))[0]
        return res

    def evict_window(self, n_sink, keys=None):
        """The sink-plus-recent-window baseline's eviction (`window_select`) on the same caches:
        scores play no part and stay as they are on the survivors."""
        res = {}
        for key in (self.units if keys is None else keys):
            u = self.units[key]
            res[key] = self._evict_unit(u, self.current_tmp(u), n_sink)[0]
        return res

    # -- Alg. 2 ----------------------------------------------------------------
    def rebudget(self):
        """New integer budgets per sequence from the window-averaged aggregated
        CRF; resets the window.  Eviction to the new budgets is a separate call."""
        if self.window_steps == 0:
            return self.budgets()
        for b in range(self.Bz):
            C = np.zeros((self.L, self.Hkv))
            B = np.zeros((self.L, self.Hkv), dtype=np.int64)
            for l in range(self.L):
                for h in range(self.Hkv):
                    u = self.units[(l, b, h)]
                    C[l, h] = float(u.crf_window) / (float(FIXED_POINT_ONE) * float(self.window_steps))
                    B[l, h] = u.budget
            newB = rebudget(C, B, int(self.budget_total[b]), self.budget_min, self.budget_max)
            for l in range(self.L):
                for h in range(self.Hkv):
                    self.units[(l, b, h)].budget = int(newB[l, h])
        for u in self.units.values():
            u.crf_window = 0
        self.window_steps = 0
        return self.budgets()

    def budgets(self):
        out = np.zeros((self.L, self.Bz, self.Hkv), dtype=np.int64)
        for (l, b, h), u in self.units.items():
            out[l, b, h] = u.budget
        return out

    def lengths(self):
        out = np.zeros((self.L, self.Bz, self.Hkv), dtype=np.int64)
        for (l, b, h), u in self.units.items():
            out[l, b, h] = u.n
        return out

    # -- Sec. 3 probe ----------------------------------------------------------
    def probe(self, key, q_probe):
        """Classes of the unit's current entries under an answer-probe query
        (q_probe: [G, d]); no state changes."""
        u = self.units[key]
        _, a = attention(q_probe, u.K, u.V, self.scale)
        abar = a.sum(axis=0) / float(self.G)
        return probe_classes(abar, u.pos), abar
