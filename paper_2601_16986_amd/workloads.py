"""Seeded synthetic inputs shaped like the paper's reasoning workloads.

This module only draws numbers: it holds none of the method's arithmetic
(no attention, no scores, no eviction) and is the one module that both the
tests of the CPU oracle and the HIP path's callers use, so that both sides
see the same inputs.  The paper evaluates on CodeForces and MATH-500 with
R1-distilled models (Sec. 6.1); neither is available here, so caches take the
models' geometry and the 8K/16K-level lengths of Table 1 and replace content
by seeded distributions:

* per KV head a mean-query vector m (norm 4, random direction);
* queries q = eps + m + r_t, eps ~ N(0, I);
* ordinary keys k = eps + r_t, values v = eps;
* heavy keys (1 % of positions, or 4 fixed positions in the tiny workload)
  carry + 3 m, so their logit stands out;
* r_t is a per-KV-head AR(1) drift (rho = 0.99, stationary variance 0.35 per
  component) shared by q_t and k_t, which gives recent keys a logit bonus of
  about 4 rho^(t - i);
* everything is rounded to bf16 (round to nearest even) and handed out as
  float32 arrays holding bf16 values exactly.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

RHO = 0.99
DRIFT_VAR = 0.35
M_NORM = 4.0
HEAVY_GAIN = 3.0
HEAVY_FRACTION = 0.01


@dataclass(frozen=True)
class Config:
    name: str
    n_layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    prompt: int
    decode_steps: int
    budget: int            # mean budget per KV head
    budget_min: int
    budget_max: int
    adaptive: bool         # budgets drawn per head (Beta(2,5) proportions)
    rebudget_interval: int
    lam: float = 0.5
    top_p: float = 0.9
    seed: int = 0

    @property
    def group(self):
        return self.n_q_heads // self.n_kv_heads

    @property
    def n_units(self):
        return self.n_layers * self.batch * self.n_kv_heads


# The five workloads.  Geometry: DeepSeek-R1-distilled Qwen2-7B / Qwen2-14B /
# Llama-3-8B / Qwen2-32B (Sec. 6.1), lengths at the 8K / 16K level (Table 1).
CONFIGS = {
    "tiny": Config("tiny", 1, 1, 8, 2, 128, 64, 512, 128, 128, 128, False, 0, seed=1000),
    "qwen7b": Config("qwen7b", 28, 8, 28, 4, 128, 256, 8192, 2048, 2048, 2048, False, 0, seed=2000),
    "qwen14b": Config("qwen14b", 48, 16, 40, 8, 128, 512, 16384, 2048, 256, 8192, True, 256, seed=3000),
    "llama8b": Config("llama8b", 32, 64, 32, 8, 128, 1024, 32768, 1024, 1024, 1024, False, 0, seed=4000),
    "qwen32b": Config("qwen32b", 64, 32, 40, 8, 128, 512, 32768, 4096, 512, 16384, True, 256, seed=5000),
}


def scaled(cfg: Config, **kw) -> Config:
    """A smaller copy of a workload (fewer layers / sequences / entries) for tests."""
    return replace(cfg, **kw)


# ---------------------------------------------------------------- bf16 helpers
def bf16_round(x):
    """float32 array rounded to the bf16 grid (round to nearest even), as float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


def bf16_bits(x):
    """uint16 bit patterns of a float32 array that already lies on the bf16 grid."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> 16).astype(np.uint16).reshape(x.shape)


def _rng(seed, *stream):
    return np.random.Generator(np.random.Philox(key=int(seed), counter=[int(s) for s in stream] + [0] * (4 - len(stream))))


def mean_query(cfg: Config):
    """m[L][Bz][Hkv][d]: the mean query direction of every KV head, norm 4."""
    g = _rng(cfg.seed, 1)
    m = g.standard_normal((cfg.n_layers, cfg.batch, cfg.n_kv_heads, cfg.head_dim)).astype(np.float32)
    m *= M_NORM / np.linalg.norm(m, axis=-1, keepdims=True)
    return m


def draw_budgets(cfg: Config):
    """Initial budgets [L][Bz][Hkv].  Fixed workloads: all equal.  Adaptive
    ones: per-head proportion ~ Beta(2, 5), scaled to the mean budget, clipped
    to [budget_min, budget_max], then nudged so every sequence's total is
    exactly L * Hkv * mean."""
    shape = (cfg.n_layers, cfg.batch, cfg.n_kv_heads)
    if not cfg.adaptive:
        return np.full(shape, cfg.budget, dtype=np.int32)
    g = _rng(cfg.seed, 2)
    pi = g.beta(2.0, 5.0, size=shape)
    out = np.zeros(shape, dtype=np.int64)
    per_seq = cfg.n_layers * cfg.n_kv_heads * cfg.budget
    for b in range(cfg.batch):
        w = pi[:, b, :]
        v = np.clip(np.rint(per_seq * w / w.sum()), cfg.budget_min, cfg.budget_max).astype(np.int64)
        diff = per_seq - int(v.sum())
        flat = v.reshape(-1)
        i = 0
        while diff != 0:                      # spread the rounding/clipping residue
            k = i % flat.size
            if diff > 0 and flat[k] < cfg.budget_max:
                flat[k] += 1
                diff -= 1
            elif diff < 0 and flat[k] > cfg.budget_min:
                flat[k] -= 1
                diff += 1
            i += 1
        out[:, b, :] = flat.reshape(w.shape)
    return out.astype(np.int32)


# ------------------------------------------------------------- full sequences
@dataclass
class Stream:
    """A whole prompt + decode sequence for every unit of a (small) workload."""
    cfg: Config
    prompt_k: np.ndarray    # [L][Bz][Hkv][P][d]
    prompt_v: np.ndarray
    q: np.ndarray           # [T][L][Bz][Hq][d]
    k_new: np.ndarray       # [T][L][Bz][Hkv][d]
    v_new: np.ndarray
    heavy: np.ndarray       # [L][Bz][Hkv][P+T] bool
    probe_q: np.ndarray     # [L][Bz][Hq][d]


def make_stream(cfg: Config, n_steps=None, *, tiny_heavy=None, drift=True) -> Stream:
    """Prompt and `n_steps` decode steps for all units, host side.  Meant for
    workloads small enough to hold whole (the tiny one, scaled-down copies).

    tiny_heavy: if true, 4 heavy positions per KV head (2 in the prompt, 2 in
    the first half of decode) with key exactly 3 m and no drift anywhere;
    default: true for the workload named "tiny".
    """
    T = cfg.decode_steps if n_steps is None else int(n_steps)
    if tiny_heavy is None:
        tiny_heavy = cfg.name == "tiny"
    L, Bz, Hq, Hkv, d, P, G = (cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads,
                                cfg.head_dim, cfg.prompt, cfg.group)
    g = _rng(cfg.seed, 3)
    m = mean_query(cfg)
    N = P + T
    k_all = g.standard_normal((L, Bz, Hkv, N, d)).astype(np.float32)
    v_all = g.standard_normal((L, Bz, Hkv, N, d)).astype(np.float32)
    q_eps = g.standard_normal((T, L, Bz, Hq, d)).astype(np.float32)
    heavy = np.zeros((L, Bz, Hkv, N), dtype=bool)
    if tiny_heavy:
        for l in range(L):
            for b in range(Bz):
                for h in range(Hkv):
                    hp = np.concatenate([g.choice(P, 2, replace=False) if P >= 2 else np.zeros(0, dtype=np.int64),
                                         P + g.choice(max(T // 2, 2), 2, replace=False)])
                    heavy[l, b, h, hp] = True
                    k_all[l, b, h, hp] = HEAVY_GAIN * m[l, b, h]
        r = np.zeros((L, Bz, Hkv, N, d), dtype=np.float32)
    else:
        heavy = g.random((L, Bz, Hkv, N)) < HEAVY_FRACTION
        k_all += HEAVY_GAIN * heavy[..., None] * m[:, :, :, None, :]
        r = np.zeros((L, Bz, Hkv, N, d), dtype=np.float32)
        if drift:
            xi = g.standard_normal((L, Bz, Hkv, N, d)).astype(np.float32)
            sig = np.float32(np.sqrt(DRIFT_VAR))
            r[..., 0, :] = sig * xi[..., 0, :]
            c = np.float32(np.sqrt(1.0 - RHO * RHO)) * sig
            for i in range(1, N):
                r[..., i, :] = np.float32(RHO) * r[..., i - 1, :] + c * xi[..., i, :]
            k_all += r
    # queries of decode step s sit at position P + s
    mq = np.repeat(m, G, axis=2)                                   # [L][Bz][Hq][d]
    rq = np.repeat(r[..., P:, :], G, axis=2)                       # [L][Bz][Hq][T][d]
    q = q_eps + mq[None] + np.moveaxis(rq, 3, 0)
    probe = g.standard_normal((L, Bz, Hq, d)).astype(np.float32)
    k_all, v_all, q, probe = bf16_round(k_all), bf16_round(v_all), bf16_round(q), bf16_round(probe)
    return Stream(cfg, k_all[..., :P, :].copy(), v_all[..., :P, :].copy(), q,
                  np.ascontiguousarray(np.moveaxis(k_all[..., P:, :], 3, 0)),
                  np.ascontiguousarray(np.moveaxis(v_all[..., P:, :], 3, 0)), heavy, probe)


# ------------------------------------------------- steady-state caches (host)
@dataclass
class UnitCache:
    K: np.ndarray      # [n][d] float32 on the bf16 grid
    V: np.ndarray
    pos: np.ndarray    # [n] int32, ascending
    crf: np.ndarray    # [n] float32
    tau: np.ndarray    # [n] int32


def steady_unit(cfg: Config, unit_index: int, n: int, t_now: int, m_vec) -> UnitCache:
    """One unit's cache as it might look mid-way through the think stage at
    time `t_now` (the next decode step): n entries, the most recent n/4
    positions plus older positions drawn uniformly; 1 % heavy keys; drift
    sampled exactly from the AR(1) law at the retained positions; scores and
    last-hit times plausible for lambda = cfg.lam (they relax to the true
    steady state during warm-up steps)."""
    g = _rng(cfg.seed, 4, unit_index)
    d = cfg.head_dim
    n_recent = min(n, max(1, n // 4))
    older = np.sort(g.choice(max(t_now - n_recent, n - n_recent), n - n_recent, replace=False))
    pos = np.concatenate([older, np.arange(t_now - n_recent, t_now)]).astype(np.int32)
    heavy = g.random(n) < HEAVY_FRACTION
    K = g.standard_normal((n, d)).astype(np.float32)
    V = g.standard_normal((n, d)).astype(np.float32)
    K += HEAVY_GAIN * heavy[:, None] * np.asarray(m_vec, np.float32)[None, :]
    r = drift_at(g, pos, d)
    K += r
    age = (t_now - 1 - pos).astype(np.int64)
    since_hit = np.minimum(age, g.geometric(0.2, size=n) - 1)
    tau = (t_now - 1 - since_hit).astype(np.int32)
    crf = (1.0 + g.random(n)).astype(np.float32)
    return UnitCache(bf16_round(K), bf16_round(V), pos, crf, tau)


def drift_at(g, pos, d):
    """AR(1) drift sampled at the (ascending) positions `pos`: exact for the
    stationary Gaussian process, r' = rho^gap r + sqrt(1 - rho^(2 gap)) sigma xi."""
    n = len(pos)
    sig = np.sqrt(DRIFT_VAR)
    xi = g.standard_normal((n, d))
    r = np.zeros((n, d))
    r[0] = sig * xi[0]
    for i in range(1, n):
        a = RHO ** float(pos[i] - pos[i - 1])
        r[i] = a * r[i - 1] + np.sqrt(1.0 - a * a) * sig * xi[i]
    return r.astype(np.float32)


def decode_inputs(cfg: Config, step: int, m, r_last=None):
    """q [L][Bz][Hq][d], k_new, v_new [L][Bz][Hkv][d] for decode step `step`
    (counted from 0), plus the drift state to pass to the next call."""
    g = _rng(cfg.seed, 5, step)
    L, Bz, Hq, Hkv, d, G = cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.group
    sig = np.float32(np.sqrt(DRIFT_VAR))
    xi = g.standard_normal((L, Bz, Hkv, d)).astype(np.float32)
    if r_last is None:
        r = sig * xi
    else:
        r = np.float32(RHO) * r_last + np.float32(np.sqrt(1 - RHO * RHO)) * sig * xi
    heavy = g.random((L, Bz, Hkv)) < HEAVY_FRACTION
    k = g.standard_normal((L, Bz, Hkv, d)).astype(np.float32) + HEAVY_GAIN * heavy[..., None] * m + r
    v = g.standard_normal((L, Bz, Hkv, d)).astype(np.float32)
    q = (g.standard_normal((L, Bz, Hq, d)).astype(np.float32)
         + np.repeat(m, G, axis=2) + np.repeat(r, G, axis=2))
    return bf16_round(q), bf16_round(k), bf16_round(v), r


# ------------------------------------------- steady-state caches (device, bulk)
def torch_generator(cfg: Config, stream: int, device):
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(int(cfg.seed) * 1000003 + int(stream))
    return g


def torch_mean_query(cfg: Config, device):
    """m[L][Bz][Hkv][d], norm 4, drawn on the device (bulk workloads)."""
    import torch
    g = torch_generator(cfg, 1, device)
    m = torch.randn((cfg.n_layers, cfg.batch, cfg.n_kv_heads, cfg.head_dim), generator=g, device=device)
    return m * (M_NORM / m.norm(dim=-1, keepdim=True))


def torch_steady_layer(cfg: Config, layer: int, lengths, t_now: int, m_layer, r_now, device):
    """Caches of one layer mid-way through the think stage, built on the device.

    lengths: int array [Bz][Hkv] (entries per unit).  Same recipe as
    `steady_unit` (most recent quarter contiguous, older positions spread over
    the past, 1 % heavy keys, plausible scores), except that the drift of an
    entry is tied only to the current drift state r_now [Bz][Hkv][d]
    (r_pos = rho^age r_now + sqrt(1 - rho^(2 age)) sigma xi): that gives every
    entry the right logit bonus against the coming queries without a
    sequential pass over 10^4 entries.
    Returns bf16 k, v [Bz][Hkv][P][d], int32 lengths, f32 crf, int32 tau, pos.
    """
    import torch
    g = torch_generator(cfg, 100 + layer, device)
    Bz, Hkv, d = cfg.batch, cfg.n_kv_heads, cfg.head_dim
    n = torch.as_tensor(np.asarray(lengths, dtype=np.int64), device=device).reshape(Bz, Hkv, 1)
    P = int(n.max().item())
    i = torch.arange(P, device=device).reshape(1, 1, P)
    n_recent = torch.clamp(n // 4, min=1)
    n_old = n - n_recent
    t_old = t_now - n_recent                                   # older positions live in [0, t_old)
    stride = t_old.double() / torch.clamp(n_old, min=1).double()
    jitter = torch.rand((Bz, Hkv, P), generator=g, device=device, dtype=torch.float64)
    lo = torch.floor(i.double() * stride).long()
    hi = torch.floor((i + 1).double() * stride).long()          # cell [lo, hi) of entry i: cells are disjoint
    pos_old = lo + torch.floor(jitter * (hi - lo).double()).long()
    pos_old = torch.minimum(pos_old, torch.clamp(hi - 1, min=0))
    pos = torch.where(i < n_old, pos_old, t_old + (i - n_old))
    pos = torch.where(i < n, pos, torch.zeros_like(pos))
    age = (t_now - 1 - pos).clamp(min=0)
    k = torch.randn((Bz, Hkv, P, d), generator=g, device=device)
    v = torch.randn((Bz, Hkv, P, d), generator=g, device=device)
    heavy = torch.rand((Bz, Hkv, P), generator=g, device=device) < HEAVY_FRACTION
    k += HEAVY_GAIN * heavy.unsqueeze(-1) * m_layer.unsqueeze(2)
    a = torch.pow(torch.tensor(RHO, device=device, dtype=torch.float64), (age + 1).double()).float().unsqueeze(-1)
    xi = torch.randn((Bz, Hkv, P, d), generator=g, device=device)
    k += a * r_now.unsqueeze(2) + torch.sqrt(1 - a * a) * float(np.sqrt(DRIFT_VAR)) * xi
    since = torch.minimum(age, torch.floor(-torch.log(torch.rand((Bz, Hkv, P), generator=g, device=device)
                                                      .clamp(min=1e-9)) * 5.0).long())
    tau = (t_now - 1 - since).int()
    crf = 1.0 + torch.rand((Bz, Hkv, P), generator=g, device=device)
    return (k.to(torch.bfloat16).contiguous(), v.to(torch.bfloat16).contiguous(),
            n.reshape(Bz, Hkv).int().contiguous(), crf.contiguous(), tau.contiguous(), pos.int().contiguous())


def torch_step_ring(cfg: Config, n_slots: int, m, r_now, device, epoch: int = 0, return_state: bool = False):
    """Inputs of `n_slots` consecutive decode steps for all layers, on the
    device: q [S][L][Bz][Hq][d], k_new, v_new [S][L][Bz][Hkv][d] (bf16).  The
    drift continues from r_now [L][Bz][Hkv][d].  `epoch` selects an independent
    batch of steps (a benchmark that runs more steps than it holds inputs for draws
    fresh ones instead of replaying old ones: replayed keys are exact duplicates of
    cached ones and tie with them); return_state also returns the final drift state."""
    import torch
    g = torch_generator(cfg, 7 + 1000 * int(epoch), device)
    L, Bz, Hq, Hkv, d, G = cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.group
    sig = float(np.sqrt(DRIFT_VAR))
    qs, ks, vs = [], [], []
    r = r_now
    for _ in range(n_slots):
        r = RHO * r + float(np.sqrt(1 - RHO * RHO)) * sig * torch.randn((L, Bz, Hkv, d), generator=g, device=device)
        heavy = torch.rand((L, Bz, Hkv), generator=g, device=device) < HEAVY_FRACTION
        k = torch.randn((L, Bz, Hkv, d), generator=g, device=device) + HEAVY_GAIN * heavy.unsqueeze(-1) * m + r
        v = torch.randn((L, Bz, Hkv, d), generator=g, device=device)
        q = (torch.randn((L, Bz, Hq, d), generator=g, device=device)
             + m.repeat_interleave(G, dim=2) + r.repeat_interleave(G, dim=2))
        qs.append(q.to(torch.bfloat16))
        ks.append(k.to(torch.bfloat16))
        vs.append(v.to(torch.bfloat16))
    ring = (torch.stack(qs).contiguous(), torch.stack(ks).contiguous(), torch.stack(vs).contiguous())
    return (ring, r) if return_state else ring
