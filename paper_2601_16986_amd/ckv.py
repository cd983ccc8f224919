"""Thin ctypes binding of libckv.so (the C ABI in include/ckv.h).

Argument marshalling only: every step of the decode path runs in the HIP
kernels of the library.  PyTorch supplies device memory and streams.  There is
no fallback: if the shared library is missing, `load()` raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libckv.so")

OK, EINVAL, ECAPACITY, ESTATE, EHIP, EWORKSPACE = 0, -1, -2, -3, -4, -5
BF16, F32 = 1, 2
REWARD_TOPP_HIT, REWARD_ATTN_WEIGHTED = 0, 1
FLAG_HIT, FLAG_SLIP = 1, 2
FUSE_EVICT = 1
ATTENTION_ONLY = 2
DEFER_BOOKKEEPING = 4

EXPORTS = [
    "ckv_workspace_bytes", "ckv_init", "ckv_destroy", "ckv_load_prompt", "ckv_seed_prompt", "ckv_load_cache", "ckv_decode_step",
    "ckv_evict",
    "ckv_evict_window",
    "ckv_rebudget", "ckv_rebalance", "ckv_pool_slots", "ckv_probe", "ckv_probe_noalloc", "ckv_get_budgets", "ckv_get_lengths", "ckv_get_segments", "ckv_set_budgets", "ckv_get_time",
    "ckv_set_time", "ckv_status", "ckv_export_unit", "ckv_import_unit", "ckv_profile_enable",
    "ckv_profile_read", "ckv_set_path", "ckv_path_info", "ckv_join", "ckv_bandwidth_probe", "ckv_strerror", "ckv_last_error",
]


class Layout(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("batch", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("cap", C.c_int32),
                ("out_dtype", C.c_int32), ("headroom", C.c_int32), ("pool_slots", C.c_int64)]


class LrfuParams(C.Structure):
    _fields_ = [("lambda_", C.c_float), ("top_p", C.c_float), ("softmax_scale", C.c_float),
                ("reward_mode", C.c_int32), ("t0", C.c_int32), ("budget_min", C.c_int32),
                ("budget_max", C.c_int32)]


class Buffers(C.Structure):
    _fields_ = [("k_pool", C.c_void_p), ("v_pool", C.c_void_p), ("crf", C.c_void_p), ("tau", C.c_void_p),
                ("pos", C.c_void_p), ("flags", C.c_void_p), ("workspace", C.c_void_p),
                ("workspace_bytes", C.c_size_t)]


_lib = None


def load():
    """The loaded library; raises if it has not been built (no CPU fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2601_16986_amd.build` "
                           "(there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, u32 = C.c_void_p, C.c_int32, C.c_uint32
    lib.ckv_workspace_bytes.restype = C.c_size_t
    lib.ckv_workspace_bytes.argtypes = [C.POINTER(Layout), C.POINTER(LrfuParams)]
    lib.ckv_init.argtypes = [C.POINTER(vp), C.POINTER(Layout), vp, C.POINTER(LrfuParams), C.POINTER(Buffers), vp]
    lib.ckv_destroy.restype = None
    lib.ckv_destroy.argtypes = [vp]
    lib.ckv_load_prompt.argtypes = [vp, i32, vp, vp, i32, vp, vp, vp]
    lib.ckv_load_cache.argtypes = [vp, i32, vp, vp, i32, vp, vp, vp, vp, vp]
    lib.ckv_seed_prompt.argtypes = [vp, i32, vp, i32, vp]
    lib.ckv_decode_step.argtypes = [vp, i32, vp, vp, vp, vp, u32, vp]
    lib.ckv_evict.argtypes = [vp, i32, vp]
    lib.ckv_evict_window.argtypes = [vp, i32, i32, vp]
    lib.ckv_rebudget.argtypes = [vp, vp]
    lib.ckv_rebalance.argtypes = [vp, vp]
    lib.ckv_pool_slots.restype = C.c_int64
    lib.ckv_pool_slots.argtypes = [C.POINTER(Layout), vp, i32]
    lib.ckv_probe.argtypes = [vp, i32, vp, vp, vp]
    lib.ckv_probe_noalloc.argtypes = [vp, i32, vp, vp, vp]
    lib.ckv_get_budgets.argtypes = [vp, vp]
    lib.ckv_get_lengths.argtypes = [vp, vp]
    lib.ckv_get_segments.argtypes = [vp, vp, vp, vp, C.POINTER(i32)]
    lib.ckv_set_budgets.argtypes = [vp, vp]
    lib.ckv_get_time.argtypes = [vp, C.POINTER(i32)]
    lib.ckv_set_time.argtypes = [vp, i32]
    lib.ckv_status.argtypes = [vp]
    lib.ckv_export_unit.argtypes = [vp, i32, i32, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32),
                                    vp, vp, vp, vp, vp, vp]
    lib.ckv_import_unit.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, i32]
    lib.ckv_profile_enable.argtypes = [vp, i32]
    lib.ckv_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i32)]
    lib.ckv_set_path.argtypes = [vp, i32]
    lib.ckv_path_info.argtypes = [vp, C.POINTER(i32), C.POINTER(i32)]
    lib.ckv_join.argtypes = [vp, vp]
    lib.ckv_bandwidth_probe.argtypes = [vp, vp, C.c_size_t, vp, vp]
    lib.ckv_strerror.restype = C.c_char_p
    lib.ckv_strerror.argtypes = [C.c_int]
    lib.ckv_last_error.restype = C.c_char_p
    lib.ckv_last_error.argtypes = [vp]
    for name in EXPORTS:
        getattr(lib, name)
    _lib = lib
    return lib


class CkvError(RuntimeError):
    def __init__(self, code, detail=""):
        self.code = code
        msg = load().ckv_strerror(code).decode()
        super().__init__(f"ckv error {code} ({msg}){': ' + detail if detail else ''}")


def _np_ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def _buffer_sizes(pool_slots, head_dim, ws):
    """Bytes of the seven caller-owned device buffers: K pool, V pool, crf, tau, pos, flags, workspace."""
    S = int(pool_slots)
    return [S * head_dim * 2, S * head_dim * 2, S * 4, S * 4, S * 4, S, int(ws) + 256]


def arena_bytes(n_layers, batch, n_q_heads, n_kv_heads, head_dim, cap, budgets, *, lam=0.5, top_p=0.9, softmax_scale=None,
                reward_mode=REWARD_TOPP_HIT, t0=0, budget_min=1, budget_max=None, out_dtype=F32, headroom=0, pool_slots=None,
                prompt_len=0, **_):
    """Bytes an `arena=` for a CrystalKV of these arguments must hold (each buffer rounded up to 2 MiB, one
    2 MiB for the arena's own alignment)."""
    lib = load()
    b32 = np.ascontiguousarray(np.asarray(budgets, dtype=np.int32).reshape(n_layers, batch, n_kv_heads))
    if pool_slots is None:
        probe = Layout(n_layers, batch, n_q_heads, n_kv_heads, head_dim, cap, out_dtype, headroom, 0)
        pool_slots = lib.ckv_pool_slots(C.byref(probe), _np_ptr(b32), int(prompt_len))
    lay = Layout(n_layers, batch, n_q_heads, n_kv_heads, head_dim, cap, out_dtype, headroom, int(pool_slots))
    par = LrfuParams(lam, top_p, softmax_scale if softmax_scale is not None else 1.0 / float(np.sqrt(head_dim)), reward_mode, t0,
                     budget_min, budget_max if budget_max is not None else cap - 1)
    ws = lib.ckv_workspace_bytes(C.byref(lay), C.byref(par))
    if pool_slots <= 0 or ws == 0:
        raise CkvError(EINVAL, "layout or parameters rejected")
    al = 2 << 20
    return sum((b_ + al - 1) // al * al for b_ in _buffer_sizes(pool_slots, head_dim, ws)) + al


class CrystalKV:
    """One ckv context plus the torch tensors that back it.

    budgets: int array [L][Bz][Hkv].  All device tensors live on `device`.
    """

    def __init__(self, n_layers, batch, n_q_heads, n_kv_heads, head_dim, cap, budgets, *, lam=0.5, top_p=0.9,
                 softmax_scale=None, reward_mode=REWARD_TOPP_HIT, t0=0, budget_min=1, budget_max=None,
                 out_dtype=F32, device="cuda:0", headroom=0, pool_slots=None, prompt_len=0, pools=None, arena=None):
        """headroom = 0: every unit owns room for `cap` entries (pools of units * ceil(cap / 256) * 256 slots).
        headroom >= 1: shared pools, a unit owns what budget + headroom entries need; pool_slots (a multiple of
        256) then sizes the pools, by default what ckv_pool_slots says for these budgets and a prompt of
        prompt_len tokens passing through one layer at a time.
        arena: a uint8 device tensor that all seven device buffers are carved from (at 2 MiB boundaries; see
        arena_bytes) instead of seven allocations; pools: caller-owned K and V pools alone."""
        import torch
        self.torch = torch
        self.lib = load()
        self.device = torch.device(device)
        if softmax_scale is None:
            softmax_scale = 1.0 / float(np.sqrt(head_dim))
        if budget_max is None:
            budget_max = cap - 1
        b32 = np.ascontiguousarray(np.asarray(budgets, dtype=np.int32).reshape(n_layers, batch, n_kv_heads))
        if pool_slots is None:
            probe = Layout(n_layers, batch, n_q_heads, n_kv_heads, head_dim, cap, out_dtype, headroom, 0)
            pool_slots = self.lib.ckv_pool_slots(C.byref(probe), _np_ptr(b32), int(prompt_len))
            if pool_slots <= 0:
                raise CkvError(EINVAL, "layout rejected")
        self.headroom, self.pool_slots = headroom, int(pool_slots)
        self.layout = Layout(n_layers, batch, n_q_heads, n_kv_heads, head_dim, cap, out_dtype, headroom, int(pool_slots))
        self.params = LrfuParams(lam, top_p, softmax_scale, reward_mode, t0, budget_min, budget_max)
        self.L, self.Bz, self.Hq, self.Hkv, self.d, self.cap = n_layers, batch, n_q_heads, n_kv_heads, head_dim, cap
        self.G = n_q_heads // max(n_kv_heads, 1)
        self.units = n_layers * batch * n_kv_heads
        self.out_dtype = out_dtype
        ws = self.lib.ckv_workspace_bytes(C.byref(self.layout), C.byref(self.params))
        if ws == 0:
            raise CkvError(EINVAL, "layout or parameters rejected")
        S = self.pool_slots
        dev = self.device
        if arena is not None:
            sizes = _buffer_sizes(S, head_dim, ws)
            if pools is not None:                 # K and V from `pools`, the other five buffers from the arena
                sizes[0] = sizes[1] = 0
            al = 2 << 20
            offs, total = [], (-arena.data_ptr()) % al
            for b_ in sizes:
                offs.append(total)
                total += (b_ + al - 1) // al * al
            if arena.dtype != torch.uint8 or not arena.is_contiguous() or arena.numel() < total:
                raise CkvError(EINVAL, f"arena must be a contiguous uint8 tensor of at least {total} bytes")
            part = lambda i, dt: arena[offs[i]:offs[i] + sizes[i]].view(dt)
            self.arena = arena
            self.k_pool, self.v_pool = (part(0, torch.bfloat16), part(1, torch.bfloat16)) if pools is None else pools
            self.crf, self.tau, self.pos = part(2, torch.float32), part(3, torch.int32), part(4, torch.int32)
            self.flags, self.workspace = part(5, torch.uint8), part(6, torch.uint8)
        elif pools is not None:                   # caller-owned K and V pools (bf16 tensors of S * head_dim elements each)
            self.k_pool, self.v_pool = pools
            for p_ in pools:
                if p_.dtype != torch.bfloat16 or p_.numel() < S * head_dim or not p_.is_contiguous() or p_.data_ptr() % 256:
                    raise CkvError(EINVAL, "pools must be contiguous, 256-byte aligned bf16 tensors of pool_slots * head_dim elements")
        else:
            self.k_pool = torch.empty(S * head_dim, dtype=torch.bfloat16, device=dev)
            self.v_pool = torch.empty(S * head_dim, dtype=torch.bfloat16, device=dev)
        if arena is None:
            self.crf = torch.empty(S, dtype=torch.float32, device=dev)
            self.tau = torch.empty(S, dtype=torch.int32, device=dev)
            self.pos = torch.empty(S, dtype=torch.int32, device=dev)
            self.flags = torch.empty(S, dtype=torch.uint8, device=dev)
            self.workspace = torch.empty(ws + 256, dtype=torch.uint8, device=dev)
        wptr = (self.workspace.data_ptr() + 255) // 256 * 256
        self.buffers = Buffers(self.k_pool.data_ptr(), self.v_pool.data_ptr(), self.crf.data_ptr(),
                               self.tau.data_ptr(), self.pos.data_ptr(), self.flags.data_ptr(), wptr, ws)
        b = np.ascontiguousarray(np.asarray(budgets, dtype=np.int32).reshape(n_layers, batch, n_kv_heads))
        self.ctx = C.c_void_p()
        with torch.cuda.device(self.device):
            rc = self.lib.ckv_init(C.byref(self.ctx), C.byref(self.layout), _np_ptr(b), C.byref(self.params),
                                   C.byref(self.buffers), self._stream())
        if rc != OK:
            self.ctx = C.c_void_p()
            raise CkvError(rc, "ckv_init")

    # ------------------------------------------------------------------ plumbing
    def _stream(self):
        return C.c_void_p(self.torch.cuda.current_stream(self.device).cuda_stream)

    def _check(self, rc):
        if rc != OK:
            raise CkvError(rc, self.lib.ckv_last_error(self.ctx).decode())

    def close(self):
        if getattr(self, "ctx", None) and self.ctx.value:
            self.torch.cuda.synchronize(self.device)
            self.lib.ckv_destroy(self.ctx)
            self.ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _dev_bf16(self, x, shape):
        t = self.torch
        if isinstance(x, np.ndarray):
            x = t.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(self.device).to(t.bfloat16)
        assert x.dtype == t.bfloat16 and x.is_contiguous() and tuple(x.shape) == tuple(shape), (x.dtype, x.shape, shape)
        return x

    # ------------------------------------------------------------------ calls
    def load_prompt(self, layer, k, v, crf0=None, tau0=None):
        """k, v: [Bz][Hkv][P][d] (numpy float32 on the bf16 grid, or device bf16 tensors)."""
        P = k.shape[2]
        k = self._dev_bf16(k, (self.Bz, self.Hkv, P, self.d))
        v = self._dev_bf16(v, (self.Bz, self.Hkv, P, self.d))
        t = self.torch
        c0 = t.as_tensor(crf0, dtype=t.float32, device=self.device).contiguous() if crf0 is not None else None
        t0 = t.as_tensor(tau0, dtype=t.int32, device=self.device).contiguous() if tau0 is not None else None
        self._check(self.lib.ckv_load_prompt(self.ctx, layer, k.data_ptr(), v.data_ptr(), P,
                                             c0.data_ptr() if c0 is not None else None,
                                             t0.data_ptr() if t0 is not None else None, self._stream()))
        self._keep = (k, v, c0, t0)

    def seed_prompt(self, layer, q_obs):
        """q_obs: [W][Bz][Hq][d], the queries of the prompt's last W positions (numpy on the bf16 grid or a
        device bf16 tensor): replaces the loaded prompt's scores by those the W queries give them."""
        W = q_obs.shape[0]
        q = self._dev_bf16(q_obs, (W, self.Bz, self.Hq, self.d))
        self._check(self.lib.ckv_seed_prompt(self.ctx, layer, q.data_ptr(), W, self._stream()))
        self._keep_q = q

    def load_cache(self, layer, k, v, lengths, crf0, tau0, pos0):
        """Device tensors: k, v bf16 [Bz][Hkv][P][d]; lengths int32 [Bz][Hkv]; crf0 f32, tau0 / pos0 int32 [Bz][Hkv][P]."""
        t = self.torch
        P = k.shape[2]
        k = self._dev_bf16(k, (self.Bz, self.Hkv, P, self.d))
        v = self._dev_bf16(v, (self.Bz, self.Hkv, P, self.d))
        for x, dt in ((lengths, t.int32), (crf0, t.float32), (tau0, t.int32), (pos0, t.int32)):
            assert x.dtype == dt and x.is_contiguous() and x.device == k.device
        self._check(self.lib.ckv_load_cache(self.ctx, layer, k.data_ptr(), v.data_ptr(), P, lengths.data_ptr(),
                                            crf0.data_ptr(), tau0.data_ptr(), pos0.data_ptr(), self._stream()))

    def decode_step(self, q, k_new, v_new, layer=-1, evict=True, out=None, attention_only=False, defer=False):
        """q [L][Bz][Hq][d], k_new / v_new [L][Bz][Hkv][d] (no leading [L] for a single layer).
        Returns the device tensor `out` of the same shape as q.  defer (single layers only): the layer's
        bookkeeping runs on one of the context's own streams, see `join`."""
        t = self.torch
        lead = (self.L,) if layer == -1 else ()
        q = self._dev_bf16(q, lead + (self.Bz, self.Hq, self.d))
        k_new = self._dev_bf16(k_new, lead + (self.Bz, self.Hkv, self.d))
        v_new = self._dev_bf16(v_new, lead + (self.Bz, self.Hkv, self.d))
        if out is None:
            out = t.empty(q.shape, dtype=t.float32 if self.out_dtype == F32 else t.bfloat16, device=self.device)
        self._check(self.lib.ckv_decode_step(self.ctx, layer, q.data_ptr(), k_new.data_ptr(), v_new.data_ptr(),
                                             out.data_ptr(),
                                             (ATTENTION_ONLY if attention_only else (FUSE_EVICT if evict else 0))
                                             | (DEFER_BOOKKEEPING if defer else 0), self._stream()))
        return out

    def join(self):
        """Order the current stream after the bookkeeping that deferred steps left in flight."""
        self._check(self.lib.ckv_join(self.ctx, self._stream()))

    def evict(self, layer=-1):
        self._check(self.lib.ckv_evict(self.ctx, layer, self._stream()))

    def evict_window(self, n_sink, layer=-1):
        """The sink-plus-recent-window comparison policy: keep positions below n_sink and the newest entries."""
        self._check(self.lib.ckv_evict_window(self.ctx, layer, n_sink, self._stream()))

    def rebudget(self):
        self._check(self.lib.ckv_rebudget(self.ctx, self._stream()))

    def rebalance(self):
        self._check(self.lib.ckv_rebalance(self.ctx, self._stream()))

    def probe(self, layer, q_probe):
        """Classes [Bz][Hkv][cap] (uint8 device tensor) of the layer's entries under q_probe [Bz][Hq][d]."""
        t = self.torch
        q = self._dev_bf16(q_probe, (self.Bz, self.Hq, self.d))
        cls = t.full((self.Bz, self.Hkv, self.cap), 255, dtype=t.uint8, device=self.device)
        self._check(self.lib.ckv_probe(self.ctx, layer, q.data_ptr(), cls.data_ptr(), self._stream()))
        return cls

    def probe_noalloc(self, layer, q_probe, classes):
        """ckv_probe with the library's static scratch; q_probe a device bf16 tensor [Bz][Hq][d], `classes` a
        caller-allocated uint8 device tensor [Bz][Hkv][cap] (nothing is allocated here either)."""
        t = self.torch
        assert q_probe.dtype == t.bfloat16 and q_probe.is_contiguous() and tuple(q_probe.shape) == (self.Bz, self.Hq, self.d)
        assert classes.dtype == t.uint8 and classes.is_contiguous() and tuple(classes.shape) == (self.Bz, self.Hkv, self.cap)
        self._check(self.lib.ckv_probe_noalloc(self.ctx, layer, q_probe.data_ptr(), classes.data_ptr(), self._stream()))
        return classes

    def budgets(self):
        b = np.zeros((self.L, self.Bz, self.Hkv), dtype=np.int32)
        self._check(self.lib.ckv_get_budgets(self.ctx, _np_ptr(b)))
        return b

    def segment_table(self):
        """Which pool segments (256 slots each) every unit owns, and the spare list."""
        max_seg = (self.cap + 255) // 256
        owned = np.zeros(self.units, dtype=np.int32)
        rows = np.zeros((self.units, max_seg), dtype=np.int32)
        spare = np.zeros(self.pool_slots // 256, dtype=np.int32)
        n_spare = C.c_int32(0)
        self._check(self.lib.ckv_get_segments(self.ctx, _np_ptr(owned), _np_ptr(rows), _np_ptr(spare), C.byref(n_spare)))
        return dict(owned=owned, rows=rows, spare=spare[:n_spare.value].copy())

    def set_budgets(self, budgets):
        b = np.ascontiguousarray(np.asarray(budgets, dtype=np.int32).reshape(self.L, self.Bz, self.Hkv))
        self._check(self.lib.ckv_set_budgets(self.ctx, _np_ptr(b)))

    def lengths(self):
        b = np.zeros((self.L, self.Bz, self.Hkv), dtype=np.int32)
        self._check(self.lib.ckv_get_lengths(self.ctx, _np_ptr(b)))
        return b

    def time(self):
        t = C.c_int32(0)
        self._check(self.lib.ckv_get_time(self.ctx, C.byref(t)))
        return t.value

    def set_time(self, t):
        self._check(self.lib.ckv_set_time(self.ctx, int(t)))

    def status(self):
        return self.lib.ckv_status(self.ctx)

    def export_unit(self, layer, seq, head, with_kv=True):
        """dict with n, n_evicted, budget and host arrays (K, V as float32) of the unit's live entries;
        `evicted_pos` lists the positions the last eviction removed."""
        n, nev, bud = C.c_int32(0), C.c_int32(0), C.c_int32(0)
        cap, d = self.cap, self.d
        K = np.zeros((cap, d), dtype=np.uint16) if with_kv else None
        V = np.zeros((cap, d), dtype=np.uint16) if with_kv else None
        crf = np.zeros(cap, dtype=np.float32)
        tau = np.zeros(cap, dtype=np.int32)
        pos = np.zeros(cap, dtype=np.int32)
        flags = np.zeros(cap, dtype=np.uint8)
        self._check(self.lib.ckv_export_unit(self.ctx, layer, seq, head, C.byref(n), C.byref(nev), C.byref(bud),
                                             _np_ptr(K) if with_kv else None, _np_ptr(V) if with_kv else None,
                                             _np_ptr(crf), _np_ptr(tau), _np_ptr(pos), _np_ptr(flags)))
        n, nev = n.value, nev.value
        res = dict(n=n, n_evicted=nev, budget=bud.value, crf=crf[:n].copy(), tau=tau[:n].copy(),
                   pos=pos[:n].copy(), flags=flags[:n].copy(), evicted_pos=np.sort(pos[n:n + nev]),
                   evicted_flags=flags[n:n + nev].copy())
        if with_kv:
            res["K"] = (K[:n].astype(np.uint32) << 16).view(np.float32)
            res["V"] = (V[:n].astype(np.uint32) << 16).view(np.float32)
        return res

    def import_unit(self, layer, seq, head, K, V, crf, tau, pos, t_unit):
        """K, V float32 arrays on the bf16 grid, [n][d]."""
        n = int(len(pos))
        Kb = np.ascontiguousarray((np.ascontiguousarray(K, np.float32).view(np.uint32) >> 16).astype(np.uint16))
        Vb = np.ascontiguousarray((np.ascontiguousarray(V, np.float32).view(np.uint32) >> 16).astype(np.uint16))
        crf = np.ascontiguousarray(crf, np.float32)
        tau = np.ascontiguousarray(tau, np.int32)
        pos = np.ascontiguousarray(pos, np.int32)
        self._check(self.lib.ckv_import_unit(self.ctx, layer, seq, head, n, _np_ptr(Kb), _np_ptr(Vb), _np_ptr(crf),
                                             _np_ptr(tau), _np_ptr(pos), int(t_unit)))

    def set_path(self, mode):
        """0 = auto, 1 = separate scan/finish kernels, 2 = fused per-unit kernel."""
        self._check(self.lib.ckv_set_path(self.ctx, int(mode)))

    def path_info(self):
        waves, lds = C.c_int32(0), C.c_int32(0)
        self._check(self.lib.ckv_path_info(self.ctx, C.byref(waves), C.byref(lds)))
        return waves.value, lds.value

    def profile_enable(self, on=True):
        self._check(self.lib.ckv_profile_enable(self.ctx, 1 if on else 0))

    def profile_read(self):
        ms, n = C.c_double(0.0), C.c_int32(0)
        self._check(self.lib.ckv_profile_read(self.ctx, C.byref(ms), C.byref(n)))
        return ms.value, n.value


def place_pools(pool_bytes, device="cuda:0", max_fraction=0.92, verbose=False, rest_bytes=0):
    """Device memory for the K and V pools (`pool_bytes` each), chosen by measurement; returns (k_pool, v_pool,
    rest, report): bf16 tensors to pass as `pools=` to CrystalKV and, if rest_bytes > 0, a uint8 tensor of at least
    rest_bytes to pass as `arena=` beside them (the per-slot arrays and the workspace are then carved from it).

    On MI355X the decode kernels run about a tenth slower or faster depending on where their buffers lie in
    physical memory (regions tens of GB wide; plain streaming reads do not see them).  Where an allocation lands
    is the driver's business, but consecutive allocations of a process walk through the memory.  So, once, at
    start-up, in two stages.  First: allocate buffers of twice the pool size one after another without freeing
    any, until `max_fraction` of the device's memory is in use (each is a different piece of memory), and time
    a few attention-only decode steps of a synthetic context whose K and V pools are the buffer's halves (random
    keys, units of 2048 entries, as many as fit; its other buffers lie wherever the allocator puts them); the
    fastest buffers whose neighbours in allocation order are about as fast (a buffer that straddles a boundary
    is not wanted) are the candidates for the pools.  Second (if rest_bytes > 0): where the other buffers lie
    matters as well, and not in a way the first stage shows (beside pools in a fast buffer, some fast buffers
    are bad places for them and the slow ones good ones), so whole decode steps (attention, scores, one
    eviction per unit) of the synthetic context are timed with the pools in each of the two best candidates and
    the other buffers in each of the others, and the fastest pair is kept (two times 47 trials of about 15 ms at
    most).  Everything else is freed."""
    import torch
    dev = torch.device(device)
    pool_bytes = (int(pool_bytes) + (2 << 20) - 1) // (2 << 20) * (2 << 20)
    L, Hq, Hkv, n_ent, cap = 1, 32, 8, 2048, 2304
    Bz = int(min(8192, pool_bytes // (cap * 256)) // Hkv)

    def unplaced(note):
        k = torch.empty(pool_bytes // 2, dtype=torch.bfloat16, device=dev)
        v = torch.empty(pool_bytes // 2, dtype=torch.bfloat16, device=dev)
        rest = torch.empty(int(rest_bytes), dtype=torch.uint8, device=dev) if rest_bytes > 0 else None
        return k, v, rest, dict(candidates=0, note=note)

    if Bz < 64:
        return unplaced("pools too small to matter: not placed")
    need = Bz * Hkv * cap * 256
    gen = torch.Generator(device=dev)
    gen.manual_seed(1)
    q = torch.randn((L, Bz, Hq, 128), generator=gen, device=dev).to(torch.bfloat16)
    kn = torch.randn((L, Bz, Hkv, 128), generator=gen, device=dev).to(torch.bfloat16)
    kc = torch.randn((Bz, Hkv, n_ent, 128), generator=gen, device=dev).to(torch.bfloat16)
    out = torch.empty((L, Bz, Hq, 128), dtype=torch.float32, device=dev)
    b_roomy = np.full((L, Bz, Hkv), cap - 1, dtype=np.int32)       # attention-only steps: nothing is ever evicted
    b_full = np.full((L, Bz, Hkv), n_ent, dtype=np.int32)         # whole steps: every unit at its budget, one eviction per step
    own_rest = arena_bytes(L, Bz, Hq, Hkv, 128, cap, b_full, t0=n_ent) - 2 * need      # the synthetic context's other buffers

    def trial(buf, rest=None, whole=False):
        g = CrystalKV(L, Bz, Hq, Hkv, 128, cap, b_full if whole else b_roomy, t0=n_ent, device=dev, arena=rest,
                      pools=(buf[:need].view(torch.bfloat16), buf[pool_bytes:pool_bytes + need].view(torch.bfloat16)))
        g.set_path(3)
        g.load_prompt(0, kc, kc)
        reps = 8 if whole else 6
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
        step = (lambda: g.decode_step(q, kn, kn, out=out, evict=True)) if whole else \
               (lambda: g.decode_step(q, kn, kn, out=out, attention_only=True, evict=False))
        step()
        ev[0].record()
        for j in range(reps):
            step()
            ev[j + 1].record()
        torch.cuda.synchronize(dev)
        ms = float(np.median([ev[j].elapsed_time(ev[j + 1]) for j in range(reps)]))
        g.close()
        return ms

    torch.cuda.empty_cache()              # what torch holds in reserve counts as in use otherwise
    cands, times, spacers = [], [], []
    # at most 48 candidates: small pools are tried at even distances, with spacers (freed afterwards) between them
    one = max(2 * pool_bytes, int(rest_bytes))
    free_b, total_b = torch.cuda.mem_get_info(dev)
    span = max(0, int(max_fraction * total_b) - (total_b - free_b))
    spacer_bytes = max(0, span // 48 - one) // (2 << 20) * (2 << 20)
    while True:
        free_b, total_b = torch.cuda.mem_get_info(dev)
        if free_b < one + (4 << 30) or (total_b - free_b + one) > max_fraction * total_b:
            break
        buf = torch.empty(one, dtype=torch.uint8, device=dev)
        cands.append(buf)
        times.append(trial(buf))
        free_b, _ = torch.cuda.mem_get_info(dev)
        if spacer_bytes and free_b > spacer_bytes + one + (4 << 30):
            spacers.append(torch.empty(spacer_bytes, dtype=torch.uint8, device=dev))
    del spacers
    if not cands:
        del kc, q, kn, out
        return unplaced("no room to try placements")
    t = np.asarray(times)
    fastest = float(t.min())
    # settled = both neighbours within 1 % of the candidate itself (the ends count their one neighbour)
    ok = [i for i in range(len(t)) if all(abs(t[j] - t[i]) <= 0.01 * t[i] for j in (i - 1, i + 1) if 0 <= j < len(t))]
    ranked = sorted((i for i in ok if t[i] <= 1.01 * fastest), key=lambda i: t[i]) or [int(np.argmin(t))]
    pick, rest_at, pairs = ranked[0], None, []
    if rest_bytes > 0 and len(cands) > 1 and own_rest <= one:
        by_time = [int(i) for i in np.argsort(t)]
        for kv in ranked[:2]:
            others = [i for i in by_time if i != kv]
            for r in sorted(others):
                pairs.append((kv, r, trial(cands[kv], cands[r], whole=True)))
        pick, rest_at, _ = min(pairs, key=lambda x: x[2])
    del kc, q, kn, out
    buf = cands[pick]
    k = buf[:pool_bytes].view(torch.bfloat16)
    v = buf[pool_bytes:2 * pool_bytes].view(torch.bfloat16)
    rest = cands[rest_at] if rest_at is not None else None
    report = dict(candidates=len(cands), calibration_units=L * Bz * Hkv, step_ms_min=round(fastest, 4),
                  step_ms_max=round(float(t.max()), 4), step_ms_first=round(float(t[0]), 4), chosen=int(pick),
                  step_ms_chosen=round(float(t[pick]), 4), rest_in=rest_at,
                  whole_step_ms={f"{kv}+{r}": round(ms, 4) for kv, r, ms in pairs})
    if verbose:
        print("place_pools:", report, [round(float(x), 3) for x in t], flush=True)
    del cands, buf
    torch.cuda.empty_cache()
    if rest is None and rest_bytes > 0:
        rest = torch.empty(int(rest_bytes), dtype=torch.uint8, device=dev)
    return k, v, rest, report


def bandwidth_probe(n_bytes=4 << 30, copy=False, reps=5, device="cuda:0"):
    """GB/s of the library's plain streaming-read (or copy: read + written bytes) kernel on this machine."""
    import torch
    lib = load()
    dev = torch.device(device)
    with torch.cuda.device(dev):
        src = torch.ones(n_bytes // 4, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src) if copy else None
        sink = torch.zeros(4, dtype=torch.int32, device=dev)
        stream = C.c_void_p(torch.cuda.current_stream(dev).cuda_stream)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

        def launch():
            rc = lib.ckv_bandwidth_probe(src.data_ptr(), dst.data_ptr() if copy else None, n_bytes, sink.data_ptr(), stream)
            if rc != OK:
                raise CkvError(rc, "ckv_bandwidth_probe")

        launch()
        a.record()
        for _ in range(reps):
            launch()
        b.record()
        torch.cuda.synchronize(dev)
        ms = a.elapsed_time(b) / reps
    return n_bytes * (2 if copy else 1) / (ms * 1e-3) / 1e9
