"""ctypes marshalling for the C oracle (adsa_oracle.c) -- TEST INFRASTRUCTURE ONLY.

No arithmetic lives here: every function converts numpy arrays to pointers and
calls the C routine of the same name.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libadsa_oracle.so")
_lib = None

PREFIX, LOCAL, CANDIDATE = 0, 1, 2


def build(force: bool = True) -> str:
    """Compile adsa_oracle.c with gcc into libadsa_oracle.so (beside the source)."""
    src = os.path.join(_HERE, "adsa_oracle.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-std=c11", "-O2", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", _SO, src, "-lm"])
    return _SO


class OracleCfg(C.Structure):
    _fields_ = [
        ("n_heads", C.c_int32), ("head_dim", C.c_int32),
        ("grid_h", C.c_int32), ("grid_w", C.c_int32),
        ("win_rows_back", C.c_int32), ("win_col_radius", C.c_int32),
        ("grid_origin", C.c_int32), ("n_keep_prefix", C.c_int32),
        ("budget", C.c_int32), ("budget_num", C.c_int32), ("budget_den", C.c_int32),
        ("score_mode", C.c_int32), ("cap", C.c_int32),
        ("win_recent_m", C.c_int32), ("evict_when_full", C.c_int32), ("q_per_kv", C.c_int32),
        ("softmax_scale", C.c_double),
    ]


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = C.CDLL(_SO)
        _lib.orc_budget.restype = C.c_int32
    return _lib


def _p(a: np.ndarray, ty):
    return a.ctypes.data_as(C.POINTER(ty))


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _chk(rc, what):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def budget(cfg: OracleCfg, s: int) -> int:
    return int(_load().orc_budget(C.byref(cfg), C.c_int32(s)))


def classify(cfg: OracleCfg, pos: np.ndarray, s: int) -> np.ndarray:
    pos = _i32(pos)
    cls = np.empty(pos.size, dtype=np.int32)
    _chk(_load().orc_classify(C.byref(cfg), C.c_int32(pos.size), _p(pos, C.c_int32), C.c_int32(s),
                              _p(cls, C.c_int32)), "classify")
    return cls


def vcos(cfg: OracleCfg, V: np.ndarray, slots: np.ndarray) -> np.ndarray:
    V = _f32(V)
    slots = _i32(slots)
    S = np.empty(slots.size, dtype=np.float64)
    _chk(_load().orc_vcos(C.byref(cfg), _p(V, C.c_float), C.c_int32(slots.size), _p(slots, C.c_int32),
                          _p(S, C.c_double)), "vcos")
    return S


def rank_keep(slots: np.ndarray, score: np.ndarray, keep_largest: bool, B: int) -> np.ndarray:
    slots = _i32(slots)
    score = _f32(score)
    keep = np.zeros(slots.size, dtype=np.uint8)
    n = _load().orc_rank_keep(C.c_int32(slots.size), _p(slots, C.c_int32), _p(score, C.c_float),
                              C.c_int(1 if keep_largest else 0), C.c_int32(B), _p(keep, C.c_uint8))
    if n < 0:
        raise RuntimeError("oracle rank_keep failed")
    return keep.astype(bool)


def select(cfg: OracleCfg, pos: np.ndarray, score: np.ndarray, V, s: int):
    """Returns (sel_idx ascending int32 array, score array after VCOS write-back)."""
    pos = _i32(pos)
    score = _f32(score).copy()
    Vp = _p(_f32(V), C.c_float) if V is not None else None
    sel = np.empty(pos.size + 1, dtype=np.int32)
    cnt = C.c_int32(0)
    _chk(_load().orc_select(C.byref(cfg), C.c_int32(pos.size), _p(pos, C.c_int32), _p(score, C.c_float),
                            Vp, C.c_int32(s), _p(sel, C.c_int32), C.byref(cnt)), "select")
    return sel[:cnt.value].copy(), score


def attend(cfg: OracleCfg, K, V, q, sel_idx, want_probs: bool = False):
    K, V, q = _f32(K), _f32(V), _f32(q)
    sel_idx = _i32(sel_idx)
    h, D = cfg.n_heads * max(cfg.q_per_kv, 1), cfg.head_dim
    out = np.empty((h, D), dtype=np.float64)
    lse = np.empty(h, dtype=np.float64)
    probs = np.empty((h, sel_idx.size), dtype=np.float64) if want_probs else None
    _chk(_load().orc_attend(C.byref(cfg), _p(K, C.c_float), _p(V, C.c_float), _p(q, C.c_float),
                            _p(sel_idx, C.c_int32), C.c_int32(sel_idx.size), _p(out, C.c_double),
                            _p(lse, C.c_double), _p(probs, C.c_double) if want_probs else None), "attend")
    return (out, lse, probs) if want_probs else (out, lse)


def accumulate(cfg: OracleCfg, score, sel_idx, probs) -> np.ndarray:
    score = _f32(score).copy()
    sel_idx = _i32(sel_idx)
    probs = np.ascontiguousarray(probs, dtype=np.float64)
    _chk(_load().orc_accumulate(C.byref(cfg), _p(score, C.c_float), _p(sel_idx, C.c_int32),
                                C.c_int32(sel_idx.size), _p(probs, C.c_double)), "accumulate")
    return score


@dataclass
class CacheState:
    """Caller-owned cache of one (sequence, layer): arrays sized to cfg.cap, n_res valid rows."""
    K: np.ndarray       # float32 [cap][h][D]
    V: np.ndarray
    pos: np.ndarray     # int32 [cap]
    score: np.ndarray   # float32 [cap]
    n_res: int

    @staticmethod
    def from_prefix(cfg: OracleCfg, k_prefix: np.ndarray, v_prefix: np.ndarray) -> "CacheState":
        h, D, cap = cfg.n_heads, cfg.head_dim, cfg.cap
        n = k_prefix.shape[0]
        K = np.zeros((cap, h, D), dtype=np.float32)
        V = np.zeros((cap, h, D), dtype=np.float32)
        K[:n] = k_prefix
        V[:n] = v_prefix
        pos = np.zeros(cap, dtype=np.int32)
        pos[:n] = np.arange(n, dtype=np.int32)
        return CacheState(K, V, pos, np.zeros(cap, dtype=np.float32), n)

    @staticmethod
    def from_arrays(cfg: OracleCfg, k, v, pos, score) -> "CacheState":
        h, D, cap = cfg.n_heads, cfg.head_dim, cfg.cap
        n = len(pos)
        st = CacheState(np.zeros((cap, h, D), np.float32), np.zeros((cap, h, D), np.float32),
                        np.zeros(cap, np.int32), np.zeros(cap, np.float32), n)
        st.K[:n], st.V[:n], st.pos[:n], st.score[:n] = k, v, pos, score
        return st

    def copy(self) -> "CacheState":
        return CacheState(self.K.copy(), self.V.copy(), self.pos.copy(), self.score.copy(), self.n_res)


def compact(cfg: OracleCfg, st: CacheState, s: int):
    """In-place row-end eviction.  Returns (keep_map over the old n_res slots, did)."""
    n_res = C.c_int32(st.n_res)
    keep_map = np.full(st.n_res, -2, dtype=np.int32)
    did = C.c_int32(0)
    _chk(_load().orc_compact(C.byref(cfg), _p(st.K, C.c_float), _p(st.V, C.c_float), _p(st.pos, C.c_int32),
                             _p(st.score, C.c_float), C.byref(n_res), C.c_int32(s),
                             _p(keep_map, C.c_int32), C.byref(did)), "compact")
    st.n_res = n_res.value
    return keep_map, bool(did.value)


def step(cfg: OracleCfg, st: CacheState, s: int, q, k_new, v_new):
    """One decode step on `st` (mutated).  Returns a dict of the step's outputs."""
    q, k_new, v_new = _f32(q), _f32(k_new), _f32(v_new)
    h, D = cfg.n_heads * max(cfg.q_per_kv, 1), cfg.head_dim
    out = np.empty((h, D), dtype=np.float64)
    lse = np.empty(h, dtype=np.float64)
    sel = np.empty(cfg.cap + 1, dtype=np.int32)
    cnt = C.c_int32(0)
    keep_map = np.full(cfg.cap + 1, -2, dtype=np.int32)
    did = C.c_int32(0)
    n_res = C.c_int32(st.n_res)
    rc = _load().orc_step(C.byref(cfg), _p(st.K, C.c_float), _p(st.V, C.c_float), _p(st.pos, C.c_int32),
                          _p(st.score, C.c_float), C.byref(n_res), C.c_int32(s), _p(q, C.c_float),
                          _p(k_new, C.c_float), _p(v_new, C.c_float), _p(out, C.c_double),
                          _p(lse, C.c_double), _p(sel, C.c_int32), C.byref(cnt), _p(keep_map, C.c_int32),
                          C.byref(did))
    _chk(rc, "step")
    n_before = st.n_res if cfg.evict_when_full else st.n_res + (1 if s >= 1 else 0)
    st.n_res = n_res.value
    return {"out": out, "lse": lse, "sel_idx": sel[:cnt.value].copy(),
            "keep_map": keep_map[:n_before].copy() if did.value else None,
            "compacted": bool(did.value), "n_res": st.n_res}


def make_cfg(*, n_heads, head_dim, grid_h, grid_w, win_rows_back, win_col_radius, grid_origin,
             n_keep_prefix=None, budget=0, budget_num=0, budget_den=0, score_mode=0, cap=0,
             softmax_scale=0.0, win_recent_m=0, evict_when_full=0, q_per_kv=0) -> OracleCfg:
    """Fill an OracleCfg; n_keep_prefix defaults to grid_origin, cap to the no-overflow bound."""
    if n_keep_prefix is None:
        n_keep_prefix = grid_origin
    if cap <= 0:
        bmax = budget if budget_den == 0 else ((grid_origin + grid_h * grid_w) * budget_num) // budget_den
        held = (win_rows_back + 1) * grid_w if win_recent_m <= 0 else (win_recent_m - 1) + grid_w
        cap = max(grid_origin, n_keep_prefix) + bmax + held
    return OracleCfg(n_heads, head_dim, grid_h, grid_w, win_rows_back, win_col_radius, grid_origin,
                     n_keep_prefix, budget, budget_num, budget_den, score_mode, cap, win_recent_m,
                     evict_when_full, q_per_kv, softmax_scale)
