"""Seeded synthetic workloads for ADSA decode (inputs only, no method arithmetic).

Every tensor the tests, the smoke check and the benchmark feed to the CPU oracle
and to the HIP library comes from here, so that both sides see bit-identical
inputs.  The generators stand in for the paper's LlamaGen runs on ImageNet and
MS-COCO (Section 5), whose datasets and weights are not available: shapes
follow the LlamaGen configurations the paper evaluates (24x24 = 576 and
32x32 = 1024 image tokens, Section 5.1), values are seeded Gaussians with the
outlier / low-rank structure each configuration names.

This module imports neither the oracle nor the HIP binding.  It draws random
numbers with numpy's counter-based Philox generator keyed by
(seed, layer, sequence, purpose); values for the bf16 configurations are
rounded to bf16 (round-to-nearest-even) here, once, so rounding of inputs never
enters an error budget.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, Tuple

import numpy as np

SCORE_ATTN_MASS = 0      # keep the candidates with the LARGEST accumulated attention mass
SCORE_VCOS = 1           # keep the candidates with the SMALLEST mean V-cosine (Eq. 2-4)
SCORE_EXT_LARGEST = 2    # caller-provided score, keep largest
SCORE_EXT_SMALLEST = 3   # caller-provided score, keep smallest

_BASE_SEED = 0xAD5A0000


@dataclass(frozen=True)
class Workload:
    """Shape and policy of one ADSA decode workload (one row of the config list)."""
    name: str
    index: int                 # position in the config list; seed = base + index
    n_seq: int
    n_layers: int
    n_heads: int
    head_dim: int
    dtype: str                 # "f32" | "bf16"
    prefix_len: int            # P (uniform configs); ragged draws per sequence
    grid_h: int
    grid_w: int
    win_rows_back: int         # R
    win_col_radius: int        # w
    budget: int                # absolute global budget B (used when budget_den == 0)
    budget_num: int = 0
    budget_den: int = 0        # B = floor((P + s) * num / den) when den > 0
    score_mode: int = SCORE_ATTN_MASS
    value_kind: str = "gauss"  # "tiny_sink" | "outlier2pct" | "lowrank8" | "gauss"
    value_scale: float = 1.0
    ragged: bool = False
    q_per_kv: int = 1          # G: query heads per cache head (grouped-query attention when > 1)
    seed: int = field(default=0)

    @property
    def n_image_tokens(self) -> int:
        return self.grid_h * self.grid_w

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def token_bytes(self) -> int:
        """K plus V bytes of one cached token over all heads."""
        return 2 * self.n_heads * self.head_dim * self.elem_bytes

    def max_budget(self) -> int:
        if self.budget_den > 0:
            return ((self.prefix_len + self.n_image_tokens) * self.budget_num) // self.budget_den
        return self.budget

    def cap(self) -> int:
        """Slots per sequence that can never overflow: prefix + budget + (R+1) rows."""
        return self.prefix_len + self.max_budget() + (self.win_rows_back + 1) * self.grid_w

    def sel_cap(self) -> int:
        """Upper bound of the attended set: prefix + local window + budget."""
        local = self.grid_w + self.win_rows_back * (2 * self.win_col_radius + 1)
        return self.prefix_len + local + self.max_budget()


def _mk(index: int, **kw) -> Workload:
    return Workload(index=index, seed=_BASE_SEED + index, **kw)


WORKLOADS: Dict[str, Workload] = {
    "tiny": _mk(0, name="tiny", n_seq=1, n_layers=1, n_heads=16, head_dim=64, dtype="f32",
                prefix_len=32, grid_h=16, grid_w=16, win_rows_back=1, win_col_radius=2,
                budget=64, value_kind="tiny_sink", value_scale=1.0 / 8.0),
    "xl": _mk(1, name="xl", n_seq=16, n_layers=36, n_heads=20, head_dim=64, dtype="bf16",
              prefix_len=120, grid_h=24, grid_w=24, win_rows_back=1, win_col_radius=3,
              budget=0, budget_num=1, budget_den=2, value_kind="outlier2pct"),
    "xxl": _mk(2, name="xxl", n_seq=32, n_layers=48, n_heads=24, head_dim=64, dtype="bf16",
               prefix_len=120, grid_h=32, grid_w=32, win_rows_back=1, win_col_radius=4,
               budget=512, value_kind="lowrank8"),
    "long": _mk(3, name="long", n_seq=4, n_layers=1, n_heads=32, head_dim=128, dtype="bf16",
                prefix_len=256, grid_h=64, grid_w=64, win_rows_back=2, win_col_radius=8,
                budget=1024, value_kind="gauss", value_scale=1.0 / np.sqrt(128.0)),
    "ragged": _mk(4, name="ragged", n_seq=64, n_layers=1, n_heads=24, head_dim=64, dtype="bf16",
                  prefix_len=120, grid_h=32, grid_w=32, win_rows_back=1, win_col_radius=4,
                  budget=512, value_kind="gauss", ragged=True),
    # grouped-query variant (not in the paper, whose models are multi-head): the attention shape of a
    # 34B-class early-fusion token model, 64 query heads over 8 cache heads of 128, on the XXL image grid
    "gqa": _mk(5, name="gqa", n_seq=32, n_layers=48, n_heads=8, head_dim=128, dtype="bf16",
               prefix_len=120, grid_h=32, grid_w=32, win_rows_back=1, win_col_radius=4,
               budget=512, value_kind="lowrank8", q_per_kv=8),
}


def get_workload(name: str, **overrides) -> Workload:
    """Named workload, optionally reshaped (tests shrink n_seq / grid, keep the recipe)."""
    wl = WORKLOADS[name]
    return replace(wl, **overrides) if overrides else wl


# --------------------------------------------------------------------------- rounding
def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are already bf16-representable."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def quantise(wl: Workload, x: np.ndarray) -> np.ndarray:
    return round_to_bf16(x) if wl.dtype == "bf16" else np.ascontiguousarray(x, dtype=np.float32)


# --------------------------------------------------------------------------- streams
_PURPOSE = {"qkv": 1, "struct": 2, "state": 3, "ragged": 4, "score": 5, "gq": 6}


def _rng(wl: Workload, layer: int, seq: int, purpose: str) -> np.random.Generator:
    key0 = (wl.seed << 8) | _PURPOSE[purpose]
    key1 = (layer << 32) | seq
    return np.random.Generator(np.random.Philox(key=[key0, key1]))


def seq_geometry(wl: Workload, seq: int) -> Tuple[int, int, int]:
    """(prefix length P, budget B, decode step s) of one sequence.

    Uniform workloads return (P, budget, -1): the step is chosen by the caller.
    The ragged serving workload draws P ~ U{16..120}, B from {128,256,384,512}
    and s ~ U{1..H*W} per sequence.
    """
    if not wl.ragged:
        return wl.prefix_len, wl.budget, -1
    g = _rng(wl, 0, seq, "ragged")
    p = int(g.integers(16, 121))
    b = int(g.choice(np.array([128, 256, 384, 512])))
    s = int(g.integers(1, wl.n_image_tokens + 1))
    return p, b, s


def gen_tokens(wl: Workload, layer: int, seq: int, prefix_len: int | None = None
               ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """q, k, v for every position of one (layer, sequence): arrays [L][h][D], float32
    (q is [L][h*G][D] for a grouped-query workload, drawn from a stream of its own with the
    same recipe; query head j shares the low-rank basis of cache head j // G).

    Row p holds the post-RoPE query, key and value of the token at absolute
    position p (prefix tokens first, then image tokens in raster order).  Values
    are already rounded to the workload's storage type.
    """
    P = wl.prefix_len if prefix_len is None else prefix_len
    L = P + wl.n_image_tokens
    h, D = wl.n_heads, wl.head_dim
    g = _rng(wl, layer, seq, "qkv")
    kind = wl.value_kind
    if kind == "lowrank8":
        rank = 8
        gs = _rng(wl, layer, seq, "struct")
        M = gs.standard_normal((h, D, rank), dtype=np.float32)          # per-head basis
        U = g.standard_normal((L, h, rank), dtype=np.float32)           # per-token coefficients
        A = g.standard_normal((L, h, rank), dtype=np.float32)
        k = np.einsum("lhr,hdr->lhd", U, M) / np.float32(np.sqrt(rank))
        q = np.einsum("lhr,hdr->lhd", A, M) / np.float32(np.sqrt(rank))
        k += np.float32(0.1) * g.standard_normal((L, h, D), dtype=np.float32)
        q += np.float32(0.1) * g.standard_normal((L, h, D), dtype=np.float32)
        v = g.standard_normal((L, h, D), dtype=np.float32)
    else:
        sc = np.float32(wl.value_scale)
        q = g.standard_normal((L, h, D), dtype=np.float32) * sc
        k = g.standard_normal((L, h, D), dtype=np.float32) * sc
        v = g.standard_normal((L, h, D), dtype=np.float32) * sc
        if kind == "tiny_sink":
            k[:4] *= np.float32(4.0)                                    # attention-sink outliers
        elif kind == "outlier2pct":
            gs = _rng(wl, layer, seq, "struct")
            mask = gs.random(L) < 0.02
            k[mask] *= np.float32(3.0)
    G = wl.q_per_kv
    if G > 1:
        gq = _rng(wl, layer, seq, "gq")
        if kind == "lowrank8":
            A = gq.standard_normal((L, h, G, rank), dtype=np.float32)
            q = (np.einsum("lhgr,hdr->lhgd", A, M) / np.float32(np.sqrt(rank))).reshape(L, h * G, D)
            q += np.float32(0.1) * gq.standard_normal((L, h * G, D), dtype=np.float32)
        else:
            q = gq.standard_normal((L, h * G, D), dtype=np.float32) * np.float32(wl.value_scale)
    return quantise(wl, q), quantise(wl, k), quantise(wl, v)


# --------------------------------------------------------------------------- states
def synthetic_state(wl: Workload, layer: int, seq: int, step: int, prefix_len: int | None = None,
                    budget: int | None = None, tie_fraction: float = 0.25):
    """A legal resident cache for the START of decode step `step` (before its append).

    Used where replaying the trajectory from step 0 is too slow (full-size and
    ragged cases).  Resident positions: the whole prefix, a seeded random subset
    of `min(B, available)` older image tokens, every token of the previous
    `R` completed rows, and the tokens of the current row before the query
    token.  Scores are seeded, non-negative, with a fraction quantised to a few
    levels so exact ties occur.  Returns a dict with
    pos[int32 n], k[n][h][D], v[n][h][D], score[float32 n], q, k_new, v_new [h][D].
    """
    P = wl.prefix_len if prefix_len is None else prefix_len
    B = wl.budget if budget is None else budget
    if wl.budget_den > 0 and budget is None:
        B = ((P + step) * wl.budget_num) // wl.budget_den
    W, R = wl.grid_w, wl.win_rows_back
    q_all, k_all, v_all = gen_tokens(wl, layer, seq, prefix_len=P)
    g = _rng(wl, layer, seq, "state")
    if step == 0:
        image_res = np.zeros(0, dtype=np.int64)
        qpos = P - 1
    else:
        jq = step - 1
        r = jq // W
        first_protected = max(0, (r - R)) * W           # rows r-R .. r-1 fully resident
        older = np.arange(0, first_protected)
        n_keep = min(B, older.size)
        kept_older = np.sort(g.choice(older, size=n_keep, replace=False)) if older.size else older
        recent = np.arange(first_protected, jq)         # excludes the query token itself
        image_res = np.concatenate([kept_older, recent]).astype(np.int64)
        qpos = P + jq
    pos = np.concatenate([np.arange(P, dtype=np.int64), P + image_res]).astype(np.int32)
    n = pos.size
    score = g.gamma(2.0, 0.5, size=n).astype(np.float32)
    tie = g.random(n) < tie_fraction
    score[tie] = np.round(score[tie] * 2.0) / 2.0       # a few exact levels, incl. 0
    return {
        "pos": pos, "k": np.ascontiguousarray(k_all[pos]), "v": np.ascontiguousarray(v_all[pos]),
        "score": score, "q": q_all[qpos].copy(), "k_new": k_all[qpos].copy(),
        "v_new": v_all[qpos].copy(), "prefix_len": P, "budget": B, "step": step,
    }


# --------------------------------------------------------------------------- on-device generation
def gen_tokens_device(wl: Workload, layer: int, device, prefix_len: int | None = None):
    """Same recipe as gen_tokens for ALL sequences of one layer, drawn on the GPU by torch.

    Used only where host generation would dominate the run (the full-size benchmark
    trajectory).  Seeded (per workload and layer) but a different random stream than the
    numpy generator, so never used for parity.  Returns q, k, v as torch tensors
    [n_seq][L][h][D] in the workload's storage type.
    """
    import torch

    P = wl.prefix_len if prefix_len is None else prefix_len
    L = P + wl.n_image_tokens
    n, h, D = wl.n_seq, wl.n_heads, wl.head_dim
    g = torch.Generator(device=device)
    g.manual_seed((wl.seed << 16) | layer)
    tdt = torch.float32 if wl.dtype == "f32" else torch.bfloat16

    def randn(*shape):
        return torch.randn(*shape, generator=g, device=device, dtype=torch.float32)

    kind = wl.value_kind
    if kind == "lowrank8":
        rank = 8
        M = randn(n, h, D, rank)
        U = randn(n, L, h, rank)
        A = randn(n, L, h, rank)
        k = torch.einsum("nlhr,nhdr->nlhd", U, M) / rank ** 0.5 + 0.1 * randn(n, L, h, D)
        q = torch.einsum("nlhr,nhdr->nlhd", A, M) / rank ** 0.5 + 0.1 * randn(n, L, h, D)
        v = randn(n, L, h, D)
        if wl.q_per_kv > 1:
            G = wl.q_per_kv
            A = randn(n, L, h, G, rank)
            q = (torch.einsum("nlhgr,nhdr->nlhgd", A, M) / rank ** 0.5).reshape(n, L, h * G, D)
            q = q + 0.1 * randn(n, L, h * G, D)
    else:
        q = randn(n, L, h, D) * wl.value_scale
        k = randn(n, L, h, D) * wl.value_scale
        v = randn(n, L, h, D) * wl.value_scale
        if kind == "tiny_sink":
            k[:, :4] *= 4.0
        elif kind == "outlier2pct":
            mask = torch.rand(n, L, generator=g, device=device) < 0.02
            k[mask] *= 3.0
        if wl.q_per_kv > 1:
            q = randn(n, L, h * wl.q_per_kv, D) * wl.value_scale
    return q.to(tdt), k.to(tdt), v.to(tdt)
