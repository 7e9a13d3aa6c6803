"""Shared helpers of the test-suite: build oracle configs / library params from a workload and
replay oracle trajectories.  The oracle (CPU) and the HIP binding are only ever brought together
here and in the tests themselves."""
from __future__ import annotations

import numpy as np

import oracle
from paper_2506_18226_amd import workloads as WL


def oracle_cfg(wl, *, P=None, budget=None, score_mode=None, cap=0, n_keep_prefix=None):
    P = wl.prefix_len if P is None else P
    use_frac = wl.budget_den > 0 and budget is None
    return oracle.make_cfg(
        n_heads=wl.n_heads, head_dim=wl.head_dim, grid_h=wl.grid_h, grid_w=wl.grid_w,
        win_rows_back=wl.win_rows_back, win_col_radius=wl.win_col_radius, grid_origin=P,
        n_keep_prefix=n_keep_prefix,
        budget=(wl.budget if budget is None else budget) if not use_frac else 0,
        budget_num=wl.budget_num if use_frac else 0, budget_den=wl.budget_den if use_frac else 0,
        score_mode=wl.score_mode if score_mode is None else score_mode, cap=cap, q_per_kv=wl.q_per_kv)


def replay(wl, cfg, layer, seq, stop_before, snapshots=()):
    """Run the oracle free from s = 0 up to (not including) step `stop_before`.
    Returns (q, k, v, state, {s: state copy taken BEFORE step s} for s in snapshots)."""
    P = cfg.grid_origin
    q, k, v = WL.gen_tokens(wl, layer, seq, prefix_len=P)
    st = oracle.CacheState.from_prefix(cfg, k[:P], v[:P])
    snaps = {}
    for s in range(0, stop_before):
        if s in snapshots:
            snaps[s] = st.copy()
        p = P + s - 1
        oracle.step(cfg, st, s, q[p], k[p], v[p])
    if stop_before in snapshots:
        snaps[stop_before] = st.copy()
    return q, k, v, st, snaps


def near_tie_ok(sel_gpu, sel_ref, score_ref, rel=1e-5, abs_tol=1e-7):
    """Two attended sets that differ only in candidates whose oracle scores tie within tolerance."""
    a, b = set(sel_gpu.tolist()), set(sel_ref.tolist())
    if a == b:
        return True
    only_a, only_b = sorted(a - b), sorted(b - a)
    if len(only_a) != len(only_b):
        return False
    vals = np.concatenate([score_ref[only_a], score_ref[only_b]]).astype(np.float64)
    spread = vals.max() - vals.min()
    return bool(spread <= abs_tol + rel * np.abs(vals).max())


def oracle_step_phases(cfg, st, s, q, k_new, v_new):
    """oracle.step spelled out phase by phase (append, select, attend, accumulate, compact) so that a
    test can look at the scores the eviction ranked.  Returns the dict of oracle.step plus
    'score_ranked': the score array just before compaction (slots before compaction)."""
    n0 = st.n_res
    if s >= 1:
        if n0 + 1 > cfg.cap:
            raise RuntimeError("cache full")
        st.K[n0], st.V[n0], st.pos[n0], st.score[n0] = k_new, v_new, cfg.grid_origin + s - 1, 0.0
        st.n_res = n0 + 1
    n = st.n_res
    sel, score = oracle.select(cfg, st.pos[:n], st.score[:n], st.V[:n], s)
    st.score[:n] = score
    out, lse, probs = oracle.attend(cfg, st.K, st.V, q, sel, want_probs=True)
    if cfg.score_mode == 0:
        st.score[:n] = oracle.accumulate(cfg, st.score[:n], sel, probs)
    ranked = st.score[:n].copy()
    keep_map, did = oracle.compact(cfg, st, s)
    if did and cfg.score_mode == 1:
        pass  # compact() recomputed the V-cosine over the rest itself
    return {"out": out, "lse": lse, "sel_idx": sel, "keep_map": keep_map if did else None,
            "compacted": did, "n_res": st.n_res, "score_ranked": ranked}


def rank_host(batch) -> np.ndarray:
    """Ranking value of every slot of a LayerBatch, [n_seq][cap]: its score rows summed (float64, on the host)."""
    return batch.score.cpu().numpy().astype(np.float64).sum(axis=1)
