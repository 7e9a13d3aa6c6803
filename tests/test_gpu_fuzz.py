"""Seeded randomised differential test: adsa_step against the oracle's step over random geometries.

Every case draws a grid, a window, a prefix length, a budget (absolute or fractional), head count,
head size, storage type, cache layout, ranking mode, query grouping and a set of decode steps; the
library gets the oracle's state before each of those steps (teacher-forced, as the graded mode) and
must reproduce the step: attended set and keep map bit-exact (or differing only among candidates
whose oracle scores tie within the float tolerance of the ranking), rows moved bit-exactly, outputs
within the float bars of test_gpu_parity.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_18226_amd import binding as B
from paper_2506_18226_amd import workloads as WL
from paper_2506_18226_amd.batch import LayerBatch, to_device, to_host

from common import oracle_cfg, replay, near_tie_ok, oracle_step_phases, rank_host
from test_gpu_parity import DEV, params_for, load_state, check_out, lse_tol

pytestmark = pytest.mark.gpu

TALLY = {"full": 0, "near_tie": 0}      # (case, step) pairs compared in full / accepted as a near tie


def draw_case(seed):
    g = np.random.default_rng(1000 + seed)
    H, W = int(g.integers(2, 9)), int(g.integers(2, 13))
    R = int(g.integers(0, min(3, H)))
    w = int(g.integers(0, W + 2))
    P = int(g.integers(1, 20))
    dtype = "bf16" if g.random() < 0.6 else "f32"
    D = int(g.choice([64, 128]))
    G = int(g.choice([1, 1, 2, 4])) if dtype == "bf16" else 1
    h = int(g.integers(1, 7))
    mode = int(g.choice([WL.SCORE_ATTN_MASS, WL.SCORE_ATTN_MASS, WL.SCORE_VCOS]))
    frac = g.random() < 0.3
    budget = int(g.integers(0, 24))
    kind = str(g.choice(["gauss", "outlier2pct", "lowrank8", "tiny_sink"]))
    wl = WL.get_workload("tiny", n_seq=1, n_heads=h, head_dim=D, grid_h=H, grid_w=W, win_rows_back=R,
                         win_col_radius=w, prefix_len=P, dtype=dtype, budget=0 if frac else budget,
                         budget_num=1 if frac else 0, budget_den=int(g.integers(2, 5)) if frac else 0,
                         score_mode=mode, value_kind=kind, value_scale=float(g.choice([0.125, 0.5, 1.0])),
                         q_per_kv=G, seed=0xF000 + seed)
    n_steps = min(H * W + 1, 10)
    steps = sorted(set(int(x) for x in g.choice(H * W + 1, size=n_steps, replace=False)) | {H * W})
    layout = str(g.choice(["head_major", "slot_major"]))
    return wl, steps, layout


@pytest.mark.parametrize("seed", range(48))
def test_random_geometry_teacher_forced(seed):
    wl, steps, layout = draw_case(seed)
    cfg = oracle_cfg(wl)
    q, k, v, _, snaps = replay(wl, cfg, 0, 0, max(steps), snapshots=set(steps))
    P = cfg.grid_origin
    params = params_for(wl, len(steps), cfg.cap, layout=layout)
    batch = LayerBatch(params, DEV)
    for b, s in enumerate(steps):
        load_state(batch, b, snaps[s], cfg, s)
    batch.upload_seqs()
    pp = [P + s - 1 for s in steps]
    qd, kd, vd = (to_device(np.stack([x[p] for p in pp]), params.dtype, DEV) for x in (q, k, v))
    batch.step(qd, kd, vd)
    torch.cuda.synchronize()
    seqs = batch.read_seqs()
    out, lse = to_host(batch.out), batch.lse.cpu().numpy()
    sel_idx, sel_cnt = batch.sel_idx.cpu().numpy(), batch.sel_cnt.cpu().numpy()
    keep_map, posd, rank = batch.keep_map.cpu().numpy(), batch.pos.cpu().numpy(), rank_host(batch)
    Kd, Vd = batch.k_host(), batch.v_host()
    vcos = wl.score_mode == WL.SCORE_VCOS
    for b, s in enumerate(steps):
        st = snaps[s].copy()
        tag = f"seed={seed} {wl.grid_h}x{wl.grid_w} R={wl.win_rows_back} w={wl.win_col_radius} P={P} h={wl.n_heads} " \
              f"D={wl.head_dim} G={wl.q_per_kv} {wl.dtype} {layout} mode={wl.score_mode} s={s}"
        ref = oracle_step_phases(cfg, st, s, q[pp[b]], k[pp[b]], v[pp[b]])
        assert seqs["status"][b] == 0 and seqs["step"][b] == s + 1, tag
        cnt = int(sel_cnt[b])
        same_sel = cnt == ref["sel_idx"].size and np.array_equal(sel_idx[b, :cnt], ref["sel_idx"])
        if not same_sel:
            # V-cosine scores are computed in fp32 on the GPU: only near-ties (by the oracle's scores) may differ
            assert vcos and near_tie_ok(sel_idx[b, :cnt], ref["sel_idx"], ref["score_ranked"], rel=1e-4, abs_tol=4e-6), tag
            TALLY["near_tie"] += 1
            continue
        check_out(wl, out[b], ref["out"], tag)
        assert np.abs(lse[b] - ref["lse"]).max() <= lse_tol(wl), tag
        assert bool(seqs["compacted"][b]) == ref["compacted"], tag
        n = st.n_res
        assert seqs["n_res"][b] == n, tag
        if ref["compacted"]:
            km = ref["keep_map"]
            gmap = keep_map[b, :km.size]
            if not np.array_equal(gmap, km):
                assert near_tie_ok(np.nonzero(gmap >= 0)[0], np.nonzero(km >= 0)[0], ref["score_ranked"],
                                   rel=1e-4 if vcos else 1e-5, abs_tol=4e-6 if vcos else 1e-7), tag
                TALLY["near_tie"] += 1
                continue
        assert np.array_equal(posd[b, :n], st.pos[:n]), tag
        assert np.array_equal(Kd[b, :n], st.K[:n]) and np.array_equal(Vd[b, :n], st.V[:n]), tag
        if not vcos:
            assert np.allclose(rank[b, :n], st.score[:n], rtol=1e-5, atol=1e-6), tag
        TALLY["full"] += 1


# ----------------------------------------------------------------------------- the paper's cache policy, free-running
def draw_streaming_case(seed):
    g = np.random.default_rng(5000 + seed)
    H, W = int(g.integers(3, 8)), int(g.integers(3, 11))
    P = int(g.integers(1, 12))
    m = int(g.integers(2, 2 * W))
    n_pin = int(g.integers(0, P + 1))                     # part of the prefix may be left unpinned (evictable)
    cap = max(n_pin, 1) + m + int(g.integers(2, 12))      # room for pinned prefix + window + a few candidates
    cap = max(cap, P + 1)                                 # the prefix itself must fit before decoding starts
    dtype = "bf16" if g.random() < 0.6 else "f32"
    D = int(g.choice([64, 128]))
    h = int(g.integers(1, 7))
    mode = int(g.choice([B.SCORE_VCOS, B.SCORE_ATTN_MASS, B.SCORE_VCOS_FUSED]))
    policy = B.EVICT_REUSE_SLOT if (mode == B.SCORE_VCOS_FUSED or g.random() < 0.5) else B.EVICT_WHEN_FULL
    layout = "head_major" if (mode == B.SCORE_VCOS_FUSED or g.random() < 0.5) else "slot_major"
    kind = str(g.choice(["gauss", "outlier2pct", "lowrank8"]))
    wl = WL.get_workload("tiny", n_seq=1, n_heads=h, head_dim=D, grid_h=H, grid_w=W, win_rows_back=0,
                         win_col_radius=0, prefix_len=P, dtype=dtype, budget=0, value_kind=kind,
                         value_scale=float(g.choice([0.25, 1.0])), seed=0xE000 + seed)
    return wl, m, n_pin, cap, mode, policy, layout


@pytest.mark.parametrize("seed", range(24))
def test_random_streaming_cache_free_running(seed):
    """Section 4.2 as written (evict the most redundant candidate when full), over random shapes, ranking
    modes (two-pass V-cosine, V-cosine fused into attention, attention mass), both eviction forms and both
    layouts: the GPU runs the whole trajectory on its own state, the oracle on its own; after every step
    the two caches must hold the same tokens (compared by position) with identical rows, and the outputs
    must agree.  A differing victim is accepted only where the oracle's scores of the two tie."""
    wl, m, n_pin, cap, mode, policy, layout = draw_streaming_case(seed)
    omode = B.SCORE_VCOS if mode == B.SCORE_VCOS_FUSED else mode
    P, H, W = wl.prefix_len, wl.grid_h, wl.grid_w
    cfg = oracle.make_cfg(n_heads=wl.n_heads, head_dim=wl.head_dim, grid_h=H, grid_w=W, win_rows_back=0,
                          win_col_radius=0, grid_origin=P, n_keep_prefix=n_pin, budget=10 ** 6, score_mode=omode,
                          cap=cap, win_recent_m=m, evict_when_full=1)
    q, k, v = WL.gen_tokens(wl, 0, 0, prefix_len=P)
    st = oracle.CacheState.from_prefix(cfg, k[:P], v[:P])
    params = B.make_params(n_seq=1, n_heads=wl.n_heads, head_dim=wl.head_dim, grid_h=H, grid_w=W, win_rows_back=0,
                           win_col_radius=0, dtype=B.F32 if wl.dtype == "f32" else B.BF16, score_mode=mode, cap=cap,
                           layout=layout, win_recent_m=m, evict_policy=policy)
    batch = LayerBatch(params, DEV)
    load_state(batch, 0, st, cfg, 0)
    batch.upload_seqs()
    qd, kd, vd = (to_device(x, params.dtype, DEV) for x in (q, k, v))
    tag0 = f"seed={seed} {H}x{W} P={P} pinned={n_pin} m={m} cap={cap} h={wl.n_heads} D={wl.head_dim} {wl.dtype} " \
           f"{layout} mode={mode} policy={policy}"
    evictions = 0
    for s in range(0, H * W + 1):
        p = P + s - 1
        before = st.copy()
        batch.step(qd[p:p + 1], kd[p:p + 1], vd[p:p + 1])
        ref = oracle.step(cfg, st, s, q[p], k[p], v[p])
        torch.cuda.synchronize()
        seqs = batch.read_seqs()
        tag = f"{tag0} s={s}"
        n = st.n_res
        assert seqs["status"][0] == 0 and seqs["step"][0] == s + 1 and seqs["n_res"][0] == n, tag
        assert bool(seqs["compacted"][0]) == ref["compacted"], tag
        evictions += int(ref["compacted"])
        posd = batch.pos.cpu().numpy()[0, :n]
        if set(posd.tolist()) != set(st.pos[:n].tolist()):
            # the two sides evicted different tokens: legitimate only if the oracle's scores of the two tie
            only_g = sorted(set(posd.tolist()) - set(st.pos[:n].tolist()))
            only_o = sorted(set(st.pos[:n].tolist()) - set(posd.tolist()))
            assert len(only_g) == 1 and len(only_o) == 1, tag
            nb = before.n_res
            if omode == B.SCORE_VCOS:
                cls = oracle.classify(cfg, before.pos[:nb], s)
                cand = np.nonzero(cls == oracle.CANDIDATE)[0]
                sc = np.zeros(nb)
                sc[cand] = oracle.vcos(cfg, before.V, cand)
            else:
                sc = before.score[:nb].astype(np.float64)
            a = sc[np.nonzero(before.pos[:nb] == only_g[0])[0][0]]       # the oracle evicted this one
            b_ = sc[np.nonzero(before.pos[:nb] == only_o[0])[0][0]]      # the GPU evicted this one
            assert abs(a - b_) <= 4e-6 + 1e-4 * max(abs(a), abs(b_)), tag
            TALLY["near_tie"] += 1
            break
        order = np.argsort(posd, kind="stable")
        assert np.array_equal(posd[order], st.pos[:n]), tag
        if policy == B.EVICT_WHEN_FULL:
            assert np.array_equal(posd, st.pos[:n]), tag                   # this form keeps position order
        assert np.array_equal(batch.k_host()[0, :n][order], st.K[:n]), tag
        assert np.array_equal(batch.v_host()[0, :n][order], st.V[:n]), tag
        if mode == B.SCORE_ATTN_MASS:
            assert np.allclose(rank_host(batch)[0, :n][order], st.score[:n], rtol=1e-5, atol=1e-6), tag
        check_out(wl, to_host(batch.out)[0], ref["out"], tag)
        TALLY["full"] += 1
    assert evictions >= 1 or cap >= P + H * W, tag0


def test_random_cases_were_compared_in_full():
    """The near-tie escape must stay the exception (runs after the cases above, same process)."""
    total = TALLY["full"] + TALLY["near_tie"]
    if total == 0:
        pytest.skip("the randomised cases did not run in this process")
    print(f"randomised cases: {TALLY['full']} steps compared in full, {TALLY['near_tie']} accepted as near ties")
    assert TALLY["near_tie"] <= 0.05 * total
