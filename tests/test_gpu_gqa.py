"""GPU parity of the grouped-query path (q_per_kv = G >= 2, matrix-core kernel) against the CPU oracle.

Bars: the same as for the multi-head path (test_gpu_parity): attended sets bit-exact when both sides
rank the same scores, bf16 outputs within one bf16 rounding of the fp64 result (+1e-4), lse within
1e-4, accumulated scores within 1e-5 relative + 1e-6 absolute.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_18226_amd import binding as B
from paper_2506_18226_amd import workloads as WL
from paper_2506_18226_amd.batch import LayerBatch, to_device, to_host

from common import oracle_cfg, replay, rank_host
from test_gpu_parity import (DEV, LAYOUTS, params_for, load_state, check_out, lse_tol, _full_layer,
                             _check_full_step)

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("G,h,D,reps", [
    (4, 3, 64, 1),        # 39 workgroups: 16 waves each
    (2, 5, 64, 2),        # 130 workgroups: 8 waves
    (8, 8, 128, 5),       # 520 workgroups: 4 waves
    (16, 1, 64, 1),       # a full 16-row query tile
    (3, 2, 128, 1),       # group size that is not a power of two
])
def test_gqa_attend_matches_oracle_on_ragged_index_lists(G, h, D, reps, layout):
    """Eq. 5 + attention with G query heads per cache head, for list lengths from 1 to several
    16-token tiles with ragged tails, and the attention mass that follows (all G queries counted)."""
    wl = WL.get_workload("xxl", n_seq=1, n_heads=h, head_dim=D, grid_h=28, grid_w=28, prefix_len=30, q_per_kv=G)
    rng = np.random.default_rng(11)
    q, k, v = WL.gen_tokens(wl, 0, 0)
    assert q.shape[1] == h * G
    n_tok = k.shape[0]
    lens = [1, 2, 15, 16, 17, 63, 64, 65, 127, 200, 301, 430, 700] * reps
    cap = n_tok
    params = params_for(wl, len(lens), cap, score_mode=B.SCORE_ATTN_MASS, layout=layout)
    batch = LayerBatch(params, DEV)
    cfg = oracle_cfg(wl, budget=cap, cap=cap, score_mode=B.SCORE_ATTN_MASS)
    sels, score0 = [], []
    sel_idx = np.full((len(lens), cap), -1, np.int32)
    for b, n in enumerate(lens):
        sel = np.sort(rng.choice(n_tok, size=n, replace=False)).astype(np.int32)
        sels.append(sel)
        sel_idx[b, :n] = sel
        sc = rng.random(n_tok).astype(np.float32)
        score0.append(sc)
        batch.set_sequence(b, k=k, v=v, pos=np.arange(n_tok, dtype=np.int32), score=sc, step=400,
                           grid_origin=30, budget=cap)
    batch.upload_seqs()
    batch.sel_idx.copy_(torch.from_numpy(sel_idx).to(DEV))
    batch.sel_cnt.copy_(torch.tensor(lens, dtype=torch.int32).to(DEV))
    qd = to_device(np.stack([q[100 + b] for b in range(len(lens))]), params.dtype, DEV)
    batch.attend(qd)
    torch.cuda.synchronize()
    out, lse, score = to_host(batch.out), batch.lse.cpu().numpy(), rank_host(batch)
    for b, n in enumerate(lens):
        ro, rl, probs = oracle.attend(cfg, k, v, q[100 + b], sels[b], want_probs=True)
        check_out(wl, out[b], ro, f"len={n} b={b}")
        assert np.abs(lse[b] - rl).max() <= lse_tol(wl), n
        ref_score = oracle.accumulate(cfg, score0[b], sels[b], probs)
        assert np.allclose(score[b], ref_score, rtol=1e-5, atol=1e-6), n
    before = batch.score.clone()
    batch.attend(qd, flags=B.FLAG_NO_ACCUMULATE)
    torch.cuda.synchronize()
    assert torch.equal(before, batch.score)


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("over,budget,steps,cap", [
    (dict(n_heads=2, head_dim=64, grid_h=6, grid_w=12, prefix_len=17, q_per_kv=4), 10, [0, 1, 3, 12, 13, 30, 36, 60, 72], None),
    (dict(n_heads=3, head_dim=128, grid_h=5, grid_w=16, prefix_len=9, q_per_kv=2), 20, [0, 1, 16, 33, 48, 64, 80], None),
    # caches allocated for 2700 slots and few (sequence, cache head) pairs: the launch splits every list into 8
    # chunks, most of them empty for these short lists; the last chunk's workgroup stores the appended row
    (dict(n_heads=2, head_dim=64, grid_h=6, grid_w=12, prefix_len=17, q_per_kv=4), 10, [0, 1, 3, 12, 13, 30, 36, 60, 72], 2700),
    (dict(n_heads=3, head_dim=128, grid_h=5, grid_w=16, prefix_len=9, q_per_kv=2), 20, [0, 1, 16, 33, 48, 64, 80], 2700),
])
def test_gqa_step_teacher_forced(over, budget, steps, cap, layout):
    """adsa_step (select, append, attend, accumulate, row-end compaction) with grouped queries on the
    oracle's state at step s reproduces the oracle's step."""
    wl = WL.get_workload("xxl", n_seq=1, **over)
    cfg = oracle_cfg(wl, budget=budget) if cap is None else oracle_cfg(wl, budget=budget, cap=cap)
    q, k, v, _, snaps = replay(wl, cfg, 0, 0, max(steps), snapshots=set(steps))
    P = cfg.grid_origin
    params = params_for(wl, len(steps), cfg.cap, layout=layout)
    assert (B.adsa_workspace_bytes(params) > len(steps) * wl.n_heads * wl.q_per_kv * cfg.cap * 4) == (cap is not None)
    batch = LayerBatch(params, DEV)
    for b, s in enumerate(steps):
        load_state(batch, b, snaps[s], cfg, s)
    batch.upload_seqs()
    pp = [P + s - 1 for s in steps]
    qd = to_device(np.stack([q[p] for p in pp]), params.dtype, DEV)
    kd = to_device(np.stack([k[p] for p in pp]), params.dtype, DEV)
    vd = to_device(np.stack([v[p] for p in pp]), params.dtype, DEV)
    batch.step(qd, kd, vd)
    torch.cuda.synchronize()
    seqs = batch.read_seqs()
    out, lse = to_host(batch.out), batch.lse.cpu().numpy()
    sel_idx, sel_cnt = batch.sel_idx.cpu().numpy(), batch.sel_cnt.cpu().numpy()
    keep_map = batch.keep_map.cpu().numpy()
    Kd, Vd, posd, rank = batch.k_host(), batch.v_host(), batch.pos.cpu().numpy(), rank_host(batch)
    for b, s in enumerate(steps):
        st = snaps[s].copy()
        p = P + s - 1
        ref = oracle.step(cfg, st, s, q[p], k[p], v[p])
        tag = f"s={s}"
        assert seqs["status"][b] == 0 and seqs["step"][b] == s + 1, tag
        assert np.array_equal(sel_idx[b, :sel_cnt[b]], ref["sel_idx"]), tag
        check_out(wl, out[b], ref["out"], tag)
        assert np.abs(lse[b] - ref["lse"]).max() <= lse_tol(wl), tag
        assert bool(seqs["compacted"][b]) == ref["compacted"], tag
        n = st.n_res
        if ref["compacted"]:
            assert np.array_equal(keep_map[b, :ref["keep_map"].size], ref["keep_map"]), tag
        assert seqs["n_res"][b] == n, tag
        assert np.array_equal(posd[b, :n], st.pos[:n]), tag
        assert np.array_equal(Kd[b, :n], st.K[:n]) and np.array_equal(Vd[b, :n], st.V[:n]), tag
        assert np.allclose(rank[b, :n], st.score[:n], rtol=1e-5, atol=1e-6), tag


def test_gqa_full_size_layer():
    """The grouped-query workload at full size in the launch configuration the benchmark times
    (32 sequences x 8 cache heads x 8 queries x 128, bf16): deep steps incl. row ends, every sequence
    checked against the oracle."""
    wl, params, batch, items, qd, kd, vd = _full_layer("gqa", steps=[1000, 992, 1024, 513, 33, 960, 1, 700])
    batch.select(flags=B.FLAG_PLAN_APPEND)
    batch.attend(qd, flags=B.FLAG_APPEND, k_new=kd, v_new=vd)
    batch.compact(flags=B.FLAG_ADVANCE)
    torch.cuda.synchronize()
    assert _check_full_step(wl, batch, items) >= 8


def test_gqa_rejects_what_it_does_not_cover():
    """fp32 caches and group sizes beyond 16 are refused on the host, not launched; a list whose logits do not fit in
    LDS is split over several workgroups instead."""
    good = dict(n_seq=2, n_heads=2, head_dim=64, grid_h=8, grid_w=8, win_rows_back=1, win_col_radius=1,
                dtype=B.BF16, score_mode=B.SCORE_ATTN_MASS, cap=256, q_per_kv=4)
    assert B.adsa_workspace_bytes(B.make_params(**good)) > 0
    assert B.adsa_workspace_bytes(B.make_params(**dict(good, dtype=B.F32))) == 0
    assert B.adsa_workspace_bytes(B.make_params(**dict(good, q_per_kv=17))) == 0
    assert B.adsa_workspace_bytes(B.make_params(**dict(good, q_per_kv=16, cap=8192))) > 0


@pytest.mark.parametrize("n_seq", [2, 48])
def test_gqa_long_lists_split_or_on_the_raised_lds_limit(n_seq):
    """Lists of 2400 and 2621 tokens with G = 8.  Two sequences (4 workgroups' worth): every list is split into 16
    chunks whose partials the last workgroup merges.  48 sequences (96 pairs): lists stay whole and the logits of one
    list need more than 64 KB of LDS."""
    G, h, D, n = 8, 2, 64, 2400
    wl = WL.get_workload("xxl", n_seq=1, n_heads=h, head_dim=D, grid_h=51, grid_w=51, prefix_len=20, q_per_kv=G)
    q, k, v = WL.gen_tokens(wl, 0, 0)
    n_tok = k.shape[0]
    params = params_for(wl, n_seq, n_tok, score_mode=B.SCORE_ATTN_MASS)
    batch = LayerBatch(params, DEV)
    cfg = oracle_cfg(wl, budget=n_tok, cap=n_tok, score_mode=B.SCORE_ATTN_MASS)
    rng = np.random.default_rng(3)
    sels = [np.sort(rng.choice(n_tok, size=m, replace=False)).astype(np.int32) for m in ((n, n_tok) * (n_seq // 2))]
    sel_idx = np.full((n_seq, n_tok), -1, np.int32)
    for b, sel in enumerate(sels):
        sel_idx[b, :sel.size] = sel
        batch.set_sequence(b, k=k, v=v, pos=np.arange(n_tok, dtype=np.int32), score=None, step=2000,
                           grid_origin=20, budget=n_tok)
    batch.upload_seqs()
    batch.sel_idx.copy_(torch.from_numpy(sel_idx).to(DEV))
    batch.sel_cnt.copy_(torch.tensor([s.size for s in sels], dtype=torch.int32).to(DEV))
    qd = to_device(np.stack([q[500 + b] for b in range(n_seq)]), params.dtype, DEV)
    batch.attend(qd)
    torch.cuda.synchronize()
    out, lse, score = to_host(batch.out), batch.lse.cpu().numpy(), rank_host(batch)
    for b, sel in enumerate(sels):
        if n_seq > 2 and b % 7 > 1:
            continue                                  # (the oracle checks a sample of the 48)
        ro, rl, probs = oracle.attend(cfg, k, v, q[500 + b], sel, want_probs=True)
        check_out(wl, out[b], ro, f"b={b}")
        assert np.abs(lse[b] - rl).max() <= lse_tol(wl)
        ref_score = oracle.accumulate(cfg, np.zeros(n_tok, np.float32), sel, probs)
        assert np.allclose(score[b], ref_score, rtol=1e-5, atol=1e-6)


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("G,h,D", [(8, 2, 128), (16, 1, 64), (3, 2, 64)])
def test_gqa_split_lists_of_ragged_lengths(G, h, D, layout):
    """Few (sequence, cache head) pairs with caches of 2631 slots: every list is cut into chunks of whole 16-token
    tiles, one workgroup each, and the last workgroup to arrive merges the partials and updates the scores.  Lengths
    from one token (a single non-empty chunk) to the full cache, ragged tails, fewer tiles than chunks."""
    wl = WL.get_workload("xxl", n_seq=1, n_heads=h, head_dim=D, grid_h=51, grid_w=51, prefix_len=30, q_per_kv=G)
    rng = np.random.default_rng(29)
    q, k, v = WL.gen_tokens(wl, 0, 0)
    n_tok = k.shape[0]
    lens = [1, 15, 16, 17, 100, 255, 256, 700, 2000, n_tok]
    params = params_for(wl, len(lens), n_tok, score_mode=B.SCORE_ATTN_MASS, layout=layout)
    # (the workspace of a split launch holds the logits of every list: that is how the split shows from outside)
    assert B.adsa_workspace_bytes(params) > len(lens) * h * G * n_tok * 4
    batch = LayerBatch(params, DEV)
    cfg = oracle_cfg(wl, budget=n_tok, cap=n_tok, score_mode=B.SCORE_ATTN_MASS)
    sels, score0 = [], []
    sel_idx = np.full((len(lens), n_tok), -1, np.int32)
    for b, n in enumerate(lens):
        sel = np.sort(rng.choice(n_tok, size=n, replace=False)).astype(np.int32)
        sels.append(sel)
        sel_idx[b, :n] = sel
        sc = rng.random(n_tok).astype(np.float32)
        score0.append(sc)
        batch.set_sequence(b, k=k, v=v, pos=np.arange(n_tok, dtype=np.int32), score=sc, step=2000,
                           grid_origin=30, budget=n_tok)
    batch.upload_seqs()
    batch.sel_idx.copy_(torch.from_numpy(sel_idx).to(DEV))
    batch.sel_cnt.copy_(torch.tensor(lens, dtype=torch.int32).to(DEV))
    qd = to_device(np.stack([q[100 + b] for b in range(len(lens))]), params.dtype, DEV)
    for rep in range(2):                              # twice: the arrival counters must be back at zero
        batch.attend(qd, flags=B.FLAG_NO_ACCUMULATE if rep == 0 else 0)
        torch.cuda.synchronize()
        out, lse = to_host(batch.out), batch.lse.cpu().numpy()
        for b, n in enumerate(lens):
            ro, rl, probs = oracle.attend(cfg, k, v, q[100 + b], sels[b], want_probs=True)
            check_out(wl, out[b], ro, f"rep={rep} len={n}")
            assert np.abs(lse[b] - rl).max() <= lse_tol(wl), n
            if rep == 1:
                ref_score = oracle.accumulate(cfg, score0[b], sels[b], probs)
                assert np.allclose(rank_host(batch)[b], ref_score, rtol=1e-5, atol=1e-6), n
