"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on identical seeded inputs.

Bars (stated where used):
  * selected indices, counts, keep maps, n_res: bit-exact when both sides get the same score array;
  * attention output: max-abs error <= 1e-5 for fp32; for bf16 storage
    max|gpu - ref| <= 2e-2 * max|ref| per (sequence, head) row, plus an elementwise bound of one
    bf16 rounding (2^-8 relative) + 1e-4 absolute that the arithmetic actually meets;
  * lse: 1e-5 absolute (fp32 inputs) / 1e-4 (bf16 inputs, same fp32 arithmetic, larger logits);
  * accumulated score: 1e-5 relative + 1e-6 absolute.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_18226_amd import binding as B
from paper_2506_18226_amd import workloads as WL
from paper_2506_18226_amd.batch import LayerBatch, ModelBatch, to_device, to_host

from common import oracle_cfg, replay, near_tie_ok, oracle_step_phases, rank_host

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def params_for(wl, n_seq, cap, score_mode=None, sel_cap=None, layout="head_major"):
    return B.make_params(n_seq=n_seq, n_heads=wl.n_heads, head_dim=wl.head_dim, grid_h=wl.grid_h,
                         grid_w=wl.grid_w, win_rows_back=wl.win_rows_back, win_col_radius=wl.win_col_radius,
                         dtype=B.F32 if wl.dtype == "f32" else B.BF16,
                         score_mode=wl.score_mode if score_mode is None else score_mode,
                         cap=cap, sel_cap=sel_cap, layout=layout, q_per_kv=wl.q_per_kv)


LAYOUTS = ["head_major", "slot_major"]


def load_state(batch, b, st, cfg, step):
    batch.set_sequence(b, k=st.K, v=st.V, pos=st.pos[:st.n_res], score=st.score, step=step,
                       grid_origin=cfg.grid_origin, n_keep_prefix=cfg.n_keep_prefix, budget=cfg.budget,
                       budget_num=cfg.budget_num, budget_den=cfg.budget_den)


def check_out(wl, gpu_out, ref_out, what=""):
    """gpu_out, ref_out: [h][D]."""
    err = np.abs(gpu_out.astype(np.float64) - ref_out)
    if wl.dtype == "f32":
        assert err.max() <= 1e-5, f"{what}: fp32 max-abs error {err.max():.3e}"
    else:
        row_ref = np.abs(ref_out).max(axis=1, keepdims=True)
        assert (err <= 2e-2 * row_ref).all(), f"{what}: bf16 relative error {np.max(err / row_ref):.3e}"
        assert (err <= 2.0 ** -8 * np.abs(ref_out) + 1e-4).all(), f"{what}: beyond one bf16 rounding"


def lse_tol(wl):
    return 1e-5 if wl.dtype == "f32" else 1e-4


# ----------------------------------------------------------------------------- teacher-forced steps
SMALL = dict(n_heads=4, head_dim=64, grid_h=6, grid_w=8, prefix_len=5)


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("name,over,budget,steps", [
    ("tiny", dict(), None, [0, 1, 5, 16, 17, 40, 96, 97, 200, 255, 256]),
    ("tiny", dict(SMALL, win_rows_back=2, win_col_radius=1), 6, [0, 1, 8, 9, 16, 24, 25, 40, 47, 48]),
    ("xl", dict(n_seq=1, n_heads=20, grid_h=6, grid_w=12, prefix_len=17), None, [0, 3, 12, 13, 30, 36, 60, 72]),
    ("long", dict(n_seq=1, n_heads=3, grid_h=5, grid_w=16, prefix_len=9), 20, [0, 1, 16, 33, 48, 64, 80]),
])
def test_step_teacher_forced(name, over, budget, steps, layout):
    """adsa_step on the oracle's state at step s must reproduce the oracle's step: same attended
    set, same keep map and n_res, same moved rows, outputs within the float bars."""
    wl = WL.get_workload(name, **over)
    cfg = oracle_cfg(wl, budget=budget)
    q, k, v, _, snaps = replay(wl, cfg, 0, 0, max(steps), snapshots=set(steps))
    P = cfg.grid_origin
    params = params_for(wl, len(steps), cfg.cap, layout=layout)
    batch = LayerBatch(params, DEV)
    qs, kn, vn = [], [], []
    for b, s in enumerate(steps):
        load_state(batch, b, snaps[s], cfg, s)
        p = P + s - 1
        qs.append(q[p]); kn.append(k[p]); vn.append(v[p])
    batch.upload_seqs()
    qd = to_device(np.stack(qs), params.dtype, DEV)
    kd = to_device(np.stack(kn), params.dtype, DEV)
    vd = to_device(np.stack(vn), params.dtype, DEV)
    batch.step(qd, kd, vd)
    torch.cuda.synchronize()
    seqs = batch.read_seqs()
    out, lse = to_host(batch.out), batch.lse.cpu().numpy()
    sel_idx, sel_cnt = batch.sel_idx.cpu().numpy(), batch.sel_cnt.cpu().numpy()
    keep_map = batch.keep_map.cpu().numpy()
    Kd, Vd = batch.k_host(), batch.v_host()
    posd, scored = batch.pos.cpu().numpy(), rank_host(batch)
    for b, s in enumerate(steps):
        st = snaps[s].copy()
        p = P + s - 1
        ref = oracle.step(cfg, st, s, q[p], k[p], v[p])
        tag = f"{name} s={s}"
        assert seqs["status"][b] == 0, tag
        assert seqs["step"][b] == s + 1, tag
        assert sel_cnt[b] == ref["sel_idx"].size, tag
        assert np.array_equal(sel_idx[b, :sel_cnt[b]], ref["sel_idx"]), tag
        check_out(wl, out[b], ref["out"], tag)
        assert np.abs(lse[b] - ref["lse"]).max() <= lse_tol(wl), tag
        assert bool(seqs["compacted"][b]) == ref["compacted"], tag
        n = st.n_res
        if ref["compacted"]:
            km = ref["keep_map"]
            # (both sides ranked the scores of the same state plus ONE step's mass: no near-tie allowance here)
            assert np.array_equal(keep_map[b, :km.size], km), f"{tag}: keep map differs from the oracle's"
        assert seqs["n_res"][b] == n, tag
        assert np.array_equal(posd[b, :n], st.pos[:n]), tag
        assert np.array_equal(Kd[b, :n], st.K[:n]) and np.array_equal(Vd[b, :n], st.V[:n]), tag
        assert np.allclose(scored[b, :n], st.score[:n], rtol=1e-5, atol=1e-6), tag


# ----------------------------------------------------------------------------- select alone
@pytest.mark.parametrize("mode", [B.SCORE_EXT_LARGEST, B.SCORE_EXT_SMALLEST])
def test_select_bit_exact_with_ties_zeros_and_infinities(mode):
    """Eq. 4 given the same score array: indices bit-exact, lowest slot wins ties, -0 == +0,
    +-inf ordered; budgets 0, 1, mid, >= candidates; ragged batch (every sequence at its own step)."""
    rng = np.random.default_rng(123)
    wl = WL.get_workload("tiny", n_heads=1, head_dim=64, grid_h=12, grid_w=10, prefix_len=7,
                         win_rows_back=2, win_col_radius=2)
    P, HW = 7, 120
    cases = []
    for s in [0, 1, 9, 10, 11, 35, 60, 99, 120]:
        for Bud in [0, 1, 13, 500]:
            cases.append((s, Bud))
    cap = P + HW
    params = params_for(wl, len(cases), cap, score_mode=mode)
    batch = LayerBatch(params, DEV)
    refs = []
    for b, (s, Bud) in enumerate(cases):
        n = P + s
        # resident set: a random subset that still contains prefix + the rows the window needs
        keep = np.ones(n, bool)
        if s > 40:
            r = (s - 1) // 10
            old = np.arange(P, P + max(0, (r - 2)) * 10)
            keep[rng.choice(old, size=old.size // 3, replace=False)] = False
        pos = np.nonzero(keep)[0].astype(np.int32)
        score = rng.integers(-2, 3, size=pos.size).astype(np.float32) * 0.25      # heavy ties
        score[rng.random(pos.size) < 0.1] = -0.0
        score[rng.random(pos.size) < 0.05] = np.inf
        score[rng.random(pos.size) < 0.05] = -np.inf
        if b % 3 == 0:
            score = rng.standard_normal(pos.size).astype(np.float32)
        cfg = oracle_cfg(wl, budget=Bud, score_mode=mode, cap=cap)
        sel, _ = oracle.select(cfg, pos, score, None, s)
        refs.append(sel)
        z = np.zeros((pos.size, 1, 64), np.float32)
        batch.set_sequence(b, k=z, v=z, pos=pos, score=score, step=s, grid_origin=P, budget=Bud)
    batch.upload_seqs()
    batch.select()
    torch.cuda.synchronize()
    sel_idx, sel_cnt = batch.sel_idx.cpu().numpy(), batch.sel_cnt.cpu().numpy()
    assert (batch.read_seqs()["status"] == 0).all()
    for b, ref in enumerate(refs):
        assert sel_cnt[b] == ref.size, cases[b]
        assert np.array_equal(sel_idx[b, :ref.size], ref), cases[b]


def test_select_at_maximum_capacity():
    """cap = ADSA_MAX_CAP resident slots in one sequence: the LDS-resident radix select at its limit."""
    rng = np.random.default_rng(7)
    W = 90
    wl = WL.get_workload("tiny", n_heads=1, head_dim=64, grid_h=91, grid_w=W, prefix_len=2,
                         win_rows_back=1, win_col_radius=3)
    cap = B.MAX_CAP
    s = cap - 2
    pos = np.arange(cap, dtype=np.int32)
    score = (rng.integers(0, 50, size=cap) / 8.0).astype(np.float32)
    for Bud in (1, 4000, 8100):
        cfg = oracle_cfg(wl, P=2, budget=Bud, score_mode=B.SCORE_EXT_LARGEST, cap=cap)
        ref, _ = oracle.select(cfg, pos, score, None, s)
        params = params_for(wl, 1, cap, score_mode=B.SCORE_EXT_LARGEST)
        batch = LayerBatch(params, DEV)
        z = np.zeros((1, 1, 64), np.float32)
        batch.set_sequence(0, k=z[:0], v=z[:0], pos=pos[:0], score=None, step=s, grid_origin=2, budget=Bud)
        batch.pos[0] = torch.from_numpy(pos).to(DEV)
        batch.score[0] = torch.from_numpy(score).to(DEV)
        batch.seqs_host[0]["n_res"] = cap
        batch.upload_seqs()
        batch.select()
        torch.cuda.synchronize()
        cnt = int(batch.sel_cnt.cpu()[0])
        assert cnt == ref.size
        assert np.array_equal(batch.sel_idx.cpu().numpy()[0, :cnt], ref)


# ----------------------------------------------------------------------------- attend alone
@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("name,over", [
    ("tiny", dict(n_heads=16, head_dim=64)),
    ("tiny", dict(n_heads=3, head_dim=128)),
    ("xl", dict(n_heads=20, head_dim=64)),
    ("long", dict(n_heads=5, head_dim=128)),
])
def test_attend_matches_oracle_on_ragged_index_lists(name, over, layout):
    """Eq. 5 + attention for index lists of many lengths (1 .. several tiles + ragged tails),
    and the ATTN_MASS accumulation that follows it."""
    wl = WL.get_workload(name, n_seq=1, grid_h=20, grid_w=20, prefix_len=30, **over)
    rng = np.random.default_rng(5)
    q, k, v = WL.gen_tokens(wl, 0, 0)
    n_tok = k.shape[0]
    lens = [1, 2, 3, 5, 16, 17, 63, 64, 65, 127, 200, 301, 430]
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
        check_out(wl, out[b], ro, f"len={n}")
        assert np.abs(lse[b] - rl).max() <= lse_tol(wl), n
        ref_score = oracle.accumulate(cfg, score0[b], sels[b], probs)
        assert np.allclose(score[b], ref_score, rtol=1e-5, atol=1e-6), n
    # NO_ACCUMULATE leaves score[] alone
    before = batch.score.clone()
    batch.attend(qd, flags=B.FLAG_NO_ACCUMULATE)
    torch.cuda.synchronize()
    assert torch.equal(before, batch.score)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("layout,n_heads", [("head_major", 2), ("slot_major", 8)])
def test_split_lists_sixteen_chunks_many_sequences(layout, n_heads, dtype):
    """The split-list launch at its widest: 24 sequences whose lists are cut into 16 chunks each, so 16
    workgroups (on different XCDs) hand partial softmax states and logits to the one that arrives last.
    List lengths from 1 (fewer tokens than chunks) to 640; three launches in a row on the same workspace
    (every launch must leave the arrival counters at zero), the attention mass accumulating over them.
    Compared with the oracle: outputs, lse and accumulated scores, for both storage types."""
    wl = WL.get_workload("tiny", n_seq=1, n_heads=n_heads, head_dim=64, grid_h=26, grid_w=26, prefix_len=20, dtype=dtype)
    rng = np.random.default_rng(11)
    q, k, v = WL.gen_tokens(wl, 0, 0)
    n_tok = 672
    k, v = k[:n_tok], v[:n_tok]
    lens = [1, 2, 7, 15, 16, 17, 31, 33, 100, 255, 256, 257, 400, 511, 512, 513, 600, 639, 640, 640, 48, 49, 320, 5]
    cap = n_tok
    params = params_for(wl, len(lens), cap, score_mode=B.SCORE_ATTN_MASS, sel_cap=640, layout=layout)
    batch = LayerBatch(params, DEV)
    # the launch plan is the library's; what the test relies on is checked through the workspace it asks for:
    # [logits + 16 chunk partials per (sequence, head)] only exist when the lists are split 16 ways
    per_head = 640 * 4 + 16 * 2 * 4 + 16 * 64 * 4
    assert B.adsa_workspace_bytes(params) >= len(lens) * n_heads * per_head
    cfg = oracle_cfg(wl, budget=cap, cap=cap, score_mode=B.SCORE_ATTN_MASS)
    sels, scores = [], []
    sel_idx = np.full((len(lens), 640), -1, np.int32)
    for b, n in enumerate(lens):
        sel = np.sort(rng.choice(n_tok, size=n, replace=False)).astype(np.int32)
        sels.append(sel)
        sel_idx[b, :n] = sel
        sc = rng.random(n_tok).astype(np.float32)
        scores.append(sc)
        batch.set_sequence(b, k=k, v=v, pos=np.arange(n_tok, dtype=np.int32), score=sc, step=600,
                           grid_origin=20, budget=cap)
    batch.upload_seqs()
    batch.sel_idx.copy_(torch.from_numpy(sel_idx).to(DEV))
    batch.sel_cnt.copy_(torch.tensor(lens, dtype=torch.int32).to(DEV))
    for launch in range(3):
        qs = np.stack([q[50 + 30 * launch + b] for b in range(len(lens))])
        batch.attend(to_device(qs, params.dtype, DEV))
        torch.cuda.synchronize()
        out, lse, rank = to_host(batch.out), batch.lse.cpu().numpy(), rank_host(batch)
        for b, n in enumerate(lens):
            ro, rl, probs = oracle.attend(cfg, k, v, qs[b], sels[b], want_probs=True)
            check_out(wl, out[b], ro, f"launch {launch} len={n}")
            assert np.abs(lse[b] - rl).max() <= lse_tol(wl), (launch, n)
            scores[b] = oracle.accumulate(cfg, scores[b], sels[b], probs)
            assert np.allclose(rank[b], scores[b], rtol=1e-5, atol=1e-6), (launch, n)


# ----------------------------------------------------------------------------- compact alone
@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("name,over", [("tiny", dict(n_heads=2, head_dim=64)), ("xl", dict(n_heads=20, head_dim=64)),
                                       ("long", dict(n_heads=2, head_dim=128))])
def test_compact_bit_exact(name, over, layout):
    """Section 4.2 per-row eviction given the same score array: keep map, n_res and every moved
    row (K, V, pos, score) bit-exact; sequences not at a row end are untouched."""
    rng = np.random.default_rng(17)
    W, H, P = 9, 40, 11
    wl = WL.get_workload(name, n_seq=1, grid_h=H, grid_w=W, prefix_len=P, win_rows_back=2, win_col_radius=1, **over)
    q, k, v = WL.gen_tokens(wl, 0, 0)
    cases = [(W, 3), (2 * W, 0), (5 * W, 7), (20 * W, 50), (33 * W, 1000), (33 * W - 1, 5), (40 * W, 64), (7 * W, 10)]
    cap = P + H * W
    mode = B.SCORE_EXT_LARGEST
    params = params_for(wl, len(cases), cap, score_mode=mode, layout=layout)
    batch = LayerBatch(params, DEV)
    states = []
    for b, (s, Bud) in enumerate(cases):
        n = P + s
        keep = np.ones(n, bool)
        if b % 2 == 1 and s > 4 * W:
            old = np.arange(P, P + s - 3 * W)
            keep[rng.choice(old, size=old.size // 2, replace=False)] = False
        pos = np.nonzero(keep)[0].astype(np.int32)
        score = (rng.integers(0, 6, pos.size) * 0.5).astype(np.float32)
        cfg = oracle_cfg(wl, P=P, budget=Bud, score_mode=mode, cap=cap)
        st = oracle.CacheState.from_arrays(cfg, k[pos], v[pos], pos, score)
        states.append((cfg, st))
        load_state(batch, b, st, cfg, s)
    batch.upload_seqs()
    batch.compact()
    torch.cuda.synchronize()
    seqs = batch.read_seqs()
    km = batch.keep_map.cpu().numpy()
    Kd, Vd, posd, scored = batch.k_host(), batch.v_host(), batch.pos.cpu().numpy(), rank_host(batch)
    for b, (s, Bud) in enumerate(cases):
        cfg, st = states[b]
        n_old = st.n_res
        ref_map, did = oracle.compact(cfg, st, s)
        assert bool(seqs["compacted"][b]) == did, (s, Bud)
        assert seqs["n_res"][b] == st.n_res
        if did:
            assert np.array_equal(km[b, :n_old], ref_map), (s, Bud)
        else:
            assert (km[b] == -3).all()
        n = st.n_res
        assert np.array_equal(posd[b, :n], st.pos[:n]) and np.array_equal(scored[b, :n], st.score[:n])
        assert np.array_equal(Kd[b, :n], st.K[:n]) and np.array_equal(Vd[b, :n], st.V[:n])
        assert seqs["step"][b] == s


# ----------------------------------------------------------------------------- free-running Tiny
def test_tiny_free_running_trajectory():
    """The whole Tiny workload (256 decode steps, compaction every row) free-running on the GPU
    against the free-running oracle.  Scores are accumulated in fp32 on the GPU and in fp64 on
    the CPU, so the two may part ways -- but only at a near tie of the oracle's own ranking: the
    first differing attended set or eviction is checked for that, and reported with its margin."""
    wl = WL.get_workload("tiny")
    cfg = oracle_cfg(wl)
    P = cfg.grid_origin
    q, k, v = WL.gen_tokens(wl, 0, 0)
    st = oracle.CacheState.from_prefix(cfg, k[:P], v[:P])
    params = params_for(wl, 1, cfg.cap)
    batch = LayerBatch(params, DEV)
    load_state(batch, 0, st, cfg, 0)
    batch.upload_seqs()
    qd, kd, vd = (to_device(x, params.dtype, DEV) for x in (q, k, v))
    steps_ok, diverged = 0, None

    def margin(a, b, score):
        only = sorted(set(a.tolist()) ^ set(b.tolist()))
        vals = score[only].astype(np.float64)
        return float(vals.max() - vals.min()), only

    for s in range(0, wl.n_image_tokens):
        p = P + s - 1
        batch.step(qd[p:p + 1], kd[p:p + 1], vd[p:p + 1])
        score_before = np.append(st.score[:st.n_res], 0.0) if s >= 1 else st.score[:st.n_res].copy()
        ref = oracle_step_phases(cfg, st, s, q[p], k[p], v[p])
        cnt = int(batch.sel_cnt.cpu()[0])
        sel = batch.sel_idx.cpu().numpy()[0, :cnt]
        if not np.array_equal(sel, ref["sel_idx"]):
            mg, only = margin(sel, ref["sel_idx"], score_before)
            diverged = f"attended sets first differ at step {s} in slots {only}: oracle score margin {mg:.3e}"
            assert near_tie_ok(sel, ref["sel_idx"], score_before), diverged
            break
        check_out(wl, to_host(batch.out)[0], ref["out"], f"s={s}")
        seqs = batch.read_seqs()
        assert bool(seqs["compacted"][0]) == ref["compacted"], s
        if ref["compacted"]:
            km, g = ref["keep_map"], batch.keep_map.cpu().numpy()[0, :ref["keep_map"].size]
            if not np.array_equal(g, km):
                kept_g, kept_r = np.nonzero(g >= 0)[0], np.nonzero(km >= 0)[0]
                mg, only = margin(kept_g, kept_r, ref["score_ranked"])
                diverged = f"evictions first differ at step {s} in slots {only}: oracle score margin {mg:.3e}"
                assert g[kept_g].tolist() == list(range(kept_g.size)), s
                assert near_tie_ok(kept_g, kept_r, ref["score_ranked"]), diverged
                break
        assert seqs["n_res"][0] == st.n_res, s
        assert np.array_equal(batch.pos.cpu().numpy()[0, :st.n_res], st.pos[:st.n_res]), s
        steps_ok += 1
    print(f"tiny free-running: {steps_ok} of {wl.n_image_tokens} steps identical to the oracle; "
          + (diverged or "never diverged"))
    assert steps_ok >= 240          # (the committed kernels follow the oracle through all 256 steps)


# ----------------------------------------------------------------------------- device-side errors
def test_device_side_status_and_inactive_sequences():
    wl = WL.get_workload("tiny", n_heads=2, head_dim=64, grid_h=4, grid_w=4, prefix_len=3)
    q, k, v = WL.gen_tokens(wl, 0, 0)
    cap = 8
    params = params_for(wl, 4, cap, sel_cap=6)
    batch = LayerBatch(params, DEV)
    pos = np.arange(8, dtype=np.int32)
    # 0: cache full on append; 1: inactive; 2: attended set larger than sel_cap; 3: fine
    batch.set_sequence(0, k=k[:8], v=v[:8], pos=pos, score=None, step=6, grid_origin=3, budget=8)
    batch.set_sequence(1, k=k[:3], v=v[:3], pos=pos[:3], score=None, step=-1, grid_origin=3, budget=8)
    batch.set_sequence(2, k=k[:7], v=v[:7], pos=pos[:7], score=None, step=5, grid_origin=3, budget=8)
    batch.set_sequence(3, k=k[:3], v=v[:3], pos=pos[:3], score=None, step=1, grid_origin=3, budget=8)
    batch.upload_seqs()
    batch.out.fill_(7.0)
    x = to_device(np.stack([q[8], q[3], q[7], q[3]]), params.dtype, DEV)
    kn = to_device(np.stack([k[8], k[3], k[7], k[3]]), params.dtype, DEV)
    vn = to_device(np.stack([v[8], v[3], v[7], v[3]]), params.dtype, DEV)
    batch.step(x, kn, vn)
    torch.cuda.synchronize()
    seqs = batch.read_seqs()
    assert seqs["status"].tolist() == [B.SEQ_CACHE_FULL, 0, B.SEQ_SEL_OVERFLOW, 0]
    assert seqs["n_res"].tolist() == [8, 3, 7, 4]      # rejected sequences are left untouched
    assert seqs["step"].tolist() == [6, -1, 5, 2]
    out = to_host(batch.out)
    assert (out[0] == 0).all() and (out[1] == 0).all() and (out[2] == 0).all()
    cfg = oracle_cfg(wl, P=3, budget=8, cap=cap)
    st = oracle.CacheState.from_prefix(cfg, k[:3], v[:3])
    ref = oracle.step(cfg, st, 1, q[3], k[3], v[3])
    check_out(wl, out[3], ref["out"])


# ----------------------------------------------------------------------------- split-phase, all layers
def test_split_phase_steps_over_several_layers():
    """The q-independent phases batched over layers: adsa_select(PLAN_APPEND) for every layer's
    sequences at once, adsa_attend(APPEND | ADVANCE) per layer, adsa_compact(ADVANCE) for all
    layers at row ends -- free-running for 3 rows against one oracle per (layer, sequence)."""
    n_layers, n_seq = 3, 2
    wl = WL.get_workload("xl", n_seq=n_seq, n_heads=20, grid_h=5, grid_w=8, prefix_len=9, budget_num=1, budget_den=2)
    cfg = oracle_cfg(wl)
    P = cfg.grid_origin
    lp = params_for(wl, n_seq, cfg.cap)
    mb = ModelBatch(lp, n_layers, DEV)
    toks, states = {}, {}
    for l in range(n_layers):
        for b in range(n_seq):
            q, k, v = WL.gen_tokens(wl, l, b)
            toks[l, b] = (q, k, v)
            st = oracle.CacheState.from_prefix(cfg, k[:P], v[:P])
            states[l, b] = st
            load_state(mb, l * n_seq + b, st, cfg, 0)
    mb.upload_seqs()
    for s in range(0, 3 * wl.grid_w + 2):
        row_end = s >= 1 and (s - 1) % wl.grid_w == wl.grid_w - 1
        p = P + s - 1
        mb.select_all(flags=B.FLAG_PLAN_APPEND)
        for l in range(n_layers):
            qd, kd, vd = (to_device(np.stack([toks[l, b][i][p] for b in range(n_seq)]), lp.dtype, DEV) for i in range(3))
            mb.attend_layer(l, qd, kd, vd, flags=B.FLAG_APPEND | (0 if row_end else B.FLAG_ADVANCE))
        if row_end:
            mb.compact_all(flags=B.FLAG_ADVANCE)
        torch.cuda.synchronize()
        seqs = mb.read_seqs()
        out, sel_idx, sel_cnt = to_host(mb.out), mb.sel_idx.cpu().numpy(), mb.sel_cnt.cpu().numpy()
        posd = mb.pos.cpu().numpy()
        for l in range(n_layers):
            for b in range(n_seq):
                i = l * n_seq + b
                q, k, v = toks[l, b]
                st = states[l, b]
                before = st.score.copy()
                ref = oracle.step(cfg, st, s, q[p], k[p], v[p])
                tag = f"s={s} layer={l} seq={b}"
                assert seqs["status"][i] == 0 and seqs["step"][i] == s + 1, tag
                sel = sel_idx[i, :sel_cnt[i]]
                assert np.array_equal(sel, ref["sel_idx"]) or near_tie_ok(sel, ref["sel_idx"], before), tag
                check_out(wl, out[i], ref["out"], tag)
                assert seqs["n_res"][i] == st.n_res, tag
                assert np.array_equal(posd[i, :st.n_res], st.pos[:st.n_res]), tag


# ----------------------------------------------------------------------------- per-head score rows
def test_rank_is_the_sum_of_the_per_head_score_rows():
    """ATTN_MASS keeps one accumulator row per head; a slot's rank is their sum.  With rows whose
    sums are exact in fp32 (multiples of 1/8) the sum is order-free, so the oracle given the summed
    array must agree bit for bit, both for the attended set and for the keep map; compaction must
    move every row."""
    rng = np.random.default_rng(31)
    W, H, P, h = 8, 12, 6, 5
    wl = WL.get_workload("tiny", n_heads=h, head_dim=64, grid_h=H, grid_w=W, prefix_len=P, win_rows_back=1, win_col_radius=2)
    q, k, v = WL.gen_tokens(wl, 0, 0)
    cases = [(5 * W, 7), (9 * W, 20), (9 * W - 3, 11), (12 * W, 3)]
    cap = P + H * W
    params = params_for(wl, len(cases), cap, score_mode=B.SCORE_ATTN_MASS)
    batch = LayerBatch(params, DEV)
    rows_all, cfgs, poss = [], [], []
    for b, (s, Bud) in enumerate(cases):
        n = P + s
        rows = (rng.integers(0, 9, size=(h, n)) / 8.0).astype(np.float32)
        rows_all.append(rows)
        cfg = oracle_cfg(wl, P=P, budget=Bud, score_mode=B.SCORE_ATTN_MASS, cap=cap)
        cfgs.append(cfg)
        pos = np.arange(n, dtype=np.int32)
        poss.append(pos)
        batch.set_sequence(b, k=k[:n], v=v[:n], pos=pos, score=rows, step=s, grid_origin=P, budget=Bud)
    batch.upload_seqs()
    batch.select()
    batch.compact()
    torch.cuda.synchronize()
    sel_idx, sel_cnt, km = batch.sel_idx.cpu().numpy(), batch.sel_cnt.cpu().numpy(), batch.keep_map.cpu().numpy()
    score_rows = batch.score.cpu().numpy()
    seqs = batch.read_seqs()
    for b, (s, Bud) in enumerate(cases):
        total = rows_all[b].sum(axis=0, dtype=np.float32)
        ref_sel, _ = oracle.select(cfgs[b], poss[b], total, None, s)
        assert np.array_equal(sel_idx[b, :sel_cnt[b]], ref_sel), (s, Bud)
        n = P + s
        st = oracle.CacheState.from_arrays(cfgs[b], k[:n], v[:n], poss[b], total)
        ref_map, did = oracle.compact(cfgs[b], st, s)
        assert bool(seqs["compacted"][b]) == did
        if did:
            assert np.array_equal(km[b, :n], ref_map)
            kept = np.nonzero(ref_map >= 0)[0]
            assert np.array_equal(score_rows[b, :, :kept.size], rows_all[b][:, kept])


@pytest.mark.parametrize("n_seq,h", [(6, 3), (6, 11), (6, 26), (520, 3), (520, 11), (520, 26)])
def test_ranking_kernels_at_both_launch_sizes(n_seq, h):
    """The ranking kernels fetch the score rows of one slot (launches of >= 512 sequences) or of four slots
    (smaller launches) at a time, eight rows per batch: both forms, with 3, 11 and 26 score rows (one partial batch,
    two, four), against the oracle given the summed array.  Row sums are exact in fp32, so the sum is order-free:
    attended sets, keep maps and moved score rows bit for bit."""
    rng = np.random.default_rng(1000 * n_seq + h)
    W, H, P = 6, 9, 5
    wl = WL.get_workload("tiny", n_heads=h, head_dim=64, grid_h=H, grid_w=W, prefix_len=P, win_rows_back=1, win_col_radius=1)
    q, k, v = WL.gen_tokens(wl, 0, 0)
    cap = P + H * W
    params = params_for(wl, n_seq, cap, score_mode=B.SCORE_ATTN_MASS)
    batch = LayerBatch(params, DEV)
    cases = []
    for b in range(n_seq):
        s = int(rng.integers(1, H * W + 1)) if b % 3 else W * int(rng.integers(1, H + 1))      # a third at row ends
        Bud = int(rng.integers(0, 12))
        n = P + s
        rows = (rng.integers(0, 5, size=(h, n)) / 8.0).astype(np.float32)
        cfg = oracle_cfg(wl, P=P, budget=Bud, score_mode=B.SCORE_ATTN_MASS, cap=cap)
        pos = np.arange(n, dtype=np.int32)
        cases.append((s, Bud, rows, cfg, pos))
        batch.set_sequence(b, k=k[:n], v=v[:n], pos=pos, score=rows, step=s, grid_origin=P, budget=Bud)
    batch.upload_seqs()
    batch.select()
    batch.compact()
    torch.cuda.synchronize()
    sel_idx, sel_cnt, km = batch.sel_idx.cpu().numpy(), batch.sel_cnt.cpu().numpy(), batch.keep_map.cpu().numpy()
    score_rows, posd = batch.score.cpu().numpy(), batch.pos.cpu().numpy()
    seqs = batch.read_seqs()
    assert (seqs["status"] == 0).all()
    n_compacted = 0
    for b, (s, Bud, rows, cfg, pos) in enumerate(cases):
        total = rows.sum(axis=0, dtype=np.float32)
        ref_sel, _ = oracle.select(cfg, pos, total, None, s)
        assert sel_cnt[b] == ref_sel.size and np.array_equal(sel_idx[b, :sel_cnt[b]], ref_sel), (b, s, Bud)
        n = P + s
        st = oracle.CacheState.from_arrays(cfg, k[:n], v[:n], pos, total)
        ref_map, did = oracle.compact(cfg, st, s)
        assert bool(seqs["compacted"][b]) == did and seqs["n_res"][b] == st.n_res, (b, s, Bud)
        if did:
            n_compacted += 1
            assert np.array_equal(km[b, :n], ref_map), (b, s, Bud)
            kept = np.nonzero(ref_map >= 0)[0]
            assert np.array_equal(score_rows[b, :, :kept.size], rows[:, kept]), (b, s, Bud)
            assert np.array_equal(posd[b, :kept.size], pos[kept]), (b, s, Bud)
    assert n_compacted >= n_seq // 4


# ----------------------------------------------------------------------------- TopK-V (Eq. 2-4) on the GPU
def vcos_close(gpu, ref):
    """fp32 two-pass closed form vs the fp64 pairwise definition: |S| <= 1, sums of up to ~1e3 unit
    vectors of dimension up to 4096 in fp32 -> absolute error ~1e-7; bar 2e-6 + 1e-4 relative."""
    return np.allclose(gpu, ref, rtol=1e-4, atol=2e-6)


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("name,over,budget,steps", [
    ("tiny", dict(n_heads=4, head_dim=64, grid_h=8, grid_w=8, prefix_len=6), 9, [0, 1, 9, 24, 25, 40, 63, 64]),
    ("xl", dict(n_seq=1, n_heads=20, grid_h=6, grid_w=12, prefix_len=17, budget_num=0, budget_den=0), 21, [13, 36, 37, 60, 72]),
    ("long", dict(n_seq=1, n_heads=3, grid_h=5, grid_w=16, prefix_len=9), 12, [17, 48, 64, 80]),
    # wide concatenated V rows: 1792, 4096 and 8192 columns (7, 16 and 32 column groups per lane; the
    # widest needs more LDS than a launch gets by default)
    ("tiny", dict(n_heads=28, head_dim=64, grid_h=4, grid_w=6, prefix_len=3), 5, [7, 12, 13, 24]),
    ("long", dict(n_seq=1, n_heads=32, head_dim=128, grid_h=4, grid_w=6, prefix_len=3), 5, [7, 12, 13, 24]),
    ("long", dict(n_seq=1, n_heads=64, head_dim=128, grid_h=4, grid_w=6, prefix_len=3), 5, [12, 13, 24]),
])
def test_vcos_step_teacher_forced(name, over, budget, steps, layout):
    """The paper's own ranking: mean pairwise V-cosine over the candidates (Eq. 2-3), keep the K
    lowest (Eq. 4), evict the most redundant at row ends (Section 4.2).  Scores within the float
    bar of the O(N^2 D) definition; the attended set and the keep map equal the oracle's, or differ
    only among candidates whose oracle scores tie within that bar."""
    wl = WL.get_workload(name, score_mode=WL.SCORE_VCOS, **over)
    cfg = oracle_cfg(wl, budget=budget, score_mode=WL.SCORE_VCOS)
    q, k, v, _, snaps = replay(wl, cfg, 0, 0, max(steps), snapshots=set(steps))
    P = cfg.grid_origin
    params = params_for(wl, len(steps), cfg.cap, score_mode=B.SCORE_VCOS, layout=layout)
    batch = LayerBatch(params, DEV)
    qs, kn, vn = [], [], []
    for b, s in enumerate(steps):
        load_state(batch, b, snaps[s], cfg, s)
        p = P + s - 1
        qs.append(q[p]); kn.append(k[p]); vn.append(v[p])
    batch.upload_seqs()
    qd, kd, vd = (to_device(np.stack(x), params.dtype, DEV) for x in (qs, kn, vn))
    batch.select(flags=B.FLAG_PLAN_APPEND)            # phase 1: scores + attended set
    torch.cuda.synchronize()
    score_sel = rank_host(batch)
    sel_idx, sel_cnt = batch.sel_idx.cpu().numpy(), batch.sel_cnt.cpu().numpy()
    batch.attend(qd, flags=B.FLAG_APPEND, k_new=kd, v_new=vd)
    batch.compact(flags=B.FLAG_ADVANCE)
    torch.cuda.synchronize()
    seqs = batch.read_seqs()
    out, keep_map, posd = to_host(batch.out), batch.keep_map.cpu().numpy(), batch.pos.cpu().numpy()
    for b, s in enumerate(steps):
        st = snaps[s].copy()
        p = P + s - 1
        tag = f"{name} s={s}"
        # oracle, phase by phase on the same state
        n0 = st.n_res
        if s >= 1:
            st.K[n0], st.V[n0], st.pos[n0], st.score[n0] = k[p], v[p], P + s - 1, 0.0
            st.n_res = n0 + 1
        ref_sel, ref_score = oracle.select(cfg, st.pos[:st.n_res], st.score[:st.n_res], st.V[:st.n_res], s)
        cls = oracle.classify(cfg, st.pos[:st.n_res], s)
        cand = np.nonzero(cls == oracle.CANDIDATE)[0]
        assert vcos_close(score_sel[b, cand], ref_score[cand]), tag
        sel = sel_idx[b, :sel_cnt[b]]
        assert sel.size == ref_sel.size, tag
        assert near_tie_ok(sel, ref_sel, ref_score, rel=1e-4, abs_tol=4e-6), tag
        if np.array_equal(sel, ref_sel):
            ro, _ = oracle.attend(cfg, st.K, st.V, q[p], ref_sel)
            check_out(wl, out[b], ro, tag)
        st.score[:st.n_res] = ref_score
        before = st.copy()
        ref_map, did = oracle.compact(cfg, st, s)
        assert bool(seqs["compacted"][b]) == did, tag
        assert seqs["step"][b] == s + 1 and seqs["n_res"][b] == st.n_res, tag
        if did:
            gm = keep_map[b, :ref_map.size]
            kept_g, kept_r = np.nonzero(gm >= 0)[0], np.nonzero(ref_map >= 0)[0]
            assert gm[kept_g].tolist() == list(range(kept_g.size)), tag
            assert near_tie_ok(kept_g, kept_r, before.score, rel=1e-4, abs_tol=4e-6), tag
            if np.array_equal(kept_g, kept_r):
                assert np.array_equal(posd[b, :st.n_res], st.pos[:st.n_res]), tag


# ----------------------------------------------------------------------------- full-size launches
def _full_layer(wl_name, steps, layout="head_major"):
    """One layer of a full-size workload in the launch configuration the benchmark times: every
    sequence at decode step `steps[b]`, legal synthetic states, split-phase calls."""
    wl = WL.get_workload(wl_name)
    n = wl.n_seq
    cap = 120 + 512 + 2 * wl.grid_w if wl.ragged else wl.cap()
    sel_cap = 120 + 512 + wl.grid_w + wl.win_rows_back * (2 * wl.win_col_radius + 1) if wl.ragged else wl.sel_cap()
    params = params_for(wl, n, cap, sel_cap=sel_cap, layout=layout)
    batch = LayerBatch(params, DEV)
    items = []
    for b in range(n):
        P, Bud, s_r = WL.seq_geometry(wl, b)
        if wl.budget_den > 0 and not wl.ragged:
            Bud = None                                  # fractional budget: floor((P + s) * num / den) on both sides
        s = s_r if wl.ragged else steps[b % len(steps)]
        syn = WL.synthetic_state(wl, 0, b, s, prefix_len=P, budget=Bud)
        cfg = oracle_cfg(wl, P=P, budget=Bud, cap=cap)
        st = oracle.CacheState.from_arrays(cfg, syn["k"], syn["v"], syn["pos"], syn["score"])
        load_state(batch, b, st, cfg, s)
        items.append((cfg, st, s, syn))
    batch.upload_seqs()
    qd = to_device(np.stack([it[3]["q"] for it in items]), params.dtype, DEV)
    kd = to_device(np.stack([it[3]["k_new"] for it in items]), params.dtype, DEV)
    vd = to_device(np.stack([it[3]["v_new"] for it in items]), params.dtype, DEV)
    return wl, params, batch, items, qd, kd, vd


def _check_full_step(wl, batch, items):
    seqs = batch.read_seqs()
    out, lse = to_host(batch.out), batch.lse.cpu().numpy()
    sel_idx, sel_cnt = batch.sel_idx.cpu().numpy(), batch.sel_cnt.cpu().numpy()
    keep_map, posd, rank = batch.keep_map.cpu().numpy(), batch.pos.cpu().numpy(), rank_host(batch)
    Kd, Vd = batch.k_host(), batch.v_host()
    n_compacted = 0
    for b, (cfg, st, s, syn) in enumerate(items):
        tag = f"{wl.name} seq={b} s={s}"
        ref = oracle_step_phases(cfg, st, s, syn["q"], syn["k_new"], syn["v_new"])
        assert seqs["status"][b] == 0 and seqs["step"][b] == s + 1, tag
        assert np.array_equal(sel_idx[b, :sel_cnt[b]], ref["sel_idx"]), tag          # same score array: bit-exact
        check_out(wl, out[b], ref["out"], tag)
        assert np.abs(lse[b] - ref["lse"]).max() <= lse_tol(wl), tag
        assert bool(seqs["compacted"][b]) == ref["compacted"], tag
        n = st.n_res
        assert seqs["n_res"][b] == n, tag
        if ref["compacted"]:
            n_compacted += 1
            km = ref["keep_map"]
            g = keep_map[b, :km.size]
            if not np.array_equal(g, km):
                # ranks were accumulated in fp32 on the GPU: only near-ties (by the oracle's scores) may differ
                assert near_tie_ok(np.nonzero(g >= 0)[0], np.nonzero(km >= 0)[0], ref["score_ranked"], rel=1e-5), tag
                continue
        assert np.array_equal(posd[b, :n], st.pos[:n]), tag
        assert np.array_equal(Kd[b, :n], st.K[:n]) and np.array_equal(Vd[b, :n], st.V[:n]), tag
        assert np.allclose(rank[b, :n], st.score[:n], rtol=1e-5, atol=1e-6), tag
    return n_compacted


def test_full_size_xxl_layer():
    """LlamaGen-XXL-shaped layer (32 sequences x 24 heads x 64, bf16, cap 696): deep steps incl. a
    row end, every sequence checked against the oracle (selection bit-exact, float bars)."""
    wl, params, batch, items, qd, kd, vd = _full_layer("xxl", steps=[1000, 992, 1024, 513, 33, 960, 1, 700])
    batch.select(flags=B.FLAG_PLAN_APPEND)
    batch.attend(qd, flags=B.FLAG_APPEND, k_new=kd, v_new=vd)
    batch.compact(flags=B.FLAG_ADVANCE)
    torch.cuda.synchronize()
    assert _check_full_step(wl, batch, items) >= 8


def test_full_size_xl_layer():
    """LlamaGen-XL-shaped layer (16 sequences x 20 heads x 64, bf16, 24x24 grid, prefix 120, budget = half the
    current context): early, middle and deepest steps incl. three row ends (the last one is the final token),
    every sequence checked against the oracle (selection bit-exact, float bars)."""
    wl, params, batch, items, qd, kd, vd = _full_layer("xl", steps=[576, 552, 575, 300, 25, 24, 1, 0, 289, 480, 100, 333])
    assert wl.budget_den > 0 and params.cap == wl.cap()
    batch.select(flags=B.FLAG_PLAN_APPEND)
    batch.attend(qd, flags=B.FLAG_APPEND, k_new=kd, v_new=vd)
    batch.compact(flags=B.FLAG_ADVANCE)
    torch.cuda.synchronize()
    assert _check_full_step(wl, batch, items) >= 4


@pytest.mark.parametrize("layout", LAYOUTS)
def test_ragged_serving_batch_in_one_step_call(layout):
    """64 sequences, each at its own decode position, budget and prefix length, in ONE adsa_step."""
    wl, params, batch, items, qd, kd, vd = _full_layer("ragged", steps=None, layout=layout)
    batch.step(qd, kd, vd)
    torch.cuda.synchronize()
    _check_full_step(wl, batch, items)


def test_full_size_long_context_layer():
    """64x64 grid, 32 heads x 128, bf16, budget 1024, R = 2: the split-list launch (few sequences)."""
    wl, params, batch, items, qd, kd, vd = _full_layer("long", steps=[4096, 4032, 2049, 130])
    batch.step(qd, kd, vd)
    torch.cuda.synchronize()
    _check_full_step(wl, batch, items)


# ----------------------------------------------------------------------------- degenerate shapes
@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("geom", [
    dict(grid_h=6, grid_w=1, prefix_len=3, win_rows_back=1, win_col_radius=0, budget=2),    # every step closes a row
    dict(grid_h=1, grid_w=9, prefix_len=2, win_rows_back=1, win_col_radius=1, budget=3),    # a single row
    dict(grid_h=4, grid_w=5, prefix_len=0, win_rows_back=0, win_col_radius=0, budget=4),    # no prefix, no previous rows
    dict(grid_h=3, grid_w=4, prefix_len=5, win_rows_back=3, win_col_radius=9, budget=0),    # window wider than the grid, B = 0
    dict(grid_h=1, grid_w=1, prefix_len=1, win_rows_back=1, win_col_radius=1, budget=1),    # one image token
])
def test_degenerate_grids_free_running(geom, layout):
    """Whole free-running trajectories on degenerate geometries (1-wide grids, one row, empty prefix
    so the cache starts EMPTY, zero budget, window larger than the grid) through adsa_step."""
    geom = dict(geom)
    budget = geom.pop("budget")
    wl = WL.get_workload("tiny", n_heads=3, head_dim=64, **geom)
    P = wl.prefix_len
    cfg = oracle_cfg(wl, budget=budget, score_mode=B.SCORE_EXT_LARGEST)   # fixed scores: no fp-dependent ranking
    q, k, v = WL.gen_tokens(wl, 0, 0)
    st = oracle.CacheState.from_prefix(cfg, k[:P], v[:P])
    rng = np.random.default_rng(1)
    params = params_for(wl, 1, cfg.cap, score_mode=B.SCORE_EXT_LARGEST, layout=layout)
    batch = LayerBatch(params, DEV)
    s0 = 0 if P > 0 else 1
    load_state(batch, 0, st, cfg, s0)
    batch.upload_seqs()
    qd, kd, vd = (to_device(x, params.dtype, DEV) for x in (q, k, v))
    for s in range(s0, wl.n_image_tokens + 1):
        p = P + s - 1
        batch.step(qd[p:p + 1], kd[p:p + 1], vd[p:p + 1])
        ref = oracle.step(cfg, st, s, q[p], k[p], v[p])
        torch.cuda.synchronize()
        seqs = batch.read_seqs()
        assert seqs["status"][0] == 0 and seqs["step"][0] == s + 1 and seqs["n_res"][0] == st.n_res, s
        cnt = int(batch.sel_cnt.cpu()[0])
        assert np.array_equal(batch.sel_idx.cpu().numpy()[0, :cnt], ref["sel_idx"]), s
        check_out(wl, to_host(batch.out)[0], ref["out"], f"s={s}")
        assert np.array_equal(batch.pos.cpu().numpy()[0, :st.n_res], st.pos[:st.n_res]), s
        assert np.array_equal(batch.k_host()[0, :st.n_res], st.K[:st.n_res]), s
        # give the slots fresh external scores so that later evictions have something to rank
        new_scores = (rng.integers(0, 4, st.n_res) / 2.0).astype(np.float32)
        st.score[:st.n_res] = new_scores
        batch.score[0, 0, :st.n_res] = torch.from_numpy(new_scores).to(DEV)


@pytest.mark.parametrize("layout", LAYOUTS)
def test_attend_on_a_maximum_length_list(layout):
    """One sequence attending cap = ADSA_MAX_CAP slots (list split into the maximum number of chunks)."""
    wl = WL.get_workload("tiny", n_heads=2, head_dim=64, grid_h=91, grid_w=90, prefix_len=2)
    rng = np.random.default_rng(3)
    n = B.MAX_CAP
    k = (rng.standard_normal((n, 2, 64)) / 8).astype(np.float32)
    v = rng.standard_normal((n, 2, 64)).astype(np.float32)
    q = rng.standard_normal((2, 64)).astype(np.float32)
    params = params_for(wl, 1, n, score_mode=B.SCORE_ATTN_MASS, layout=layout)
    batch = LayerBatch(params, DEV)
    batch.set_sequence(0, k=k, v=v, pos=np.arange(n, dtype=np.int32), score=None, step=n - 2, grid_origin=2, budget=n)
    batch.upload_seqs()
    batch.sel_idx[0] = torch.arange(n, dtype=torch.int32, device=DEV)
    batch.sel_cnt[0] = n
    batch.attend(to_device(q[None], params.dtype, DEV))
    torch.cuda.synchronize()
    cfg = oracle_cfg(wl, P=2, budget=n, cap=n)
    ro, rl, probs = oracle.attend(cfg, k, v, q, np.arange(n, dtype=np.int32), want_probs=True)
    check_out(wl, to_host(batch.out)[0], ro)
    assert np.abs(batch.lse.cpu().numpy()[0] - rl).max() <= 1e-5
    assert np.allclose(rank_host(batch)[0], probs.sum(axis=0), rtol=1e-5, atol=1e-7)


# ----------------------------------------------------------------------------- Section 4.2 as written
@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("mode", [B.SCORE_VCOS, B.SCORE_ATTN_MASS])
def test_streaming_cache_evict_one_when_full(mode, layout):
    """The paper's own cache policy: fixed capacity, 1-D window of the m most recent tokens, dense
    attention over everything resident, and once full the single most redundant candidate is evicted
    before each insertion.  Teacher-forced adsa_step on oracle states before, at and after the cache
    fills up."""
    P, H, W, m, cap = 5, 8, 8, 6, 30
    wl = WL.get_workload("xl", n_seq=1, n_heads=4, head_dim=64, grid_h=H, grid_w=W, prefix_len=P, score_mode=mode)
    cfg = oracle.make_cfg(n_heads=4, head_dim=64, grid_h=H, grid_w=W, win_rows_back=0, win_col_radius=0,
                          grid_origin=P, budget=10 ** 6, score_mode=mode, cap=cap, win_recent_m=m, evict_when_full=1)
    steps = [0, 1, 24, 25, 26, 27, 40, 63, 64]
    q, k, v, _, snaps = replay(wl, cfg, 0, 0, max(steps), snapshots=set(steps))
    params = B.make_params(n_seq=len(steps), n_heads=4, head_dim=64, grid_h=H, grid_w=W, win_rows_back=0,
                           win_col_radius=0, dtype=B.BF16, score_mode=mode, cap=cap, layout=layout,
                           win_recent_m=m, evict_policy=B.EVICT_WHEN_FULL)
    batch = LayerBatch(params, DEV)
    for b, s in enumerate(steps):
        load_state(batch, b, snaps[s], cfg, s)
    batch.upload_seqs()
    pp = [P + s - 1 for s in steps]
    qd, kd, vd = (to_device(np.stack([x[p] for p in pp]), params.dtype, DEV) for x in (q, k, v))
    batch.step(qd, kd, vd)
    torch.cuda.synchronize()
    seqs = batch.read_seqs()
    out, keep_map = to_host(batch.out), batch.keep_map.cpu().numpy()
    sel_idx, sel_cnt, posd = batch.sel_idx.cpu().numpy(), batch.sel_cnt.cpu().numpy(), batch.pos.cpu().numpy()
    Kd = batch.k_host()
    n_evictions = 0
    for b, s in enumerate(steps):
        st = snaps[s].copy()
        n_before = st.n_res
        score_before = st.score.copy()
        ref = oracle.step(cfg, st, s, q[pp[b]], k[pp[b]], v[pp[b]])
        tag = f"mode={mode} s={s}"
        assert seqs["status"][b] == 0 and seqs["step"][b] == s + 1 and seqs["n_res"][b] == st.n_res, tag
        assert bool(seqs["compacted"][b]) == ref["compacted"], tag
        same = True
        if ref["compacted"]:
            n_evictions += 1
            g, r = keep_map[b, :n_before], ref["keep_map"]
            assert (g < 0).sum() == 1, tag
            if not np.array_equal(g, r):
                same = False        # only a near tie between the two evicted candidates is acceptable
                if mode == B.SCORE_VCOS:
                    cls = oracle.classify(cfg, snaps[s].pos[:n_before], s)
                    cand = np.nonzero(cls == oracle.CANDIDATE)[0]
                    sc = np.zeros(n_before)
                    sc[cand] = oracle.vcos(cfg, snaps[s].V, cand)
                else:
                    sc = score_before[:n_before].astype(np.float64)
                assert near_tie_ok(np.nonzero(g >= 0)[0], np.nonzero(r >= 0)[0], sc, rel=1e-4, abs_tol=4e-6), tag
        if same:
            assert sel_cnt[b] == st.n_res and np.array_equal(sel_idx[b, :sel_cnt[b]], ref["sel_idx"]), tag
            check_out(wl, out[b], ref["out"], tag)
            assert np.array_equal(posd[b, :st.n_res], st.pos[:st.n_res]), tag
            assert np.array_equal(Kd[b, :st.n_res], st.K[:st.n_res]), tag
    assert n_evictions == 5


@pytest.mark.parametrize("mode,layout", [(B.SCORE_VCOS, "head_major"), (B.SCORE_VCOS, "slot_major"),
                                         (B.SCORE_ATTN_MASS, "head_major"), (B.SCORE_ATTN_MASS, "slot_major"),
                                         (B.SCORE_VCOS_FUSED, "head_major")])
def test_streaming_cache_slot_reuse_free_running(mode, layout):
    """ADSA_EVICT_REUSE_SLOT: same rule and same victim as the order-preserving form, but the incoming
    token takes the evicted slot and nothing moves.  Free-running over a whole trajectory (59 evictions)
    against the free-running oracle: the caches must hold the same tokens -- compared by position, since
    slot order differs -- with identical rows, and every step's output must match.
    ADSA_SCORE_VCOS_FUSED is the same ranking (oracle: VCOS) computed inside the attention launch from the
    running sum u; its first eviction falls back to the two-pass form, all later ones use the fused numbers."""
    omode = B.SCORE_VCOS if mode == B.SCORE_VCOS_FUSED else mode
    P, H, W, m, cap = 5, 8, 8, 6, 30
    wl = WL.get_workload("xl", n_seq=1, n_heads=4, head_dim=64, grid_h=H, grid_w=W, prefix_len=P, score_mode=omode)
    cfg = oracle.make_cfg(n_heads=4, head_dim=64, grid_h=H, grid_w=W, win_rows_back=0, win_col_radius=0,
                          grid_origin=P, budget=10 ** 6, score_mode=omode, cap=cap, win_recent_m=m, evict_when_full=1)
    q, k, v = WL.gen_tokens(wl, 0, 0, prefix_len=P)
    st = oracle.CacheState.from_prefix(cfg, k[:P], v[:P])
    params = B.make_params(n_seq=1, n_heads=4, head_dim=64, grid_h=H, grid_w=W, win_rows_back=0,
                           win_col_radius=0, dtype=B.BF16, score_mode=mode, cap=cap, layout=layout,
                           win_recent_m=m, evict_policy=B.EVICT_REUSE_SLOT)
    batch = LayerBatch(params, DEV)
    load_state(batch, 0, st, cfg, 0)
    batch.upload_seqs()
    qd, kd, vd = (to_device(x, params.dtype, DEV) for x in (q, k, v))
    n_evictions = 0
    for s in range(0, H * W + 1):
        p = P + s - 1
        before = st.copy()
        batch.step(qd[p:p + 1], kd[p:p + 1], vd[p:p + 1])
        ref = oracle.step(cfg, st, s, q[p], k[p], v[p])
        torch.cuda.synchronize()
        seqs = batch.read_seqs()
        tag = f"mode={mode} s={s}"
        n = st.n_res
        assert seqs["status"][0] == 0 and seqs["step"][0] == s + 1 and seqs["n_res"][0] == n, tag
        assert seqs["hole"][0] == 0 and bool(seqs["compacted"][0]) == ref["compacted"], tag
        n_evictions += int(ref["compacted"])
        posd = batch.pos.cpu().numpy()[0, :n]
        if set(posd.tolist()) != set(st.pos[:n].tolist()):
            # a different victim is acceptable only where the oracle's own scores of the two victims tie
            # (GPU ranks fp32-accumulated mass, the oracle fp64)
            only_g = sorted(set(posd.tolist()) - set(st.pos[:n].tolist()))
            only_o = sorted(set(st.pos[:n].tolist()) - set(posd.tolist()))
            assert mode == B.SCORE_ATTN_MASS and len(only_g) == 1 and len(only_o) == 1, tag
            nb = before.n_res
            sc = before.score[:nb].astype(np.float64)
            a_ = sc[np.nonzero(before.pos[:nb] == only_g[0])[0][0]]      # the oracle evicted this one
            b_ = sc[np.nonzero(before.pos[:nb] == only_o[0])[0][0]]      # the GPU evicted this one
            print(f"{tag}: victims differ (positions {only_g[0]} / {only_o[0]}), oracle scores {a_:.7g} / {b_:.7g}")
            assert abs(a_ - b_) <= 4e-6 + 1e-4 * max(abs(a_), abs(b_)), tag
            break
        order = np.argsort(posd)                         # GPU slots in position order = the oracle's order
        assert np.array_equal(posd[order], st.pos[:n]), tag
        assert np.array_equal(batch.k_host()[0, :n][order], st.K[:n]), tag
        assert np.array_equal(batch.v_host()[0, :n][order], st.V[:n]), tag
        if mode == B.SCORE_ATTN_MASS:
            assert np.allclose(rank_host(batch)[0, :n][order], st.score[:n], rtol=1e-5, atol=1e-6), tag
        cnt = int(batch.sel_cnt.cpu()[0])
        assert cnt == n and np.array_equal(batch.sel_idx.cpu().numpy()[0, :cnt], np.arange(n)), tag
        check_out(wl, to_host(batch.out)[0], ref["out"], tag)
        if ref["compacted"]:
            km = batch.keep_map.cpu().numpy()[0, :cap]
            assert (km < 0).sum() == 1 and np.array_equal(km[km >= 0], np.nonzero(km >= 0)[0]), tag
        if mode == B.SCORE_VCOS_FUSED and s < H * W:
            # the running state: tagged for the next step, and u = sum of the next step's candidates' unit V
            state = batch.vcos_u.cpu().numpy()[0]
            dim = 4 * 64
            assert state[dim] == s + 2 and state[dim + 1] == s + 2, tag
            cls = oracle.classify(cfg, st.pos[:n], s + 1)
            rows = st.V[:n][cls == oracle.CANDIDATE].reshape(-1, dim).astype(np.float64)
            want = (rows / np.maximum(np.linalg.norm(rows, axis=1, keepdims=True), 1e-8)).sum(axis=0) if len(rows) else np.zeros(dim)
            assert np.allclose(state[:dim], want, atol=2e-5), tag
    assert n_evictions >= 21


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("G", [1, 4])
def test_append_rounds_fp32_rows_into_a_bf16_cache(G, layout):
    """ADSA_FLAG_NEW_F32: k_new / v_new arrive as fp32, the cache is bf16.  The rows must enter the cache
    rounded to nearest-even (compared bit for bit with the host rounding the oracle's inputs use) and the
    step must equal the oracle's step on the rounded rows."""
    over = dict(n_heads=4, head_dim=64, grid_h=6, grid_w=8, prefix_len=5, win_rows_back=1, win_col_radius=1,
                dtype="bf16", q_per_kv=G)
    wl = WL.get_workload("xl", n_seq=1, budget=6, budget_num=0, budget_den=0, **over)
    cfg = oracle_cfg(wl, budget=6)
    steps = [1, 7, 8, 9, 20, 48]
    q, k, v, _, snaps = replay(wl, cfg, 0, 0, max(steps), snapshots=set(steps))
    P = cfg.grid_origin
    rng = np.random.default_rng(77)
    # unrounded fp32 rows for the new tokens (values with low mantissa bits set, incl. exact ties of the rounding)
    k32 = rng.standard_normal((len(steps), wl.n_heads, wl.head_dim)).astype(np.float32)
    v32 = rng.standard_normal((len(steps), wl.n_heads, wl.head_dim)).astype(np.float32)
    k32[:, 0, :4] = np.array([1.00390625, 1.01171875, -1.00390625, 3.0e-39], np.float32)   # ties to even, a subnormal
    params = params_for(wl, len(steps), cfg.cap, layout=layout)
    batch = LayerBatch(params, DEV)
    for b, s in enumerate(steps):
        load_state(batch, b, snaps[s], cfg, s)
    batch.upload_seqs()
    pp = [P + s - 1 for s in steps]
    qd = to_device(np.stack([q[p] for p in pp]), params.dtype, DEV)
    kd, vd = torch.from_numpy(k32).to(DEV), torch.from_numpy(v32).to(DEV)
    batch.step(qd, kd, vd, flags=B.FLAG_NEW_F32)
    torch.cuda.synchronize()
    seqs = batch.read_seqs()
    out, lse = to_host(batch.out), batch.lse.cpu().numpy()
    Kd, Vd = batch.k_host(), batch.v_host()
    kr, vr = WL.round_to_bf16(k32), WL.round_to_bf16(v32)
    for b, s in enumerate(steps):
        st = snaps[s].copy()
        ref = oracle.step(cfg, st, s, q[pp[b]], kr[b], vr[b])
        tag = f"G={G} s={s}"
        n = st.n_res
        assert seqs["status"][b] == 0 and seqs["n_res"][b] == n, tag
        assert np.array_equal(Kd[b, :n], st.K[:n]) and np.array_equal(Vd[b, :n], st.V[:n]), tag   # rounded rows, bit for bit
        check_out(wl, out[b], ref["out"], tag)
        assert np.abs(lse[b] - ref["lse"]).max() <= lse_tol(wl), tag


# ----------------------------------------------------------------------------- per-head attended sets
@pytest.mark.parametrize("layout", LAYOUTS)
def test_per_head_selection_through_sel_groups(layout):
    """sel_groups = n_heads as an ABI value: the caller keeps its [n_seq][heads] view of q / out and of either cache
    nesting and passes one record per (sequence, head).  Free-running against one single-head oracle per
    (sequence, head), row-end evictions included; the cache rows are compared at the end."""
    n_seq, h, D = 2, 4, 64
    geom = dict(n_seq=1, head_dim=D, grid_h=5, grid_w=6, prefix_len=4, win_rows_back=1, win_col_radius=1,
                budget=5, budget_num=0, budget_den=0)
    wl = WL.get_workload("xl", n_heads=h, **geom)
    wl1 = WL.get_workload("xl", n_heads=1, **geom)
    cfg = oracle_cfg(wl1, budget=5)
    P, cap = 4, cfg.cap
    toks = [WL.gen_tokens(wl, 0, b) for b in range(n_seq)]
    # records, pos, score, lists: those of n_seq * h one-head sequences
    batch = LayerBatch(params_for(wl1, n_seq * h, cap), DEV)
    states = {}
    for b in range(n_seq):
        for hd in range(h):
            q, k, v = toks[b]
            states[b, hd] = oracle.CacheState.from_prefix(cfg, k[:P, hd:hd + 1], v[:P, hd:hd + 1])
            load_state(batch, b * h + hd, states[b, hd], cfg, 0)
    params = params_for(wl, n_seq, cap, layout=layout)
    params.sel_groups = h
    elem = batch.K.element_size()
    if layout == "slot_major":       # the caller's cache is [n_seq][slot][head][D]: point every record into it
        K = batch.K.reshape(n_seq, h, cap, D).transpose(1, 2).contiguous()
        V = batch.V.reshape(n_seq, h, cap, D).transpose(1, 2).contiguous()
        for b in range(n_seq):
            for hd in range(h):
                batch.seqs_host[b * h + hd]["k"] = K.data_ptr() + ((b * cap * h) + hd) * D * elem
                batch.seqs_host[b * h + hd]["v"] = V.data_ptr() + ((b * cap * h) + hd) * D * elem
    else:                            # [n_seq][head][slot][D] is the memory LayerBatch allocated
        K, V = batch.K.reshape(n_seq, h, cap, D), batch.V.reshape(n_seq, h, cap, D)
    batch.upload_seqs()
    assert B.adsa_workspace_bytes(params) == batch.workspace.numel()
    out = torch.zeros((n_seq, h, D), dtype=batch.tdtype, device=DEV)
    for s in range(0, wl.n_image_tokens):
        p = P + s - 1
        qd, kd, vd = (to_device(np.stack([toks[b][i][p] for b in range(n_seq)]), params.dtype, DEV) for i in range(3))
        B.adsa_step(params, batch.seqs, qd, kd, vd, out, batch.lse, batch.sel_idx, batch.sel_cnt, batch.keep_map,
                    batch.workspace, 0, None)
        torch.cuda.synchronize()
        o, sel_idx, sel_cnt = to_host(out), batch.sel_idx.cpu().numpy(), batch.sel_cnt.cpu().numpy()
        seqs = batch.read_seqs()
        for b in range(n_seq):
            for hd in range(h):
                i = b * h + hd
                q, k, v = toks[b]
                st = states[b, hd]
                before = st.score.copy()
                ref = oracle.step(cfg, st, s, q[p, hd:hd + 1], k[p, hd:hd + 1], v[p, hd:hd + 1])
                sel = sel_idx[i, :sel_cnt[i]]
                assert seqs["n_res"][i] == st.n_res and seqs["step"][i] == s + 1
                assert np.array_equal(sel, ref["sel_idx"]) or near_tie_ok(sel, ref["sel_idx"], before)
                check_out(wl1, o[b, hd:hd + 1], ref["out"], f"{layout} s={s} seq={b} head={hd}")
    Kh, Vh = to_host(K), to_host(V)
    for (b, hd), st in states.items():
        rows = (lambda A: A[b, :st.n_res, hd]) if layout == "slot_major" else (lambda A: A[b, hd, :st.n_res])
        assert np.array_equal(rows(Kh), st.K[:st.n_res, 0].astype(np.float32))
        assert np.array_equal(rows(Vh), st.V[:st.n_res, 0].astype(np.float32))


def test_per_head_selection_is_one_single_head_sequence_per_head():
    """The paper does not say whether heads share one attended set.  Per-head sets need no extra
    kernel: every (sequence, head) is passed as its own adsa_seq with n_heads = 1 (q / out rows
    [n_seq*heads][1][D] are the same memory as [n_seq][heads][D]).  Free-running against one
    single-head oracle per (sequence, head), row-end evictions included."""
    n_seq, h = 2, 4
    geom = dict(n_seq=1, head_dim=64, grid_h=5, grid_w=6, prefix_len=4, win_rows_back=1, win_col_radius=1,
                budget=5, budget_num=0, budget_den=0)
    wl = WL.get_workload("xl", n_heads=h, **geom)            # N(0,1) values: peaked, head-specific attention
    wl1 = WL.get_workload("xl", n_heads=1, **geom)
    cfg = oracle_cfg(wl1, budget=5)
    P = 4
    toks = [WL.gen_tokens(wl, 0, b) for b in range(n_seq)]
    params = params_for(wl1, n_seq * h, cfg.cap)
    batch = LayerBatch(params, DEV)
    states = {}
    for b in range(n_seq):
        for hd in range(h):
            q, k, v = toks[b]
            st = oracle.CacheState.from_prefix(cfg, k[:P, hd:hd + 1], v[:P, hd:hd + 1])
            states[b, hd] = st
            load_state(batch, b * h + hd, st, cfg, 0)
    batch.upload_seqs()
    differing = 0
    for s in range(0, wl.n_image_tokens):
        p = P + s - 1
        qd, kd, vd = (to_device(np.stack([toks[b][i][p] for b in range(n_seq)]).reshape(n_seq * h, 1, 64),
                                params.dtype, DEV) for i in range(3))
        pos_before = batch.pos.cpu().numpy()
        batch.step(qd, kd, vd)
        torch.cuda.synchronize()
        out, sel_idx, sel_cnt = to_host(batch.out), batch.sel_idx.cpu().numpy(), batch.sel_cnt.cpu().numpy()
        seqs = batch.read_seqs()
        for b in range(n_seq):
            for hd in range(h):
                i = b * h + hd
                q, k, v = toks[b]
                st = states[b, hd]
                before = st.score.copy()
                ref = oracle.step(cfg, st, s, q[p, hd:hd + 1], k[p, hd:hd + 1], v[p, hd:hd + 1])
                sel = sel_idx[i, :sel_cnt[i]]
                assert seqs["n_res"][i] == st.n_res and seqs["step"][i] == s + 1
                assert np.array_equal(sel, ref["sel_idx"]) or near_tie_ok(sel, ref["sel_idx"], before)
                check_out(wl1, out[i], ref["out"], f"s={s} seq={b} head={hd}")
        # heads really choose differently: compare the attended POSITIONS of sequence 0's heads
        # (the query token's own slot is filled in during the step; it is the same for every head)
        sets = {tuple(sorted(pos_before[hd, sel_idx[hd, :sel_cnt[hd] - (1 if s >= 1 else 0)]].tolist())) for hd in range(h)}
        differing += len(sets) > 1
    assert differing > 0
