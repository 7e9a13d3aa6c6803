"""Pins for the CPU oracle: it is checked against things other than itself.

Each test names the passage of the paper (or the mathematics) that fixes the
expected value: hand-enumerated partitions, library routines (torch softmax
attention, torch cosine similarity), brute force over subsets, closed forms and
invariants.  None of these tests touches the HIP library.
"""
import itertools
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2506_18226_amd import workloads as WL

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def table_context_lengths():
    """(grid side, kept context, printed reduction) rows of tests/golden/tables_context_lengths.txt."""
    rows = []
    for line in open(os.path.join(GOLDEN, "tables_context_lengths.txt")):
        if line.strip() and not line.startswith("#"):
            side, full, kept, pct = line.split()
            assert int(full) == int(side) ** 2
            rows.append((int(side), int(kept), pct))
    assert len(rows) == 5
    return rows


def tiny_cfg(**kw):
    base = dict(n_heads=2, head_dim=8, grid_h=3, grid_w=4, win_rows_back=1, win_col_radius=1,
                grid_origin=2, budget=0)
    base.update(kw)
    return oracle.make_cfg(**base)


# ----------------------------------------------------------------------------- partition
def test_partition_matches_hand_enumeration():
    """Section 4.1 Eq. 1 with the 2-D local region: fixture enumerated by hand."""
    cfg = tiny_cfg()
    letters = {"P": oracle.PREFIX, "L": oracle.LOCAL, "C": oracle.CANDIDATE}
    n_lines = 0
    for line in open(os.path.join(GOLDEN, "window_3x4.txt")):
        if line.startswith("#") or not line.strip():
            continue
        s_txt, cls_txt = line.split(":")
        s = int(s_txt)
        want = np.array([letters[c] for c in cls_txt.split()], dtype=np.int32)
        pos = np.arange(2 + s, dtype=np.int32)
        got = oracle.classify(cfg, pos, s)
        assert got.tolist() == want.tolist(), f"s={s}"
        n_lines += 1
    assert n_lines == 13


@pytest.mark.parametrize("H,W,R,w,P", [(5, 6, 1, 2, 3), (4, 7, 2, 1, 0), (6, 5, 3, 0, 4), (4, 4, 1, 3, 1)])
def test_partition_brute_force_geometry(H, W, R, w, P):
    """Same predicate stated as a set of grid cells (rows r-R..r, column distance), all steps."""
    cfg = tiny_cfg(grid_h=H, grid_w=W, win_rows_back=R, win_col_radius=w, grid_origin=P)
    for s in range(0 if P else 1, H * W + 1):
        pos = np.arange(P + s, dtype=np.int32)
        got = oracle.classify(cfg, pos, s)
        if s == 0:
            assert (got == oracle.PREFIX).all()
            continue
        r, c = divmod(s - 1, W)
        cells = {(r, cc) for cc in range(0, c + 1)}
        cells |= {(rr, cc) for rr in range(max(0, r - R), r) for cc in range(W) if abs(cc - c) <= w}
        want_local = {P + rr * W + cc for rr, cc in cells}
        assert set(np.nonzero(got == oracle.LOCAL)[0].tolist()) == want_local
        assert set(np.nonzero(got == oracle.PREFIX)[0].tolist()) == set(range(P))
        assert (P + s - 1) in want_local            # the query token attends to itself


@pytest.mark.parametrize("R", [1, 2])
def test_wide_window_is_the_papers_recent_m_tokens(R):
    """Section 4.1: local = 'the most recent m tokens'.  With w >= W-1 the 2-D region
    is exactly the last (c+1) + R*W image tokens in sequence order."""
    H, W, P = 5, 6, 3
    cfg = tiny_cfg(grid_h=H, grid_w=W, win_rows_back=R, win_col_radius=W - 1, grid_origin=P)
    for s in range(1, H * W + 1):
        got = oracle.classify(cfg, np.arange(P + s, dtype=np.int32), s)
        c = (s - 1) % W
        m = min(s, (c + 1) + R * W)
        want = np.full(P + s, oracle.CANDIDATE)
        want[:P] = oracle.PREFIX
        want[P + s - m:] = oracle.LOCAL
        assert got.tolist() == want.tolist()


def test_partition_rejects_bad_state():
    cfg = tiny_cfg()
    with pytest.raises(RuntimeError):
        oracle.classify(cfg, np.arange(2 + 5, dtype=np.int32), 3)      # entries from the future
    with pytest.raises(RuntimeError):
        oracle.classify(cfg, np.arange(4, dtype=np.int32), 0)          # image entry at s = 0
    with pytest.raises(RuntimeError):
        oracle.classify(cfg, np.arange(2, dtype=np.int32), 13)         # s beyond the grid


# ----------------------------------------------------------------------------- Eq. 2-3
def test_vcos_closed_forms():
    """Eq. 2-3 special cases: identical vectors -> 1, orthogonal -> 0, antipodal pair -> -1."""
    cfg = tiny_cfg(n_heads=1, head_dim=4)
    same = np.tile(np.array([[1.0, 2.0, -3.0, 0.5]], dtype=np.float32), (5, 1))
    assert np.allclose(oracle.vcos(cfg, same, np.arange(5)), 1.0, atol=1e-12)
    eye = np.eye(4, dtype=np.float32) * np.array([1, 2, 3, 4], dtype=np.float32)
    assert np.allclose(oracle.vcos(cfg, eye, np.arange(4)), 0.0, atol=1e-15)
    anti = np.array([[1, 1, 0, 0], [-2, -2, 0, 0]], dtype=np.float32)
    assert np.allclose(oracle.vcos(cfg, anti, np.arange(2)), -1.0, atol=1e-12)
    assert oracle.vcos(cfg, anti, np.array([1])).tolist() == [0.0]     # N = 1
    zero = np.zeros((3, 4), dtype=np.float32)
    zero[0, 0] = 1.0
    assert np.allclose(oracle.vcos(cfg, zero, np.arange(3)), 0.0)      # zero-norm rows: eps guard


def test_vcos_matches_torch_cosine_similarity_and_closed_form():
    """Eq. 2 is torch.nn.functional.cosine_similarity pairwise; Eq. 3 its off-diagonal mean,
    which equals (v^_i . sum_j v^_j - 1)/(N-1)."""
    rng = np.random.default_rng(3)
    h, D, n = 3, 8, 17
    cfg = tiny_cfg(n_heads=h, head_dim=D)
    V = rng.standard_normal((30, h * D)).astype(np.float32)
    slots = np.sort(rng.choice(30, n, replace=False)).astype(np.int32)
    got = oracle.vcos(cfg, V, slots)
    vt = torch.from_numpy(V[slots]).double()
    S = torch.nn.functional.cosine_similarity(vt[:, None, :], vt[None, :, :], dim=-1)
    S.fill_diagonal_(0.0)
    want = (S.sum(dim=1) / (n - 1)).numpy()
    assert np.allclose(got, want, atol=1e-12)
    vh = V[slots].astype(np.float64)
    vh /= np.linalg.norm(vh, axis=1, keepdims=True)
    closed = (vh @ vh.sum(axis=0) - 1.0) / (n - 1)
    assert np.allclose(got, closed, atol=1e-12)


# ----------------------------------------------------------------------------- Eq. 4
@pytest.mark.parametrize("keep_largest", [True, False])
def test_rank_keep_is_the_argmin_over_subsets(keep_largest):
    """Eq. 4: argmin over all size-K subsets of the summed score (argmax for keep-largest).
    Enumerate every subset; the oracle must reach the optimum and, among optimal subsets,
    return the lexicographically smallest (lowest-index tie-break)."""
    rng = np.random.default_rng(11)
    for trial in range(30):
        n = int(rng.integers(1, 11))
        levels = rng.integers(1, 5)
        score = (rng.integers(0, levels + 1, size=16).astype(np.float32) - 1.0) * 0.5   # many ties, -0.5..
        if trial % 3 == 0:
            score = rng.standard_normal(16).astype(np.float32)
        slots = np.sort(rng.choice(16, n, replace=False)).astype(np.int32)
        for K in range(0, n + 2):
            got = oracle.rank_keep(slots, score, keep_largest, K)
            k_eff = min(K, n)
            assert got.sum() == k_eff
            best, best_sets = None, []
            for sub in itertools.combinations(range(n), k_eff):
                tot = float(np.sum(score[slots[list(sub)]].astype(np.float64)))
                key = -tot if keep_largest else tot
                if best is None or key < best - 1e-12:
                    best, best_sets = key, [sub]
                elif abs(key - best) <= 1e-12:
                    best_sets.append(sub)
            assert tuple(np.nonzero(got)[0].tolist()) == min(best_sets)


def test_rank_keep_signed_zero_and_infinities():
    score = np.array([0.0, -0.0, np.inf, -np.inf, 0.0], dtype=np.float32)
    slots = np.arange(5, dtype=np.int32)
    assert oracle.rank_keep(slots, score, True, 3).tolist() == [True, True, True, False, False]
    assert oracle.rank_keep(slots, score, False, 3).tolist() == [True, True, False, True, False]


# ----------------------------------------------------------------------------- attention
def _sdpa(q, K, V, scale=None):
    """torch softmax attention in fp64: q [h][D], K,V [n][h][D] -> out [h][D], lse [h]."""
    qt = torch.from_numpy(np.asarray(q, dtype=np.float64))[:, None, :]           # h,1,D
    Kt = torch.from_numpy(np.asarray(K, dtype=np.float64)).permute(1, 0, 2)      # h,n,D
    Vt = torch.from_numpy(np.asarray(V, dtype=np.float64)).permute(1, 0, 2)
    out = torch.nn.functional.scaled_dot_product_attention(qt, Kt, Vt, scale=scale)
    sc = scale if scale is not None else 1.0 / np.sqrt(q.shape[-1])
    lse = torch.logsumexp((qt @ Kt.transpose(1, 2)) * sc, dim=-1)[:, 0]
    return out[:, 0, :].numpy(), lse.numpy()


def test_attend_matches_torch_sdpa_on_a_gathered_set():
    """Eq. 5 + attention: identical to library softmax attention over the gathered rows."""
    rng = np.random.default_rng(5)
    h, D, n = 3, 16, 40
    cfg = tiny_cfg(n_heads=h, head_dim=D)
    K = rng.standard_normal((n, h, D)).astype(np.float32)
    V = rng.standard_normal((n, h, D)).astype(np.float32)
    q = rng.standard_normal((h, D)).astype(np.float32)
    sel = np.sort(rng.choice(n, 13, replace=False)).astype(np.int32)
    out, lse, probs = oracle.attend(cfg, K, V, q, sel, want_probs=True)
    want_out, want_lse = _sdpa(q, K[sel], V[sel])
    assert np.allclose(out, want_out, atol=1e-12)
    assert np.allclose(lse, want_lse, atol=1e-12)
    assert np.allclose(probs.sum(axis=1), 1.0, atol=1e-12)             # softmax rows sum to 1
    lo, hi = V[sel].min(axis=0), V[sel].max(axis=0)
    assert (out >= lo - 1e-12).all() and (out <= hi + 1e-12).all()     # convex combination
    cfg2 = tiny_cfg(n_heads=h, head_dim=D, softmax_scale=0.37)
    out2, lse2 = oracle.attend(cfg2, K, V, q, sel)
    w2, l2 = _sdpa(q, K[sel], V[sel], scale=0.37)
    assert np.allclose(out2, w2, atol=1e-12) and np.allclose(lse2, l2, atol=1e-12)


def _run_trajectory(wl, cfg, n_steps=None, s0=0, check=None):
    q, k, v = WL.gen_tokens(wl, 0, 0, prefix_len=cfg.grid_origin)
    P = cfg.grid_origin
    st = oracle.CacheState.from_prefix(cfg, k[:P], v[:P])
    outs = []
    last = wl.n_image_tokens if n_steps is None else n_steps
    for s in range(s0, last):
        p = P + s - 1
        res = oracle.step(cfg, st, s, q[p], k[p], v[p])
        if check:
            check(s, st, res)
        outs.append(res)
    return q, k, v, st, outs


@pytest.mark.parametrize("mode", [WL.SCORE_ATTN_MASS, WL.SCORE_VCOS])
def test_budget_covering_context_equals_dense_causal_attention(mode):
    """Section 4.2: the compact cache 'behaves identically to the baseline when the cache is
    not full'.  With B >= context nothing is dropped, so every step must equal dense causal
    attention over all L tokens (torch SDPA), and nothing is ever evicted."""
    wl = WL.get_workload("tiny", n_heads=2, head_dim=16, grid_h=5, grid_w=6, prefix_len=4)
    L = 4 + 30
    cfg = oracle.make_cfg(n_heads=2, head_dim=16, grid_h=5, grid_w=6, win_rows_back=1, win_col_radius=1,
                          grid_origin=4, budget=L, score_mode=mode, cap=L)
    q, k, v, st, outs = _run_trajectory(wl, cfg, n_steps=31)
    for s, res in enumerate(outs):
        n = 4 + s
        assert res["sel_idx"].tolist() == list(range(n))
        want, want_lse = _sdpa(q[n - 1], k[:n], v[:n])
        assert np.allclose(res["out"], want, atol=1e-12)
        assert np.allclose(res["lse"], want_lse, atol=1e-12)
        if res["compacted"]:
            assert res["keep_map"].tolist() == list(range(n))
    assert st.n_res == L and st.pos[:L].tolist() == list(range(L))


def test_accumulated_mass_is_the_column_sum_of_the_causal_attention_matrix():
    """ATTN_MASS with nothing dropped: score_i after the trajectory equals the sum over
    query rows and heads of the dense causal attention matrix column i (torch softmax)."""
    wl = WL.get_workload("tiny", n_heads=3, head_dim=8, grid_h=4, grid_w=5, prefix_len=3)
    P, n_img, h, D = 3, 20, 3, 8
    L = P + n_img
    cfg = oracle.make_cfg(n_heads=h, head_dim=D, grid_h=4, grid_w=5, win_rows_back=1, win_col_radius=1,
                          grid_origin=P, budget=L, cap=L)
    q, k, v, st, outs = _run_trajectory(wl, cfg, n_steps=n_img + 1)
    # query rows: positions P-1 .. L-1 (decode steps s = 0 .. n_img)
    qt = torch.from_numpy(q[P - 1:L].astype(np.float64)).permute(1, 0, 2)       # h, nq, D
    kt = torch.from_numpy(k[:L].astype(np.float64)).permute(1, 0, 2)
    logits = qt @ kt.transpose(1, 2) / np.sqrt(D)
    rows = torch.arange(P - 1, L)[:, None]
    cols = torch.arange(L)[None, :]
    logits = logits.masked_fill(cols > rows, float("-inf"))
    A = torch.softmax(logits, dim=-1)
    want = A.sum(dim=(0, 1)).numpy()
    assert np.allclose(st.score[:L], want, rtol=2e-6, atol=1e-6)
    assert abs(float(st.score[:L].astype(np.float64).sum()) - h * (n_img + 1)) < 1e-4   # mass conservation


def test_zero_budget_is_window_attention_with_prefix_and_plain_window():
    """Fig. 2's named baselines as special cases: B = 0 -> window attention with prefix;
    B = 0 and no pinned prefix -> plain window attention (the prefix is dropped)."""
    pos = np.arange(2 + 9, dtype=np.int32)
    score = np.linspace(1, 2, pos.size).astype(np.float32)
    cfg = tiny_cfg(budget=0)
    sel, _ = oracle.select(cfg, pos, score, None, 9)
    cls = oracle.classify(cfg, pos, 9)
    assert sel.tolist() == np.nonzero(cls != oracle.CANDIDATE)[0].tolist()
    assert sel.tolist() == [0, 1, 6, 7, 10]
    cfg0 = tiny_cfg(budget=0, n_keep_prefix=0)
    sel0, _ = oracle.select(cfg0, pos, score, None, 9)
    assert sel0.tolist() == [6, 7, 10]


def test_select_invariants_and_direction():
    """|GLOBAL| = min(B, |C|); PREFIX and LOCAL always attended (Table 3: dropping either is
    catastrophic); list strictly ascending; ATTN_MASS keeps the largest, VCOS the lowest
    mean cosine (Eq. 4 argmin)."""
    rng = np.random.default_rng(9)
    P, H, W = 5, 6, 7
    for mode in (WL.SCORE_ATTN_MASS, WL.SCORE_EXT_SMALLEST, WL.SCORE_EXT_LARGEST):
        for B in (0, 1, 4, 9, 100):
            cfg = tiny_cfg(grid_h=H, grid_w=W, grid_origin=P, win_rows_back=1, win_col_radius=2,
                           budget=B, score_mode=mode)
            for s in (0, 1, 8, 20, 42):
                pos = np.arange(P + s, dtype=np.int32)
                score = rng.standard_normal(pos.size).astype(np.float32)
                sel, _ = oracle.select(cfg, pos, score, None, s)
                cls = oracle.classify(cfg, pos, s)
                cand = np.nonzero(cls == oracle.CANDIDATE)[0]
                fixed = np.nonzero(cls != oracle.CANDIDATE)[0]
                assert set(fixed.tolist()) <= set(sel.tolist())
                glob = sorted(set(sel.tolist()) - set(fixed.tolist()))
                assert len(glob) == min(B, cand.size)
                assert (np.diff(sel) > 0).all()
                order = np.argsort(-score[cand] if mode != WL.SCORE_EXT_SMALLEST else score[cand],
                                   kind="stable")
                assert glob == sorted(cand[order[:len(glob)]].tolist())


def test_vcos_select_keeps_the_most_diverse_tokens():
    """Section 4.1: the K tokens with the lowest average similarity are kept.  Build V with a
    tight cluster plus a few outliers in distinct directions: the outliers must be chosen."""
    h, D = 1, 8
    P, H, W = 1, 4, 4
    cfg = oracle.make_cfg(n_heads=h, head_dim=D, grid_h=H, grid_w=W, win_rows_back=1, win_col_radius=0,
                          grid_origin=P, budget=3, score_mode=WL.SCORE_VCOS)
    s = 16
    pos = np.arange(P + s, dtype=np.int32)
    rng = np.random.default_rng(2)
    V = np.tile(np.array([1, 1, 1, 1, 0, 0, 0, 0], np.float32), (P + s, 1))
    V += 0.01 * rng.standard_normal(V.shape).astype(np.float32)
    outliers = [3, 6, 8]                                 # candidate slots (rows 0..1 of the grid)
    for t, slot in enumerate(outliers):
        V[slot] = 0
        V[slot, 4 + t] = 5.0
    sel, score = oracle.select(cfg, pos, np.zeros(pos.size, np.float32), V.reshape(-1, h, D), s)
    cls = oracle.classify(cfg, pos, s)
    glob = sorted(set(sel.tolist()) - set(np.nonzero(cls != oracle.CANDIDATE)[0].tolist()))
    assert glob == outliers
    cand = np.nonzero(cls == oracle.CANDIDATE)[0]
    assert np.allclose(score[cand], oracle.vcos(cfg, V, cand).astype(np.float32))


def test_context_bookkeeping_reproduces_table_1_and_2_totals():
    """Tables 1-2 report context = prefix + selected + local: 256 of 576 (-55.6 %), 384 of 576
    (-33.3 %), 512 / 640 / 768 of 1024 (-50 / -37.5 / -25 %).  The paper's window is the most
    recent m tokens, so use w >= W-1; at the last decode step the attended count must hit the
    total exactly.  (The split into n, K, m is not given in the paper: only the sum is pinned.)"""
    for W, total, pct in table_context_lengths():
        n_prefix = W                                    # pin the first image row as the prefix
        cfg = oracle.make_cfg(n_heads=1, head_dim=4, grid_h=W, grid_w=W, win_rows_back=1,
                              win_col_radius=W - 1, grid_origin=0, n_keep_prefix=n_prefix,
                              budget=total - n_prefix - 2 * W, cap=W * W)
        s = W * W
        pos = np.arange(s, dtype=np.int32)
        sel, _ = oracle.select(cfg, pos, np.arange(s, dtype=np.float32), None, s)
        assert sel.size == total
        assert f"{100.0 * (1 - sel.size / (W * W)):.1f}" == pct


# ----------------------------------------------------------------------------- eviction
@pytest.mark.parametrize("mode,R", [(WL.SCORE_ATTN_MASS, 1), (WL.SCORE_VCOS, 1), (WL.SCORE_ATTN_MASS, 2)])
def test_trajectory_invariants_of_the_dynamic_cache(mode, R):
    """Section 4.2 in its per-row form, over a whole trajectory: capacity bound, ascending
    positions, the keep map is an order-preserving bijection onto [0, n_keep), the prefix is
    never evicted, every step's local window is resident, and evicted tokens never return."""
    P, H, W, w, B = 6, 8, 8, 2, 10
    wl = WL.get_workload("tiny", n_heads=2, head_dim=8, grid_h=H, grid_w=W, prefix_len=P)
    cfg = oracle.make_cfg(n_heads=2, head_dim=8, grid_h=H, grid_w=W, win_rows_back=R, win_col_radius=w,
                          grid_origin=P, budget=B, score_mode=mode)
    assert cfg.cap == P + B + (R + 1) * W
    seen_evicted = set()
    n_compactions = [0]

    def check(s, st, res):
        n = st.n_res
        assert n <= cfg.cap
        pos = st.pos[:n]
        assert (np.diff(pos) > 0).all()
        assert pos[:P].tolist() == list(range(P))
        assert not (set(pos.tolist()) & seen_evicted)
        if s >= 1:
            r, c = divmod(s - 1, W)
            need = {P + r * W + cc for cc in range(c + 1)}
            need |= {P + rr * W + cc for rr in range(max(0, r - R), r) for cc in range(W) if abs(cc - c) <= w}
            # sel_idx refers to slots before this step's compaction; map through keep_map
            if res["compacted"]:
                km = res["keep_map"]
                kept = km[km >= 0]
                assert kept.tolist() == list(range(kept.size)) and kept.size == n
                assert (s - 1) % W == W - 1
                n_compactions[0] += 1
                # protected rows survive, so the next row's windows are resident
                surv = set(pos.tolist())
                for rr in range(max(0, r - R + 1), r + 1):
                    assert {P + rr * W + cc for cc in range(W)} <= surv
                rest = n - P - sum(1 for p in pos if p >= P and (p - P) // W >= r - R + 1)
                assert rest <= B
            else:
                assert need <= set(pos.tolist())
        if res["compacted"]:
            seen_evicted.update(set(range(P, P + s)) - set(pos.tolist()))

    _run_trajectory(wl, cfg, n_steps=H * W + 1, check=check)
    assert n_compactions[0] == H


def test_compaction_preserves_rows_and_later_attention():
    """Compaction only moves rows: after it, slot keep_map[i] holds exactly what slot i held,
    and attention over the same tokens gives the same result (softmax is order-free up to
    rounding; here the order is also preserved, so it is bit-identical)."""
    rng = np.random.default_rng(4)
    P, H, W, R, B = 3, 5, 6, 1, 7
    h, D = 2, 8
    cfg = oracle.make_cfg(n_heads=h, head_dim=D, grid_h=H, grid_w=W, win_rows_back=R, win_col_radius=1,
                          grid_origin=P, budget=B, score_mode=WL.SCORE_EXT_LARGEST, cap=P + H * W)
    s = 3 * W                                           # closes row 2
    n = P + s
    st = oracle.CacheState.from_arrays(cfg, rng.standard_normal((n, h, D)).astype(np.float32),
                                       rng.standard_normal((n, h, D)).astype(np.float32),
                                       np.arange(n, dtype=np.int32),
                                       rng.integers(0, 4, n).astype(np.float32))
    before = st.copy()
    km, did = oracle.compact(cfg, st, s)
    assert did and km.size == n
    kept = np.nonzero(km >= 0)[0]
    assert km[kept].tolist() == list(range(kept.size)) and st.n_res == kept.size
    assert np.array_equal(st.K[:st.n_res], before.K[kept]) and np.array_equal(st.V[:st.n_res], before.V[kept])
    assert np.array_equal(st.pos[:st.n_res], before.pos[kept])
    assert np.array_equal(st.score[:st.n_res], before.score[kept])
    # kept = prefix + row 2 + top-B of the rest (largest score, lowest slot on ties)
    rest = np.arange(P, P + 2 * W)
    order = np.argsort(-before.score[rest], kind="stable")[:B]
    want = sorted(list(range(P)) + rest[order].tolist() + list(range(P + 2 * W, n)))
    assert kept.tolist() == want
    q = rng.standard_normal((h, D)).astype(np.float32)
    o1, l1 = oracle.attend(cfg, before.K, before.V, q, kept.astype(np.int32))
    o2, l2 = oracle.attend(cfg, st.K, st.V, q, np.arange(st.n_res, dtype=np.int32))
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)
    # not a row end: nothing happens
    st2 = before.copy()
    km2, did2 = oracle.compact(cfg, st2, s - 1)
    assert not did2 and st2.n_res == n


def test_fractional_budget_and_overflow():
    """'Global budget: 50 % of the current context' = floor((P+s)/2); a full cache is an error."""
    cfg = oracle.make_cfg(n_heads=1, head_dim=4, grid_h=4, grid_w=4, win_rows_back=1, win_col_radius=1,
                          grid_origin=5, budget_num=1, budget_den=2)
    assert [oracle.budget(cfg, s) for s in (0, 1, 2, 16)] == [2, 3, 3, 10]
    small = oracle.make_cfg(n_heads=1, head_dim=4, grid_h=4, grid_w=4, win_rows_back=1, win_col_radius=1,
                            grid_origin=2, budget=1, cap=3)
    st = oracle.CacheState.from_prefix(small, np.ones((2, 1, 4), np.float32), np.ones((2, 1, 4), np.float32))
    one = np.ones((1, 4), np.float32)
    oracle.step(small, st, 1, one, one, one)
    with pytest.raises(RuntimeError):
        oracle.step(small, st, 2, one, one, one)


# ----------------------------------------------------------------------------- Section 4.2 as written
def test_recent_m_window_partition_by_hand():
    """Section 4.1: 'the most recent m tokens closest to the current step' -- m = 3, prefix n = 2
    (positions 0, 1), 7 image tokens: written out by hand for every step."""
    cfg = tiny_cfg(grid_h=1, grid_w=7, win_recent_m=3)
    P, L, C = oracle.PREFIX, oracle.LOCAL, oracle.CANDIDATE
    want = {0: [P, P], 1: [P, P, L], 2: [P, P, L, L], 3: [P, P, L, L, L], 4: [P, P, C, L, L, L],
            5: [P, P, C, C, L, L, L], 7: [P, P, C, C, C, C, L, L, L]}
    for s, w in want.items():
        assert oracle.classify(cfg, np.arange(2 + s, dtype=np.int32), s).tolist() == w, s


@pytest.mark.parametrize("P,H,W,m,B_", [(2, 4, 4, 10, 0), (3, 5, 6, 4, 2), (1, 6, 3, 7, 1), (4, 3, 8, 2, 3), (2, 4, 5, 13, 0)])
def test_row_end_eviction_with_the_1d_window_never_evicts_a_token_a_later_window_holds(P, H, W, m, B_):
    """Section 4.1's local region (the m most recent tokens) combined with the per-row eviction: local
    tokens are exempt from eviction like the prefix (Table 3: without the local region generation
    collapses).  Over whole trajectories, for both rankings: every step attends its complete window --
    all of image tokens jq-m+1 .. jq that exist --, a row-end eviction removes only tokens that no
    later window contains (j <= jq + 1 - m at the row-closing query jq), keeps at most B of those,
    and the cache never exceeds prefix + B + (m - 1) + W.  (First case: 4x4 grid, m = 10, B = 0 --
    after the first row end the cache must still hold the whole first row, not just the prefix.)"""
    for mode in (WL.SCORE_ATTN_MASS, WL.SCORE_VCOS):
        wl = WL.get_workload("tiny", n_heads=2, head_dim=8, grid_h=H, grid_w=W, prefix_len=P, seed=0xF100 + m)
        cfg = oracle.make_cfg(n_heads=2, head_dim=8, grid_h=H, grid_w=W, win_rows_back=0, win_col_radius=0,
                              grid_origin=P, budget=B_, score_mode=mode, win_recent_m=m)
        assert cfg.cap == P + B_ + (m - 1) + W
        q, k, v = WL.gen_tokens(wl, 0, 0, prefix_len=P)
        st = oracle.CacheState.from_prefix(cfg, k[:P], v[:P])
        n_evicted = 0
        for s in range(0, H * W + 1):
            p = P + s - 1
            pos_before = np.append(st.pos[:st.n_res], P + s - 1) if s >= 1 else st.pos[:st.n_res].copy()
            res = oracle.step(cfg, st, s, q[p], k[p], v[p])
            attended = set(pos_before[res["sel_idx"]].tolist())
            jq = s - 1
            window = {P + j for j in range(max(0, jq - m + 1), jq + 1)}
            assert window <= attended and set(range(P)) <= attended, (mode, s)
            assert len(attended) <= P + len(window) + B_, (mode, s)
            n = st.n_res
            assert n <= cfg.cap, (mode, s)
            if res["compacted"]:
                assert (s - 1) % W == W - 1
                evicted = set(pos_before.tolist()) - set(st.pos[:n].tolist())
                assert all(pp - P <= jq + 1 - m for pp in evicted), (mode, s, sorted(evicted))
                older = [pp for pp in st.pos[:n].tolist() if pp >= P and pp - P <= jq + 1 - m]
                assert len(older) <= B_, (mode, s)
                n_evicted += len(evicted)
        if H * W > m + B_:
            assert n_evicted > 0


def test_streaming_cache_is_the_baseline_until_full_then_evicts_the_most_redundant_token():
    """Section 4.2's cache policy: until the fixed capacity is reached nothing differs from the dense
    baseline; from then on, before each insertion, the candidate with the highest mean pairwise V-cosine
    (Eq. 2-3) -- the most redundant one -- is evicted.
    Checked against torch: dense SDPA while not full; afterwards the evicted token is the argmax of
    the mean pairwise cosine (torch) over the candidates, the cache stays exactly full, prefix and the
    recent window are never touched, order is preserved, and attention runs over everything resident
    (Tables 1-2: KV cache == context)."""
    P, H, W, h, D, m, cap = 3, 5, 6, 2, 8, 4, 14
    wl = WL.get_workload("tiny", n_heads=h, head_dim=D, grid_h=H, grid_w=W, prefix_len=P)
    cfg = oracle.make_cfg(n_heads=h, head_dim=D, grid_h=H, grid_w=W, win_rows_back=0, win_col_radius=0,
                          grid_origin=P, budget=10 ** 6, score_mode=WL.SCORE_VCOS, cap=cap, win_recent_m=m,
                          evict_when_full=1)
    q, k, v = WL.gen_tokens(wl, 0, 0)
    st = oracle.CacheState.from_prefix(cfg, k[:P], v[:P])
    evicted_ever = set()
    for s in range(0, H * W + 1):
        p = P + s - 1
        before = st.copy()
        res = oracle.step(cfg, st, s, q[p], k[p], v[p])
        n_dense = P + s
        if n_dense <= cap:                               # not full yet: the baseline
            assert not res["compacted"]
            assert res["sel_idx"].tolist() == list(range(n_dense))
            want, _ = _sdpa(q[p], k[:n_dense], v[:n_dense])
            assert np.allclose(res["out"], want, atol=1e-12)
            continue
        assert res["compacted"] and st.n_res == cap      # evict one, insert one
        assert res["sel_idx"].tolist() == list(range(cap))           # context == cache
        pos_b = before.pos[:before.n_res]
        cand = [i for i, pp in enumerate(pos_b) if pp >= P and (pp - P) <= (s - 1) - m]   # neither prefix nor recent
        vt = torch.from_numpy(before.V[cand].reshape(len(cand), -1).astype(np.float64))
        S = torch.nn.functional.cosine_similarity(vt[:, None, :], vt[None, :, :], dim=-1)
        S.fill_diagonal_(0.0)
        mean = (S.sum(1) / (len(cand) - 1)).numpy()
        worst = max(i for i in range(len(cand)) if mean[i] >= mean.max() - 1e-15)
        km = res["keep_map"]
        gone = np.nonzero(km < 0)[0].tolist()
        assert gone == [cand[worst]], s
        evicted_ever.add(int(pos_b[cand[worst]]))
        assert st.pos[:P].tolist() == list(range(P))
        assert st.pos[cap - 1] == p and (np.diff(st.pos[:cap]) > 0).all()
        assert not (set(st.pos[:cap].tolist()) & evicted_ever)
        kept = np.nonzero(km >= 0)[0]
        assert np.array_equal(st.K[:cap - 1], before.K[kept]) and np.array_equal(st.V[:cap - 1], before.V[kept])
        want, _ = _sdpa(q[p], st.K[:cap], st.V[:cap])
        assert np.allclose(res["out"], want, atol=1e-12)


def test_streaming_cache_reproduces_the_tables_cache_lengths():
    """Tables 1-2: KV cache = context = 384 / 256 of 576 and 768 / 640 / 512 of 1024 image tokens
    (-33.3, -55.6, -25, -37.5, -50 %).  The paper's cache 'initialises with only half the length':
    capacity is the only knob; run the policy (tiny head size) and read the final cache length."""
    for W, cap, pct in table_context_lengths():
        cfg = oracle.make_cfg(n_heads=1, head_dim=2, grid_h=W, grid_w=W, win_rows_back=0, win_col_radius=0,
                              grid_origin=0, n_keep_prefix=8, budget=10 ** 6, score_mode=WL.SCORE_EXT_SMALLEST,
                              cap=cap, win_recent_m=W + 2, evict_when_full=1)
        st = oracle.CacheState.from_prefix(cfg, np.zeros((0, 1, 2), np.float32), np.zeros((0, 1, 2), np.float32))
        one = np.ones((1, 2), np.float32)
        rng = np.random.default_rng(W + cap)
        longest = 0
        for s in range(1, W * W + 1):
            res = oracle.step(cfg, st, s, one, one, one)
            st.score[st.n_res - 1] = rng.random()
            longest = max(longest, st.n_res, res["sel_idx"].size)
        assert st.n_res == cap and longest == cap
        assert f"{100.0 * (1 - cap / (W * W)):.1f}" == pct


# ----------------------------------------------------------------------------- grouped-query attention
def test_grouped_query_attend_matches_torch_gqa_and_expanded_multi_head():
    """Query head j reads cache head floor(j/G): identical to torch's grouped-query SDPA (a library
    definition) and to the multi-head oracle on a cache whose heads are repeated G times."""
    rng = np.random.default_rng(17)
    h, G, D, n = 3, 4, 16, 50
    cfg = tiny_cfg(n_heads=h, head_dim=D, q_per_kv=G)
    K = rng.standard_normal((n, h, D)).astype(np.float32)
    V = rng.standard_normal((n, h, D)).astype(np.float32)
    q = rng.standard_normal((h * G, D)).astype(np.float32)
    sel = np.sort(rng.choice(n, 21, replace=False)).astype(np.int32)
    out, lse, probs = oracle.attend(cfg, K, V, q, sel, want_probs=True)
    assert out.shape == (h * G, D) and probs.shape == (h * G, sel.size)
    qt = torch.from_numpy(q.astype(np.float64))[None, :, None, :]                      # 1,hq,1,D
    Kt = torch.from_numpy(K[sel].astype(np.float64)).permute(1, 0, 2)[None]            # 1,h,n,D
    Vt = torch.from_numpy(V[sel].astype(np.float64)).permute(1, 0, 2)[None]
    want = torch.nn.functional.scaled_dot_product_attention(qt, Kt, Vt, enable_gqa=True)[0, :, 0, :].numpy()
    assert np.allclose(out, want, atol=1e-12)
    # the multi-head oracle on the expanded cache (np.repeat: head j of the copy = head j // G)
    cfg_mha = tiny_cfg(n_heads=h * G, head_dim=D)
    out2, lse2, probs2 = oracle.attend(cfg_mha, np.repeat(K, G, axis=1), np.repeat(V, G, axis=1), q, sel,
                                       want_probs=True)
    assert np.array_equal(out, out2) and np.array_equal(lse, lse2) and np.array_equal(probs, probs2)
    # the wrong mapping (j % G) is a different function: the pin would catch it
    wrong = tiny_cfg(n_heads=h * G, head_dim=D)
    out3, _ = oracle.attend(wrong, np.tile(K, (1, G, 1)), np.tile(V, (1, G, 1)), q, sel)
    assert not np.allclose(out, out3, atol=1e-6)
    # G = 0 and G = 1 are the multi-head case
    for g1 in (0, 1):
        c1 = tiny_cfg(n_heads=h, head_dim=D, q_per_kv=g1)
        o1, l1 = oracle.attend(c1, K, V, q[:h], sel)
        o0, l0 = _sdpa(q[:h], K[sel], V[sel])
        assert np.allclose(o1, o0, atol=1e-12) and np.allclose(l1, l0, atol=1e-12)


def test_grouped_query_mass_counts_every_query_head():
    """ATTN_MASS under grouped queries: each step hands out exactly one unit of probability per QUERY
    head, and a whole trajectory equals the multi-head trajectory on the expanded cache."""
    wl = WL.get_workload("tiny")
    G, P = 3, wl.prefix_len
    cfg = oracle_cfg_gqa(wl, G)
    cfg_mha = oracle_cfg_gqa(wl, 1, n_heads=wl.n_heads * G)
    rng = np.random.default_rng(23)
    q, k, v = WL.gen_tokens(wl, 0, 0, prefix_len=P)
    L = k.shape[0]
    qg = WL.round_to_bf16(rng.standard_normal((L, wl.n_heads * G, wl.head_dim)).astype(np.float32))
    st = oracle.CacheState.from_prefix(cfg, k[:P], v[:P])
    st2 = oracle.CacheState.from_prefix(cfg_mha, np.repeat(k[:P], G, axis=1), np.repeat(v[:P], G, axis=1))
    for s in range(0, 2 * wl.grid_w + 3):
        p = P + s - 1
        before = st.score[:st.n_res].astype(np.float64).sum()
        r = oracle.step(cfg, st, s, qg[p], k[p], v[p])
        r2 = oracle.step(cfg_mha, st2, s, qg[p], np.repeat(k[p], G, axis=0), np.repeat(v[p], G, axis=0))
        assert np.array_equal(r["sel_idx"], r2["sel_idx"]) and np.array_equal(r["out"], r2["out"])
        assert np.array_equal(st.score[:st.n_res], st2.score[:st2.n_res]) and st.n_res == st2.n_res
        if not r["compacted"]:
            after = st.score[:st.n_res].astype(np.float64).sum()
            assert abs(after - before - wl.n_heads * G) < 1e-4


def oracle_cfg_gqa(wl, G, n_heads=None):
    return oracle.make_cfg(
        n_heads=wl.n_heads if n_heads is None else n_heads, head_dim=wl.head_dim, grid_h=wl.grid_h,
        grid_w=wl.grid_w, win_rows_back=wl.win_rows_back, win_col_radius=wl.win_col_radius,
        grid_origin=wl.prefix_len, budget=wl.budget, score_mode=WL.SCORE_ATTN_MASS, q_per_kv=G)


# ----------------------------------------------------------------------------- randomised properties
@pytest.mark.parametrize("seed", range(30))
def test_random_configurations_keep_the_methods_invariants(seed):
    """Seeded random grids, windows, prefixes, budgets and ranking modes: at every step of the whole
    trajectory the attended set is prefix + local + exactly min(B, |candidates|) candidates, ascending;
    the kept candidates are the best by score with the lower slot first among equals (re-derived here by
    a plain sort); the window of every step is resident; positions stay ascending and within capacity;
    evicted tokens never come back; softmax rows sum to one through the mass bookkeeping."""
    g = np.random.default_rng(9000 + seed)
    H, W = int(g.integers(2, 7)), int(g.integers(2, 9))
    R, w = int(g.integers(0, min(3, H))), int(g.integers(0, W + 1))
    P = int(g.integers(1, 9))
    n_pin = int(g.integers(1, P + 1))                 # (with nothing pinned and B = 0, step 0 would attend nothing)
    B_ = int(g.integers(0, 10))
    mode = int(g.choice([WL.SCORE_ATTN_MASS, WL.SCORE_VCOS]))
    h, D = int(g.integers(1, 4)), 8
    wl = WL.get_workload("tiny", n_heads=h, head_dim=D, grid_h=H, grid_w=W, prefix_len=P, value_kind="gauss",
                         value_scale=0.5, seed=0xD000 + seed)
    cfg = oracle.make_cfg(n_heads=h, head_dim=D, grid_h=H, grid_w=W, win_rows_back=R, win_col_radius=w,
                          grid_origin=P, n_keep_prefix=n_pin, budget=B_, score_mode=mode)
    q, k, v = WL.gen_tokens(wl, 0, 0, prefix_len=P)
    st = oracle.CacheState.from_prefix(cfg, k[:P], v[:P])
    gone = set()
    for s in range(0, H * W + 1):
        p = P + s - 1
        n0 = st.n_res
        pos_before = np.append(st.pos[:n0], P + s - 1) if s >= 1 else st.pos[:n0].copy()
        score_before = np.append(st.score[:n0], 0.0).astype(np.float32) if s >= 1 else st.score[:n0].copy()
        mass_before = float(score_before.astype(np.float64).sum())
        res = oracle.step(cfg, st, s, q[p], k[p], v[p])
        sel = res["sel_idx"]
        cls = oracle.classify(cfg, pos_before, s)
        fixed = np.nonzero(cls != oracle.CANDIDATE)[0]
        cand = np.nonzero(cls == oracle.CANDIDATE)[0]
        assert (np.diff(sel) > 0).all() and set(fixed.tolist()) <= set(sel.tolist()), (seed, s)
        chosen = np.array(sorted(set(sel.tolist()) - set(fixed.tolist())), dtype=np.int64)
        assert chosen.size == min(B_, cand.size) and set(chosen.tolist()) <= set(cand.tolist()), (seed, s)
        if mode == WL.SCORE_ATTN_MASS and cand.size:
            # the ranking saw the scores before this step's accumulation: best first, lower slot among equals
            order = sorted(cand.tolist(), key=lambda i: (-float(score_before[i]), i))
            assert sorted(order[:chosen.size]) == chosen.tolist(), (seed, s)
        if s >= 1:                                        # the query's window is resident and attended
            r, c = divmod(s - 1, W)
            need = {P + r * W + cc for cc in range(c + 1)}
            need |= {P + rr * W + cc for rr in range(max(0, r - R), r) for cc in range(W) if abs(cc - c) <= w}
            assert need <= set(pos_before[sel].tolist()), (seed, s)
        n = st.n_res
        assert n <= cfg.cap and (np.diff(st.pos[:n]) > 0).all(), (seed, s)
        assert not (set(st.pos[:n].tolist()) & gone), (seed, s)
        if res["compacted"]:
            km = res["keep_map"]
            assert km[km >= 0].tolist() == list(range(n)), (seed, s)
            gone |= set(pos_before.tolist()) - set(st.pos[:n].tolist())
            assert all(pp >= n_pin for pp in gone), (seed, s)           # pinned positions are never evicted
        elif mode == WL.SCORE_ATTN_MASS:
            # one unit of probability per head was handed out (nothing left the cache in this step)
            assert abs(float(st.score[:n].astype(np.float64).sum()) - mass_before - h) < 1e-4, (seed, s)
