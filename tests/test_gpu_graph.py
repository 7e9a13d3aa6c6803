"""A whole decode step captured once as a HIP graph and replayed for every step.

Every decision that depends on the sequences' state (row end or not, what to evict, where the new
token goes) is taken on the device, and the entry points only enqueue kernels (no allocation, no
synchronisation, no memset node), so ONE captured adsa_step serves all steps of a trajectory: the
caller refreshes q / k_new / v_new in place and replays.  Each replay is checked, bit for bit, against
the same step run eagerly on a twin batch; the eager path itself is checked against the oracle in
test_gpu_parity and test_gpu_gqa.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_18226_amd import binding as B
from paper_2506_18226_amd import workloads as WL
from paper_2506_18226_amd.batch import LayerBatch, to_device, to_host

from common import oracle_cfg
from test_gpu_parity import DEV, params_for, load_state, check_out

pytestmark = pytest.mark.gpu


def _twin_batches(wl, cfg, n_seq, make=None):
    batches = []
    toks = [WL.gen_tokens(wl, 0, b, prefix_len=cfg.grid_origin) for b in range(n_seq)]
    for _ in range(3):
        batch = LayerBatch(make() if make else params_for(wl, n_seq, cfg.cap), DEV)
        for b in range(n_seq):
            q, k, v = toks[b]
            st = oracle.CacheState.from_prefix(cfg, k[:cfg.grid_origin], v[:cfg.grid_origin])
            load_state(batch, b, st, cfg, 0)
        batch.upload_seqs()
        batches.append(batch)
    return batches, toks


@pytest.mark.parametrize("over", [
    dict(n_heads=4, head_dim=64, grid_h=5, grid_w=8, prefix_len=5, dtype="bf16"),
    dict(n_heads=2, head_dim=128, grid_h=4, grid_w=8, prefix_len=7, dtype="bf16", q_per_kv=4),
    dict(n_heads=3, head_dim=64, grid_h=4, grid_w=6, prefix_len=4, dtype="f32", score_mode=WL.SCORE_VCOS),
])
def test_one_captured_step_replayed_over_a_trajectory(over):
    wl = WL.get_workload("tiny", n_seq=3, win_rows_back=1, win_col_radius=1, budget=6, value_kind="gauss",
                         value_scale=0.5, **over)
    cfg = oracle_cfg(wl)
    n, P, S = wl.n_seq, cfg.grid_origin, wl.n_image_tokens
    (eager, graphed, warm), toks = _twin_batches(wl, cfg, n)
    qs, ks, vs = (np.stack([t[i] for t in toks], axis=1) for i in range(3))        # [L][n][heads][D]
    qd, kd, vd = (to_device(x, eager.params.dtype, DEV) for x in (qs, ks, vs))
    q_in, k_in, v_in = (torch.zeros_like(x[0]) for x in (qd, kd, vd))              # fixed addresses for the graph

    # warm-up launch of every kernel outside the capture (first-use set-up of a kernel is not capturable work)
    warm.step(qd[P - 1], kd[P - 1], vd[P - 1])
    torch.cuda.synchronize()

    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        graphed.step(q_in, k_in, v_in)
    torch.cuda.synchronize()
    assert (graphed.read_seqs()["step"] == 0).all()                                  # capturing ran nothing

    for s in range(S + 1):
        p = P + s - 1
        q_in.copy_(qd[p]); k_in.copy_(kd[p]); v_in.copy_(vd[p])
        g.replay()
        eager.step(qd[p], kd[p], vd[p])
        torch.cuda.synchronize()
        a, b = eager.read_seqs(), graphed.read_seqs()
        tag = f"s={s}"
        for f in ("n_res", "step", "status", "compacted", "pending_slot"):
            assert np.array_equal(a[f], b[f]), (tag, f)
        assert (a["status"] == 0).all() and (a["step"] == s + 1).all(), tag
        assert torch.equal(eager.sel_cnt, graphed.sel_cnt), tag
        for b_ in range(n):
            c = int(eager.sel_cnt[b_])
            assert torch.equal(eager.sel_idx[b_, :c], graphed.sel_idx[b_, :c]), tag
        assert torch.equal(eager.out, graphed.out) and torch.equal(eager.lse, graphed.lse), tag
        assert torch.equal(eager.K, graphed.K) and torch.equal(eager.V, graphed.V), tag
        assert torch.equal(eager.pos, graphed.pos) and torch.equal(eager.score, graphed.score), tag
    out = to_host(graphed.out)
    assert np.isfinite(out).all()
    final = graphed.read_seqs()
    assert (final["n_res"] <= cfg.cap).all() and (final["step"] == S + 1).all()


def test_captured_step_of_the_papers_cache_policy_with_fused_ranking():
    """Evict-one-when-full with slot reuse and the V-cosine ranking fused into the attention launch: five
    kernels per step (two-pass fallback pair, eviction plan, advance of the running sum, selection, attention),
    all decisions on the device, captured once and replayed over a whole trajectory; bit-identical to eager."""
    P, H, W, m, cap, n, h, D = 4, 6, 6, 5, 16, 2, 3, 64
    wl = WL.get_workload("tiny", n_seq=n, n_heads=h, head_dim=D, grid_h=H, grid_w=W, prefix_len=P, dtype="bf16",
                         value_kind="gauss", value_scale=0.5, win_rows_back=0, win_col_radius=0)
    cfg = oracle.make_cfg(n_heads=h, head_dim=D, grid_h=H, grid_w=W, win_rows_back=0, win_col_radius=0, grid_origin=P,
                          budget=10 ** 6, score_mode=B.SCORE_VCOS, cap=cap, win_recent_m=m, evict_when_full=1)

    def make():
        return B.make_params(n_seq=n, n_heads=h, head_dim=D, grid_h=H, grid_w=W, win_rows_back=0, win_col_radius=0,
                             dtype=B.BF16, score_mode=B.SCORE_VCOS_FUSED, cap=cap, win_recent_m=m,
                             evict_policy=B.EVICT_REUSE_SLOT)

    (eager, graphed, warm), toks = _twin_batches(wl, cfg, n, make)
    qs, ks, vs = (np.stack([t[i] for t in toks], axis=1) for i in range(3))
    qd, kd, vd = (to_device(x, eager.params.dtype, DEV) for x in (qs, ks, vs))
    q_in, k_in, v_in = (torch.zeros_like(x[0]) for x in (qd, kd, vd))
    warm.step(qd[P - 1], kd[P - 1], vd[P - 1])
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        graphed.step(q_in, k_in, v_in)
    torch.cuda.synchronize()
    evictions = 0
    for s in range(H * W + 1):
        p = P + s - 1
        q_in.copy_(qd[p]); k_in.copy_(kd[p]); v_in.copy_(vd[p])
        g.replay()
        eager.step(qd[p], kd[p], vd[p])
        torch.cuda.synchronize()
        a, b = eager.read_seqs(), graphed.read_seqs()
        for f in ("n_res", "step", "status", "compacted", "pending_slot", "hole"):
            assert np.array_equal(a[f], b[f]), (s, f)
        assert (a["status"] == 0).all() and (a["step"] == s + 1).all(), s
        evictions += int(a["compacted"].sum())
        assert torch.equal(eager.out, graphed.out) and torch.equal(eager.lse, graphed.lse), s
        assert torch.equal(eager.K, graphed.K) and torch.equal(eager.V, graphed.V) and torch.equal(eager.pos, graphed.pos), s
        assert torch.equal(eager.vcos_u, graphed.vcos_u) and torch.equal(eager.score, graphed.score), s
    assert evictions >= 2 * 20 and (eager.read_seqs()["n_res"] == cap).all()


def test_one_graph_per_decode_step_of_a_whole_model():
    """A decode step of ALL layers as one captured graph -- one selection launch for every layer's sequences,
    one attention launch per layer, and (the second graph) the eviction/compaction launch pair of a step that
    closes a grid row -- replayed over a whole trajectory; inputs reach fixed staging buffers through a gather
    captured in the same graph, indexed by a device-side step counter.  After every replay everything the step
    produced is compared, bit for bit, with the same step issued eagerly, launch by launch, on a twin model."""
    from paper_2506_18226_amd.batch import ModelBatch
    n_layers, n, h, D, P, H, W = 3, 4, 4, 64, 6, 5, 8
    wl = WL.get_workload("tiny", n_seq=n, n_heads=h, head_dim=D, grid_h=H, grid_w=W, prefix_len=P, dtype="bf16",
                         win_rows_back=1, win_col_radius=2, budget=9, value_kind="gauss", value_scale=0.5)
    cfg = oracle_cfg(wl)
    lp = params_for(wl, n, cfg.cap)
    S = H * W + 1                                               # steps 0 .. H*W
    toks = [[WL.gen_tokens(wl, l, b, prefix_len=P) for b in range(n)] for l in range(n_layers)]
    # [layer][step][sequence][head][D]: step s uses the token at position P + s - 1
    def stack(i):
        return np.stack([np.stack([toks[l][b][i][P - 1:P - 1 + S] for b in range(n)], axis=1) for l in range(n_layers)])
    q_all, k_all, v_all = (to_device(stack(i), lp.dtype, DEV) for i in range(3))
    models = []
    for _ in range(2):
        mb = ModelBatch(lp, n_layers, DEV)
        for l in range(n_layers):
            for b in range(n):
                _, k, v = toks[l][b]
                st = oracle.CacheState.from_prefix(cfg, k[:P], v[:P])
                load_state(mb, l * n + b, st, cfg, 0)
        mb.upload_seqs()
        models.append(mb)
    eager, graphed = models

    def launch_step(mb, row_end, q_of, k_of, v_of):
        mb.select_all(flags=B.FLAG_PLAN_APPEND)
        for l in range(n_layers):
            mb.attend_layer(l, q_of(l), k_new=k_of(l), v_new=v_of(l),
                            flags=B.FLAG_APPEND | (0 if row_end else B.FLAG_ADVANCE))
        if row_end:
            mb.compact_all(flags=B.FLAG_ADVANCE)

    def is_row_end(s):
        return s >= 1 and (s - 1) % W == W - 1

    step_idx = torch.zeros(1, dtype=torch.int64, device=DEV)
    q_in, k_in, v_in = (torch.zeros((n_layers, 1) + tuple(x.shape[2:]), dtype=x.dtype, device=DEV) for x in (q_all, k_all, v_all))
    torch.index_select(q_all, 1, step_idx, out=q_in)             # first use of these kernels outside the capture
    step_idx.add_(0)
    launch_step(ModelBatch(lp, n_layers, DEV), True, lambda l: q_in[l, 0], lambda l: k_in[l, 0], lambda l: v_in[l, 0])
    torch.cuda.synchronize()
    graphs = {}
    for row_end in (False, True):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            torch.index_select(q_all, 1, step_idx, out=q_in)
            torch.index_select(k_all, 1, step_idx, out=k_in)
            torch.index_select(v_all, 1, step_idx, out=v_in)
            step_idx.add_(1)
            launch_step(graphed, row_end, lambda l: q_in[l, 0], lambda l: k_in[l, 0], lambda l: v_in[l, 0])
        graphs[row_end] = g
    torch.cuda.synchronize()
    assert (graphed.read_seqs()["step"] == 0).all() and int(step_idx) == 0          # capturing ran nothing
    n_row_ends = 0
    for s in range(S):
        graphs[is_row_end(s)].replay()
        launch_step(eager, is_row_end(s), lambda l: q_all[l, s], lambda l: k_all[l, s], lambda l: v_all[l, s])
        torch.cuda.synchronize()
        a, b = eager.read_seqs(), graphed.read_seqs()
        for f in ("n_res", "step", "status", "compacted", "pending_slot"):
            assert np.array_equal(a[f], b[f]), (s, f)
        assert (a["status"] == 0).all() and (a["step"] == s + 1).all(), s
        n_row_ends += int(is_row_end(s))
        assert torch.equal(eager.sel_cnt, graphed.sel_cnt), s
        for i in range(n_layers * n):
            c = int(eager.sel_cnt[i])
            assert torch.equal(eager.sel_idx[i, :c], graphed.sel_idx[i, :c]), s
        assert torch.equal(eager.out, graphed.out) and torch.equal(eager.lse, graphed.lse), s
        assert torch.equal(eager.K, graphed.K) and torch.equal(eager.V, graphed.V), s
        assert torch.equal(eager.pos, graphed.pos) and torch.equal(eager.score, graphed.score), s
    assert n_row_ends == H and int(step_idx) == S
    assert np.isfinite(to_host(graphed.out)).all()
