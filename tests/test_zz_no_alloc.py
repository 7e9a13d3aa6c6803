"""adsa_step_static -- the entry point for callers that cannot allocate -- against adsa_step.

Both run the same kernels; the only difference is where the scratch lives (the library's built-in
array instead of a caller workspace), so everything the step produces must be IDENTICAL: attended
sets, keep maps, cache rows, scores, outputs.  Two calls in a row through the raw C ABI, the second
with a smaller problem (fewer sequences, a shorter cache), so the second call finds the array full
of the first call's leftovers.  The shapes are small batches on purpose: their lists are split over
several workgroups, which hand partial results over through the scratch memory.
"""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2506_18226_amd import binding as B
from paper_2506_18226_amd import workloads as WL
from paper_2506_18226_amd.batch import LayerBatch, to_device

pytestmark = pytest.mark.gpu


def _run_steps(n_seq, grid_w, cap, n_steps, static, seed):
    """n_steps decode steps from the prefix-only cache; returns everything the steps produced."""
    dev = "cuda:0"
    h, D, P = 8, 64, 24
    p = B.make_params(n_seq=n_seq, n_heads=h, head_dim=D, grid_h=8, grid_w=grid_w, win_rows_back=1, win_col_radius=2,
                      dtype=B.F32, score_mode=B.SCORE_ATTN_MASS, cap=cap, sel_cap=cap)
    assert 0 < B.adsa_workspace_bytes(p) <= B.STATIC_SCRATCH_BYTES
    lb = LayerBatch(p, dev)
    rng = np.random.default_rng(seed)
    L = P + n_steps
    q = (rng.standard_normal((n_seq, L, h, D)) / 8).astype(np.float32)
    k = (rng.standard_normal((n_seq, L, h, D)) / 8).astype(np.float32)
    v = rng.standard_normal((n_seq, L, h, D)).astype(np.float32)
    for b in range(n_seq):
        lb.set_sequence(b, k=k[b, :P], v=v[b, :P], pos=np.arange(P, dtype=np.int32), score=None, step=0, grid_origin=P,
                        budget=12 + 4 * b)
    lb.upload_seqs()
    qd, kd, vd = (to_device(x, B.F32, dev) for x in (q, k, v))
    lib = B.load_library()
    stream = torch.cuda.current_stream().cuda_stream
    outs = []
    for s in range(n_steps):
        t = P + s - 1
        qs, ks, vs = qd[:, t].contiguous(), kd[:, t].contiguous(), vd[:, t].contiguous()
        args = [C.byref(p), lb.seqs.data_ptr(), qs.data_ptr(), ks.data_ptr(), vs.data_ptr(), lb.out.data_ptr(),
                lb.lse.data_ptr(), lb.sel_idx.data_ptr(), lb.sel_cnt.data_ptr(), lb.keep_map.data_ptr(), 0]
        if static:
            rc = lib.adsa_step_static(*args, stream)
        else:
            rc = lib.adsa_step(*args, lb.workspace.data_ptr(), lb.workspace.numel(), stream)
        assert rc == 0, B.strerror(rc)
        torch.cuda.synchronize()
        outs.append((lb.out.cpu().numpy().copy(), lb.lse.cpu().numpy().copy(), lb.sel_idx.cpu().numpy().copy(),
                     lb.sel_cnt.cpu().numpy().copy(), lb.keep_map.cpu().numpy().copy()))
    seqs = lb.read_seqs()
    assert (seqs["status"] == 0).all()
    final = (lb.K.cpu().numpy().copy(), lb.V.cpu().numpy().copy(), lb.score.cpu().numpy().copy(), lb.pos.cpu().numpy().copy(),
             seqs["n_res"].copy(), seqs["step"].copy())
    return outs, final


def _same(a, b, what):
    for i, (x, y) in enumerate(zip(a, b)):
        assert np.array_equal(x, y), f"{what}: item {i} differs between adsa_step_static and adsa_step"


def test_static_scratch_step_equals_workspace_step_on_two_calls_the_second_smaller():
    # (sequences, grid width, cap, steps): the second problem is smaller in every size
    for call, (n_seq, grid_w, cap, n_steps) in enumerate([(3, 8, 96, 20), (1, 4, 64, 11)]):
        ref_steps, ref_final = _run_steps(n_seq, grid_w, cap, n_steps, static=False, seed=100 + call)
        got_steps, got_final = _run_steps(n_seq, grid_w, cap, n_steps, static=True, seed=100 + call)
        for s, (r, g) in enumerate(zip(ref_steps, got_steps)):
            cnt = r[3]
            assert np.array_equal(g[3], cnt), f"call {call} step {s}: sel_cnt"
            for b in range(n_seq):
                assert np.array_equal(g[2][b, :cnt[b]], r[2][b, :cnt[b]]), f"call {call} step {s}: attended set"
            assert np.array_equal(g[4], r[4]), f"call {call} step {s}: keep_map"
            assert np.array_equal(g[0], r[0]) and np.array_equal(g[1], r[1]), f"call {call} step {s}: out / lse"
        _same(got_final, ref_final, f"call {call}: final cache state")


def test_static_scratch_rejects_what_does_not_fit():
    lib = B.load_library()
    # V-cosine ranking over a long cache of many wide sequences needs far more than the built-in array
    p = B.make_params(n_seq=64, n_heads=32, head_dim=128, grid_h=64, grid_w=64, win_rows_back=1, win_col_radius=2,
                      dtype=B.BF16, score_mode=B.SCORE_VCOS, cap=4096, sel_cap=4096)
    assert B.adsa_workspace_bytes(p) > B.STATIC_SCRATCH_BYTES
    t = torch.zeros(4096, dtype=torch.uint8, device="cuda:0")      # never dereferenced: the size check comes first
    a = t.data_ptr()
    rc = lib.adsa_step_static(C.byref(p), a, a, a, a, a, a, a, a, a, 0, None)
    assert rc == -9 and "built-in" in B.strerror(rc)
