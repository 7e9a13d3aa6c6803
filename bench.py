#!/usr/bin/env python3
"""Benchmark of the ADSA decode hot path on one MI355X.

A "step" is one decode step of the whole workload: every layer's append, selection, gather
attention and score accumulation for every sequence, plus the row-end eviction + compaction when
the step closes a grid row.  The default workload is the LlamaGen-XXL-shaped configuration
(48 layers, 32 sequences, 24 heads x 64, bf16, 120 prefix + 32x32 grid, window prev-row +-4,
budget 512).  With no --steps the complete 1024-step trajectory is timed, free-running from the
prefix-only cache; --steps K times the LAST ceil(K / grid_w) grid rows of the trajectory (the
deepest contexts), i.e. K rounded up to whole rows so that every run contains its share of row-end
compactions -- the JSON line reports the number of steps actually timed ("steps") next to the
request ("steps_requested").  All inputs are resident in HBM before the clock starts.

Prints ONE JSON line: decode tokens/s (whole job), the HBM roofline of the attention kernel
(algorithmic selected-KV bytes / its HIP-event-timed duration), KV bytes resident, the same window
replayed as captured HIP graphs (one graph per decode step of all layers), and the CPU oracle
timed on a bounded sample of the same workload, which also re-checks sampled caches of the timed
run against the oracle.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0     # MI355X HBM3E peak


def measured_traffic_ratio(workload):
    """HBM bytes / algorithmic bytes of the attention kernel from the committed rocprofv3 --pmc summary
    (FETCH_SIZE + WRITE_SIZE, scaled by a plain copy), or None if there is none for this workload."""
    path = os.path.join(ROOT, "profiles", f"{workload}_attend_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("k_attend_traffic_over_algorithmic:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0,
                    help="decode steps to time, rounded up to whole grid rows (0 = the whole trajectory)")
    ap.add_argument("--warmup", type=int, default=32, help="untimed decode steps before the timed region")
    ap.add_argument("--workload", default="xxl", choices=["tiny", "xl", "xxl", "long", "ragged", "gqa"])
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (debugging only)")
    ap.add_argument("--replicas", type=int, default=0,
                    help="single-layer workloads (long, ragged): independent copies of the state that the run rotates "
                         "through, so that the working set cannot sit in the memory-side cache (default 8)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-roofline-pass", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay of the timed window")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="CPU time budget of the oracle sample")
    ap.add_argument("--paper-cache", action="store_true",
                    help="run the paper's own cache policy instead of the headline one: capacity = prefix + half the "
                         "image tokens, V-cosine ranking (Eq. 2-3), evict one when full, 1-D window, dense attention "
                         "over everything resident (Section 4.2, Tables 1-2); the incoming token takes the evicted slot")
    ap.add_argument("--two-pass-vcos", action="store_true",
                    help="with --paper-cache: rank with two passes over V per step (ADSA_SCORE_VCOS) instead of the numbers "
                         "the attention launch leaves behind (ADSA_SCORE_VCOS_FUSED)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain device copy of known size (1 GiB read + 1 GiB written, 4 times): the "
                         "reference that scales rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    return ap.parse_args()


class Job:
    """All device state of a trajectory benchmark: every layer's caches as one layer-major batch,
    step-major inputs, and the per-step launch sequence.  For a single-layer workload the "layers" are
    independent replicas of the state."""

    def __init__(self, wl, n_layers, device, paper_cache=False, two_pass_vcos=False):
        import torch
        from paper_2506_18226_amd import binding as B
        from paper_2506_18226_amd import workloads as WL
        from paper_2506_18226_amd.batch import ModelBatch

        self.torch, self.B, self.wl, self.n_layers, self.device = torch, B, wl, n_layers, device
        P, n, h, D = wl.prefix_len, wl.n_seq, wl.n_heads, wl.head_dim
        self.n_steps_total = wl.n_image_tokens          # s = 0 .. H*W-1
        self.paper_cache = paper_cache
        if paper_cache:      # Section 4.2 as written: half-length cache, evict one when full, TopK-V ranking
            cap = P + wl.n_image_tokens // 2
            self.layer_params = B.make_params(
                n_seq=n, n_heads=h, head_dim=D, grid_h=wl.grid_h, grid_w=wl.grid_w, win_rows_back=0,
                win_col_radius=0, dtype=B.F32 if wl.dtype == "f32" else B.BF16,
                score_mode=B.SCORE_VCOS if two_pass_vcos else B.SCORE_VCOS_FUSED,
                cap=cap, sel_cap=cap, win_recent_m=2 * wl.grid_w + 1, evict_policy=B.EVICT_REUSE_SLOT,
                q_per_kv=wl.q_per_kv)
        else:
            self.layer_params = B.make_params(
                n_seq=n, n_heads=h, head_dim=D, grid_h=wl.grid_h, grid_w=wl.grid_w,
                win_rows_back=wl.win_rows_back, win_col_radius=wl.win_col_radius,
                dtype=B.F32 if wl.dtype == "f32" else B.BF16, score_mode=wl.score_mode,
                cap=wl.cap(), sel_cap=wl.sel_cap(), q_per_kv=wl.q_per_kv)
        mb = self.mb = ModelBatch(self.layer_params, n_layers, device)
        S = self.n_steps_total
        hq = h * wl.q_per_kv
        tdt = mb.K.dtype
        # step s queries with the token at position P+s-1: [layer][step 0 .. S][n][heads][D] (one step beyond the
        # trajectory, s = H*W, for the re-check against the oracle)
        self.q_all = torch.empty((n_layers, S + 1, n, hq, D), dtype=tdt, device=device)
        self.kn_all = torch.empty((n_layers, S + 1, n, h, D), dtype=tdt, device=device)
        self.vn_all = torch.empty((n_layers, S + 1, n, h, D), dtype=tdt, device=device)
        for l in range(n_layers):
            qd, kd, vd = WL.gen_tokens_device(wl, l, device)        # [n][L][h][D]
            mb.K[l * n:(l + 1) * n, :, :P] = kd[:, :P].transpose(1, 2)      # [head][slot][D] caches
            mb.V[l * n:(l + 1) * n, :, :P] = vd[:, :P].transpose(1, 2)
            self.q_all[l] = qd[:, P - 1:P + S].permute(1, 0, 2, 3)
            self.kn_all[l] = kd[:, P - 1:P + S].permute(1, 0, 2, 3)
            self.vn_all[l] = vd[:, P - 1:P + S].permute(1, 0, 2, 3)
            del qd, kd, vd
        mb.pos[:, :P] = torch.arange(P, dtype=torch.int32, device=device)[None, :]
        self.sel_cnt_log = torch.zeros((S + 1, n_layers * n), dtype=torch.int32, device=device)
        self.row_bytes = n * h * D * mb.K.element_size()
        self.q_row_bytes = self.row_bytes * wl.q_per_kv
        self.graphs = None
        self.reset()

    def reset(self):
        wl, P, mb = self.wl, self.wl.prefix_len, self.mb
        for s in mb.seqs_host:
            s["n_res"], s["step"], s["grid_origin"], s["n_keep_prefix"] = P, 0, P, P
            s["budget"], s["budget_num"], s["budget_den"] = wl.budget, wl.budget_num, wl.budget_den
            s["status"], s["compacted"], s["pending_slot"], s["hole"] = 0, 0, -1, 0
        mb.upload_seqs()
        mb.score.zero_()
        if mb.vcos_u is not None:
            mb.vcos_u.zero_()
        self.sel_cnt_log.zero_()
        self.torch.cuda.synchronize()

    def is_row_end(self, s):
        W = self.wl.grid_w
        return (not self.paper_cache) and s >= 1 and (s - 1) % W == W - 1

    def _launch_step(self, s, q_of, kn_of, vn_of, cnt_ptr):
        """The launch sequence of decode step s.  q_of(l) etc. give layer l's input pointers.  ONE selection
        launch for every layer's sequences (it does not depend on q/k/v), one attention launch per layer
        (append + gather attention + merge + score update), and at row ends ONE eviction/compaction launch
        pair for every layer."""
        B, mb = self.B, self.mb
        stream = self.torch.cuda.current_stream().cuda_stream
        n, L = self.wl.n_seq, self.n_layers
        lp, tp = mb.layer_params, mb.params
        seqs0, sel0 = mb.seqs.data_ptr(), mb.sel_idx.data_ptr()
        out0, lse0 = mb.out.data_ptr(), mb.lse.data_ptr()
        seq_sz, sel_row = B.SEQ_DTYPE.itemsize, lp.sel_cap * 4
        hq = B.query_heads(lp)
        out_row, lse_row = n * hq * lp.head_dim * mb.out.element_size(), n * hq * 4
        row_end = self.is_row_end(s)
        if self.paper_cache and s >= 1:
            # evict-one-if-full for every layer, then plan, then the layers; nothing happens at row ends
            B.adsa_compact(tp, seqs0, mb.keep_map, mb.workspace, 0, stream)
        B.adsa_select(tp, seqs0, sel0, cnt_ptr, None, B.FLAG_PLAN_APPEND, stream)
        flags = B.FLAG_APPEND | (0 if row_end else B.FLAG_ADVANCE)
        for l in range(L):
            B.adsa_attend(lp, seqs0 + l * n * seq_sz, q_of(l), sel0 + l * n * sel_row, cnt_ptr + l * n * 4,
                          out0 + l * out_row, lse0 + l * lse_row, mb.layer_workspace, flags,
                          kn_of(l), vn_of(l), stream)
        if row_end:
            B.adsa_compact(tp, seqs0, mb.keep_map, mb.workspace, B.FLAG_ADVANCE, stream)

    def run(self, s_begin, s_end, on_row_end=None):
        """Enqueue decode steps s_begin .. s_end-1 (no host sync inside)."""
        S1 = self.n_steps_total + 1
        q0, k0, v0 = self.q_all.data_ptr(), self.kn_all.data_ptr(), self.vn_all.data_ptr()
        L, n = self.n_layers, self.wl.n_seq
        cnt0 = self.sel_cnt_log.data_ptr()
        for s in range(s_begin, s_end):
            self._launch_step(s, lambda l: q0 + (l * S1 + s) * self.q_row_bytes,
                              lambda l: k0 + (l * S1 + s) * self.row_bytes,
                              lambda l: v0 + (l * S1 + s) * self.row_bytes, cnt0 + s * L * n * 4)
            if on_row_end is not None and self.is_row_end(s):
                on_row_end(s)

    # ---- the same steps as captured HIP graphs: one graph per decode step of ALL layers
    def build_graphs(self):
        """Two graphs (a step that closes a grid row, and any other step).  Inputs reach fixed staging buffers
        through a captured gather indexed by a device-side step counter, as a model's projection kernels would
        leave them; every state-dependent decision of the path is taken on the device."""
        torch = self.torch
        L, n = self.n_layers, self.wl.n_seq
        self.step_idx = torch.zeros(1, dtype=torch.int64, device=self.device)
        self.q_in = torch.empty((L, 1) + tuple(self.q_all.shape[2:]), dtype=self.q_all.dtype, device=self.device)
        self.kn_in = torch.empty((L, 1) + tuple(self.kn_all.shape[2:]), dtype=self.kn_all.dtype, device=self.device)
        self.vn_in = torch.empty_like(self.kn_in)
        self.cnt_in = torch.zeros(L * n, dtype=torch.int32, device=self.device)
        torch.index_select(self.q_all, 1, self.step_idx, out=self.q_in)      # first use of these kernels: outside the capture
        self.step_idx.add_(0)
        torch.cuda.synchronize()
        qp, kp, vp = self.q_in.data_ptr(), self.kn_in.data_ptr(), self.vn_in.data_ptr()
        graphs = {}
        for row_end in (False, True):
            s_like = self.wl.grid_w if row_end else 1        # any step of that kind: only the kind is captured
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                torch.index_select(self.q_all, 1, self.step_idx, out=self.q_in)
                torch.index_select(self.kn_all, 1, self.step_idx, out=self.kn_in)
                torch.index_select(self.vn_all, 1, self.step_idx, out=self.vn_in)
                self.step_idx.add_(1)
                self._launch_step(s_like, lambda l: qp + l * self.q_row_bytes, lambda l: kp + l * self.row_bytes,
                                  lambda l: vp + l * self.row_bytes, self.cnt_in.data_ptr())
            graphs[row_end] = g
        self.graphs = graphs

    def run_graph(self, s_begin, s_end):
        self.step_idx.fill_(s_begin)
        for s in range(s_begin, s_end):
            self.graphs[self.is_row_end(s)].replay()


class RaggedJob:
    """The ragged serving batch: 64 sequences, each at its own decode position, prefix length and budget, advanced
    by ONE adsa_step call per decode step; `replicas` independent copies of the batch are stepped in turn."""

    def __init__(self, wl, replicas, n_steps, device):
        import numpy as np
        import torch
        from paper_2506_18226_amd import binding as B
        from paper_2506_18226_amd import workloads as WL
        from paper_2506_18226_amd.batch import LayerBatch, to_device

        self.torch, self.B, self.wl, self.replicas, self.n_steps = torch, B, wl, replicas, n_steps
        n, h, D = wl.n_seq, wl.n_heads, wl.head_dim
        cap = 120 + 512 + 2 * wl.grid_w
        sel_cap = 120 + 512 + wl.grid_w + wl.win_rows_back * (2 * wl.win_col_radius + 1)
        self.params = B.make_params(n_seq=n, n_heads=h, head_dim=D, grid_h=wl.grid_h, grid_w=wl.grid_w,
                                    win_rows_back=wl.win_rows_back, win_col_radius=wl.win_col_radius, dtype=B.BF16,
                                    score_mode=wl.score_mode, cap=cap, sel_cap=sel_cap)
        self.batches = [LayerBatch(self.params, device) for _ in range(replicas)]
        last = wl.n_image_tokens - n_steps          # a sequence drawn deeper than this starts here instead
        q_in = np.zeros((n_steps, n, h, D), np.float32)
        k_in, v_in = np.zeros_like(q_in), np.zeros_like(q_in)
        self.states = []
        for b in range(n):
            P, Bud, s = WL.seq_geometry(wl, b)
            s = min(s, last)
            syn = WL.synthetic_state(wl, 0, b, s, prefix_len=P, budget=Bud)
            q, k, v = WL.gen_tokens(wl, 0, b, prefix_len=P)
            for t in range(n_steps):
                p = P + s + t - 1
                q_in[t, b], k_in[t, b], v_in[t, b] = q[p], k[p], v[p]
            self.states.append((P, Bud, s, syn["k"], syn["v"], syn["pos"], syn["score"]))
        self.q, self.kn, self.vn = (to_device(x, B.BF16, device) for x in (q_in, k_in, v_in))
        self.cnt_log = torch.zeros((replicas, n_steps, n), dtype=torch.int32, device=device)
        self.load()

    def load(self):
        """(Re)load every replica with the start states."""
        for lb in self.batches:
            for b, (P, Bud, s, k, v, pos, score) in enumerate(self.states):
                lb.set_sequence(b, k=k, v=v, pos=pos, score=score, step=s, grid_origin=P, budget=Bud)
            lb.upload_seqs()
        self.torch.cuda.synchronize()

    def run(self):
        B = self.B
        stream = self.torch.cuda.current_stream().cuda_stream
        for t in range(self.n_steps):
            for r, lb in enumerate(self.batches):
                B.adsa_step(self.params, lb.seqs, self.q[t], self.kn[t], self.vn[t], lb.out, lb.lse, lb.sel_idx,
                            self.cnt_log[r, t], lb.keep_map, lb.workspace, 0, stream)


def oracle_cfg_for(wl, P=None, budget=None, cap=None):
    import oracle
    P = wl.prefix_len if P is None else P
    frac = wl.budget_den > 0 and budget is None
    return oracle.make_cfg(n_heads=wl.n_heads, head_dim=wl.head_dim, grid_h=wl.grid_h, grid_w=wl.grid_w,
                           win_rows_back=wl.win_rows_back, win_col_radius=wl.win_col_radius, grid_origin=P,
                           budget=0 if frac else (wl.budget if budget is None else budget),
                           budget_num=wl.budget_num if frac else 0, budget_den=wl.budget_den if frac else 0,
                           score_mode=wl.score_mode, cap=wl.cap() if cap is None else cap, q_per_kv=wl.q_per_kv)


def cpu_baseline(wl, n_layers_real, seconds, job=None):
    """The oracle as it stands, one thread, on whole single-(layer, sequence) trajectories -- and, with the
    trajectory job of the timed run at hand, one more decode step of sampled (layer, sequence) caches of that
    run on both sides (the GPU's own state handed to the oracle), as a check of what was timed."""
    import numpy as np
    import oracle
    from paper_2506_18226_amd import workloads as WL

    P = wl.prefix_len
    cfg = oracle_cfg_for(wl)
    done, spent = 0, 0.0
    seq = 0
    while spent < seconds and seq < wl.n_seq:
        q, k, v = WL.gen_tokens(wl, 0, seq)
        st = oracle.CacheState.from_prefix(cfg, k[:P], v[:P])
        t0 = time.perf_counter()
        for s in range(wl.n_image_tokens):
            p = P + s - 1
            oracle.step(cfg, st, s, q[p], k[p], v[p])
        spent += time.perf_counter() - t0
        done += wl.n_image_tokens
        seq += 1
    seq_layer_steps_per_s = done / spent
    res = {
        "value": seq_layer_steps_per_s / n_layers_real, "unit": "tokens/s", "cores": 1, "kind": "oracle",
        "sample": f"complete {wl.n_image_tokens}-step trajectories of {seq} of the {wl.n_seq * n_layers_real} "
                  f"(sequence, layer) caches, {spent:.1f} s of CPU time, scaled by 1/{n_layers_real} layers",
        "host_cpus": os.cpu_count(), "cpu_model": cpu_model(),
    }
    if job is not None and not job.paper_cache and wl.q_per_kv == 1:
        res["verify"] = verify_against_oracle(job, cfg)
    return res


def verify_against_oracle(job, cfg):
    """After the timed trajectory (all sequences at step S = H*W, the final token): sampled (layer, sequence)
    caches go to the host as they are, the GPU runs step S for everything, the oracle runs it on the samples.
    Both rank the same fp32 scores, so the attended sets must be identical; outputs within the bf16 bar."""
    import numpy as np
    import oracle
    torch, mb, wl = job.torch, job.mb, job.wl
    n, L, S, P = wl.n_seq, job.n_layers, job.n_steps_total, wl.prefix_len
    seqs = mb.read_seqs()
    if not (seqs["step"] == S).all():
        return {"skipped": "the job is not at the end of its trajectory"}
    samples = sorted({(0, 0), (L // 2, n // 2), (L - 1, n - 1)})
    snaps = {}
    for (l, b) in samples:
        i = l * n + b
        nr = int(seqs["n_res"][i])
        K = mb.K[i, :, :nr].float().cpu().numpy().transpose(1, 0, 2)        # [slot][head][D]
        V = mb.V[i, :, :nr].float().cpu().numpy().transpose(1, 0, 2)
        rows = mb.score[i, :, :nr].cpu().numpy()
        rank = rows[0].copy()
        for r in range(1, rows.shape[0]):                                   # the kernels' order: ascending rows, fp32
            rank = (rank + rows[r]).astype(np.float32)
        snaps[(l, b)] = (K, V, mb.pos[i, :nr].cpu().numpy().copy(), rank)
    job.run(S, S + 1)                                                       # s = H*W: the last grid token, a row end
    torch.cuda.synchronize()
    seqs = mb.read_seqs()
    cnt = job.sel_cnt_log[S].cpu().numpy()
    worst, sel_same, nres_same, map_same = 0.0, True, True, True
    for (l, b) in samples:
        i = l * n + b
        K, V, pos, rank = snaps[(l, b)]
        st = oracle.CacheState.from_arrays(cfg, K, V, pos, rank)
        qh = job.q_all[l, S, b].float().cpu().numpy()
        kh = job.kn_all[l, S, b].float().cpu().numpy()
        vh = job.vn_all[l, S, b].float().cpu().numpy()
        ref = oracle.step(cfg, st, S, qh, kh, vh)
        sel = mb.sel_idx[i, :int(cnt[i])].cpu().numpy()
        sel_same &= bool(np.array_equal(sel, ref["sel_idx"]))
        out = mb.out[i].float().cpu().numpy().astype(np.float64)
        row_ref = np.abs(ref["out"]).max(axis=1, keepdims=True)
        worst = max(worst, float((np.abs(out - ref["out"]) / row_ref).max()))
        nres_same &= int(seqs["n_res"][i]) == st.n_res
        if ref["keep_map"] is not None:
            km = mb.keep_map[i, :ref["keep_map"].size].cpu().numpy()
            map_same &= bool(np.array_equal(km, ref["keep_map"]))
    return {"samples": [list(x) for x in samples], "step": S, "attended_sets_identical": sel_same,
            "out_max_rel_err": worst, "out_within_bf16_bar": worst <= 2e-2, "n_res_identical": nres_same,
            "keep_maps_identical": map_same,
            "ok": bool(sel_same and worst <= 2e-2 and nres_same)}


def workload_text(wl, n_layers, args, job_params, replicas):
    txt = (f"{wl.name}: {n_layers} layers x {wl.n_seq} sequences, {wl.n_heads} heads x {wl.head_dim}"
           + (f" with {wl.q_per_kv} query heads each" if wl.q_per_kv > 1 else "") + f", "
           f"{wl.dtype}, prefix {wl.prefix_len} + {wl.grid_h}x{wl.grid_w} grid, window R={wl.win_rows_back} "
           f"w={wl.win_col_radius}, budget "
           + (f"{wl.budget}" if wl.budget_den == 0 else f"{wl.budget_num}/{wl.budget_den} of context"))
    if replicas > 1:
        txt = txt.replace(f"{n_layers} layers", f"1 layer ({replicas} independent replicas of the state, stepped in turn)")
    if args.paper_cache:
        txt += (f"; PAPER CACHE POLICY: capacity {job_params.cap}, V-cosine ranking "
                + ("(two passes over V per step)" if args.two_pass_vcos else "(fused into the attention launch)")
                + f", evict one when full (the incoming token takes its slot), 1-D window of "
                  f"{job_params.win_recent_m}, attention over everything resident")
    else:
        txt += ", ranking=accumulated attention mass, row-end eviction"
    return txt


def other_algorithmic_bytes(wl, att_bytes, n_launch):
    e = 2 if wl.dtype == "bf16" else 4
    tokens = att_bytes / wl.token_bytes / max(1, n_launch)              # attended tokens per launch, all sequences
    per_token = 4 + (8 * wl.n_heads if wl.score_mode == 0 else 0)
    hq = wl.n_heads * max(wl.q_per_kv, 1)
    per_seq = 2 * hq * wl.head_dim * e + 2 * wl.n_heads * wl.head_dim * e + 4 * hq
    return tokens * per_token + wl.n_seq * per_seq


def roofline_block(wl, att_bytes, n_launch, att_ms, flops=None):
    achieved = att_bytes / (att_ms * 1e-3) / 1e9
    ratio = measured_traffic_ratio(wl.name)
    r = {
        "kernel": "k_attend" if wl.q_per_kv == 1 else "k_attend_gqa", "bound": "hbm", "achieved": achieved,
        "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
        "traffic": None if ratio is None else ratio * att_bytes / max(1, n_launch),
        "traffic_source": None if ratio is None else
        f"profiles/{wl.name}_attend_hbm_traffic.txt: measured HBM bytes / algorithmic bytes = {ratio} x this run's bytes per launch",
        "launches": int(n_launch), "avg_launch_us": 1e3 * att_ms / max(1, n_launch),
        "algorithmic_bytes_per_launch": att_bytes / max(1, n_launch),
        # what else one launch must move, by the same kind of count: per attended token its slot-list entry (4 B) and,
        # with attention-mass ranking, one score word read and written per cache head; per sequence q, out, the
        # appended k/v rows and lse
        "other_algorithmic_bytes_per_launch": other_algorithmic_bytes(wl, att_bytes, n_launch),
    }
    if flops is not None:        # the contraction runs on the matrix cores: 4 flops per (query head, token, column)
        r["mfma_tflops"] = flops / (att_ms * 1e-3) / 1e12
        r["mfma_frac_of_bf16_peak"] = flops / (att_ms * 1e-3) / 2.5e15
    return r


def main_ragged(args, wl, device):
    import numpy as np
    import torch
    from paper_2506_18226_amd import binding as B

    replicas = args.replicas if args.replicas > 0 else 8
    K = args.steps if args.steps > 0 else 16
    t_setup = time.perf_counter()
    job = RaggedJob(wl, replicas, K, device)
    torch.cuda.synchronize()
    t_setup = time.perf_counter() - t_setup
    job.run()                                           # warm-up pass over the same steps
    torch.cuda.synchronize()
    job.load()
    t0 = time.perf_counter()
    job.run()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    for lb in job.batches:
        assert (lb.read_seqs()["status"] == 0).all(), "a sequence reported a device-side error"
    calls = K * replicas
    cnt = job.cnt_log.cpu().numpy().astype(np.int64)
    tau = wl.token_bytes
    result = {
        "metric": "adsa_decode_tokens_per_s", "value": wl.n_seq * calls / elapsed, "unit": "tokens/s",
        "n_gpus": 1, "steps": calls, "steps_requested": args.steps, "warmup": calls, "ms_per_step": 1e3 * elapsed / calls,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {
            "workload": f"ragged: 1 layer x {wl.n_seq} sequences at decode positions U[1,{wl.n_image_tokens}] (capped at "
                        f"{wl.n_image_tokens - K} so that {K} steps fit), prefix U[16,120], budget from {{128,256,384,512}}, "
                        f"{wl.n_heads} heads x {wl.head_dim}, bf16, {wl.grid_h}x{wl.grid_w} grid, window R={wl.win_rows_back} "
                        f"w={wl.win_col_radius}; one adsa_step call per decode step; {replicas} independent replicas of the "
                        f"batch stepped in turn (a step = one adsa_step call)",
            "global_batch": wl.n_seq, "layers": 1, "replicas": replicas, "setup_seconds": round(t_setup, 1),
        },
        "selected_kv_gb_per_step": int(cnt.sum()) * tau / calls / 1e9,
        "selected_kv_gbs_whole_path": int(cnt.sum()) * tau / elapsed / 1e9,
    }
    if not args.no_roofline_pass:
        job.load()
        B.adsa_profile_enable(True)
        job.run()
        torch.cuda.synchronize()
        n_launch, att_ms = B.adsa_profile_read()
        B.adsa_profile_enable(False)
        cnt2 = job.cnt_log.cpu().numpy().astype(np.int64)
        result["roofline"] = roofline_block(wl, int(cnt2.sum()) * tau, n_launch, att_ms)
    print(json.dumps(result))


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    from paper_2506_18226_amd import binding as B
    from paper_2506_18226_amd import workloads as WL

    B.load_library()                                   # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    device = "cuda:0"
    if args.calibrate_copy:
        src = torch.ones(1 << 29, dtype=torch.bfloat16, device=device)      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": src.numel() * 2, "calibrate_copy_bytes_written": src.numel() * 2,
                          "copies": 4}))
        return
    wl = WL.get_workload(args.workload)
    if wl.ragged:
        return main_ragged(args, wl, device)
    # a single-layer workload runs as several independent replicas of its state, so that it streams from HBM
    replicas = 1
    if wl.n_layers == 1 and wl.name != "tiny":
        replicas = args.replicas if args.replicas > 0 else 8
    n_layers = args.layers if args.layers > 0 else wl.n_layers * replicas
    t_setup = time.perf_counter()
    job = Job(wl, n_layers, device, paper_cache=args.paper_cache, two_pass_vcos=args.two_pass_vcos)
    torch.cuda.synchronize()
    t_setup = time.perf_counter() - t_setup
    S, W = job.n_steps_total, wl.grid_w
    # the timed window: the whole trajectory, or the last ceil(K / W) grid rows of it
    K = S if args.steps <= 0 else min(S, -(-args.steps // W) * W)
    Wm = max(0, args.warmup)

    # warm-up: Wm steps, then start again from the prefix-only cache and run up to the window
    job.run(0, min(Wm, S))
    torch.cuda.synchronize()
    job.reset()
    s0 = S - K
    if s0 > 0:
        job.run(0, s0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    job.run(s0, S)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    assert (job.mb.read_seqs()["status"] == 0).all(), "a sequence reported a device-side error"
    cnt_log = job.sel_cnt_log.cpu().numpy().astype(np.int64)           # [S + 1][layers * n_seq]
    out_eager = job.mb.out.clone()
    nres_eager = job.mb.read_seqs()["n_res"].copy()
    tau = wl.token_bytes
    tokens = wl.n_seq * K * replicas
    result = {
        "metric": "adsa_decode_tokens_per_s", "value": tokens / elapsed, "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "steps_requested": args.steps, "warmup": Wm, "ms_per_step": 1e3 * elapsed / K,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if wl.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {
            "workload": workload_text(wl, n_layers, args, job.layer_params, replicas),
            "decode_steps_timed": [s0, S], "row_end_compactions_in_window": sum(job.is_row_end(s) for s in range(s0, S)),
            "global_batch": wl.n_seq, "layers": n_layers // replicas, "replicas": replicas, "setup_seconds": round(t_setup, 1),
        },
    }
    if replicas > 1:
        result["config"]["note"] = (f"ms_per_step covers one decode step of all {replicas} replicas; tokens/s counts "
                                    f"{replicas} x {wl.n_seq} tokens per step")
    # classifier-free guidance runs two sequences (conditional / unconditional, separate caches) per image
    result["image_tokens_per_s_under_cfg_pairing"] = tokens / elapsed / 2.0
    timed_attended = int(cnt_log[s0:S].sum())
    result["selected_kv_gb_per_step"] = timed_attended * tau / K / 1e9
    result["selected_kv_gbs_whole_path"] = timed_attended * tau / elapsed / 1e9

    # ---- roofline of the dominant kernel: same window again with HIP events around the attention kernel
    if not args.no_roofline_pass:
        job.reset()
        if s0 > 0:
            job.run(0, s0)
        torch.cuda.synchronize()
        n_peak = int(job.mb.read_seqs()["n_res"].astype(np.int64).sum())
        n_after = []

        def at_row_end(s):
            n_after.append((s, int(job.mb.read_seqs()["n_res"].astype(np.int64).sum())))

        B.adsa_profile_enable(True)
        job.run(s0, S, on_row_end=at_row_end)
        torch.cuda.synchronize()
        n_launch, att_ms = B.adsa_profile_read()
        B.adsa_profile_enable(False)
        cnt2 = job.sel_cnt_log.cpu().numpy().astype(np.int64)
        att_tokens = int(cnt2[s0:S].sum())
        flops = att_tokens * 4 * wl.n_heads * wl.q_per_kv * wl.head_dim if wl.q_per_kv > 1 else None
        result["roofline"] = roofline_block(wl, att_tokens * tau, n_launch, att_ms, flops)
        # KV bytes resident: between row ends every sequence grows by one slot per step; a compaction shrinks it
        dense = (wl.prefix_len + wl.n_image_tokens) * wl.n_seq * n_layers * tau
        n_end = int(job.mb.read_seqs()["n_res"].astype(np.int64).sum())
        after = dict(n_after)
        cur = peak = n_peak
        for s in range(s0, S):                             # every sequence appends one row per step s >= 1
            if s >= 1:
                cur += wl.n_seq * n_layers
            peak = max(peak, cur)
            if s in after:
                cur = after[s]
        if not job.paper_cache:
            assert cur == n_end, (cur, n_end)
        else:
            peak = n_end
        result["kv_bytes_resident"] = {
            "max": peak * tau, "after_last_compaction": (n_after[-1][1] if n_after else n_end) * tau,
            "dense_cache": dense, "ratio_max_to_dense": peak * tau / dense,
            "allocated": job.layer_params.cap * wl.n_seq * n_layers * tau,
        }

    # ---- the same window as captured HIP graphs (one replay = one decode step of all layers)
    if not args.no_graph and not args.paper_cache:
        try:
            job.reset()
            if s0 > 0:
                job.run(0, s0)
            torch.cuda.synchronize()
            job.build_graphs()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            job.run_graph(s0, S)
            torch.cuda.synchronize()
            g_elapsed = time.perf_counter() - t0
            same = bool(torch.equal(out_eager, job.mb.out)) and bool(
                np.array_equal(nres_eager, job.mb.read_seqs()["n_res"]))
            result["hip_graph"] = {
                "ms_per_step": 1e3 * g_elapsed / K, "eager_ms_per_step": 1e3 * elapsed / K,
                "tokens_per_s": tokens / g_elapsed, "speedup_over_eager": elapsed / g_elapsed,
                "identical_to_eager": same,
                "what": "one captured graph per decode step of all layers (select, one attention launch per layer, "
                        "compaction at row ends), inputs gathered into fixed staging buffers inside the graph",
            }
        except Exception as e:       # the graph leg must never cost the run its headline number
            result["hip_graph"] = {"error": f"{type(e).__name__}: {e}"[:300]}

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, wl.n_layers, args.cpu_seconds, job=job)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
