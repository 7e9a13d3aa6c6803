#!/usr/bin/env python3
"""Benchmark of the ADSA decode hot path on one MI355X.

A "step" is one decode step of the whole workload: every layer's adsa_step (append, select,
gather attention, score accumulation, and the row-end eviction + compaction when the step closes
a grid row) for every sequence.  The default workload is the LlamaGen-XXL-shaped configuration
(48 layers, 32 sequences, 24 heads x 64, bf16, 120 prefix + 32x32 grid, window prev-row +-4,
budget 512) and the default run times its complete 1024-step trajectory, free-running from the
prefix-only cache, with all inputs resident in HBM before the clock starts.

Prints ONE JSON line: decode tokens/s (whole job), the HBM roofline of the attention kernel
(algorithmic selected-KV bytes / its HIP-event-timed duration), KV bytes resident, and the CPU
oracle timed on a bounded sample of the same workload.
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
    """HBM bytes / algorithmic bytes of k_attend from the committed rocprofv3 --pmc summary
    (FETCH_SIZE + WRITE_SIZE, scaled by a plain copy), or None if there is none for this workload."""
    path = os.path.join(ROOT, "profiles", f"{workload}_attend_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("k_attend_traffic_over_algorithmic:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="decode steps to time (0 = the whole trajectory)")
    ap.add_argument("--warmup", type=int, default=32, help="untimed decode steps before the timed region")
    ap.add_argument("--workload", default="xxl", choices=["tiny", "xl", "xxl", "long", "gqa"])
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (debugging only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-roofline-pass", action="store_true")
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
    """All device state of the benchmark: every layer's caches as one layer-major batch,
    step-major inputs, and the per-step launch sequence."""

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
        self.q, self.kn, self.vn = [], [], []
        S = self.n_steps_total
        for l in range(n_layers):
            qd, kd, vd = WL.gen_tokens_device(wl, l, device)        # [n][L][h][D]
            mb.K[l * n:(l + 1) * n, :, :P] = kd[:, :P].transpose(1, 2)      # [head][slot][D] caches
            mb.V[l * n:(l + 1) * n, :, :P] = vd[:, :P].transpose(1, 2)
            # step s queries with the token at position P+s-1: step-major [S][n][h][D]
            self.q.append(qd[:, P - 1:P - 1 + S].permute(1, 0, 2, 3).contiguous())
            self.kn.append(kd[:, P - 1:P - 1 + S].permute(1, 0, 2, 3).contiguous())
            self.vn.append(vd[:, P - 1:P - 1 + S].permute(1, 0, 2, 3).contiguous())
            del qd, kd, vd
        mb.pos[:, :P] = torch.arange(P, dtype=torch.int32, device=device)[None, :]
        self.sel_cnt_log = torch.zeros((S, n_layers * n), dtype=torch.int32, device=device)
        self.row_bytes = n * h * D * mb.K.element_size()
        self.q_row_bytes = self.row_bytes * wl.q_per_kv
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

    def run(self, s_begin, s_end, on_row_end=None):
        """Enqueue decode steps s_begin .. s_end-1 (no host sync inside).  Per step: ONE selection
        launch for every layer's sequences (it does not depend on q/k/v), one attention launch per
        layer (append + gather attention + merge + score update), and at row ends ONE
        eviction/compaction launch pair for every layer."""
        B, wl, mb = self.B, self.wl, self.mb
        W = wl.grid_w
        stream = self.torch.cuda.current_stream().cuda_stream
        n, L = wl.n_seq, self.n_layers
        lp, tp = mb.layer_params, mb.params
        seqs0, sel0 = mb.seqs.data_ptr(), mb.sel_idx.data_ptr()
        out0, lse0 = mb.out.data_ptr(), mb.lse.data_ptr()
        qb = [t.data_ptr() for t in self.q]
        kb = [t.data_ptr() for t in self.kn]
        vb = [t.data_ptr() for t in self.vn]
        cnt0 = self.sel_cnt_log.data_ptr()
        seq_sz, sel_row = B.SEQ_DTYPE.itemsize, lp.sel_cap * 4
        hq = B.query_heads(lp)
        out_row, lse_row = n * hq * lp.head_dim * mb.out.element_size(), n * hq * 4
        for s in range(s_begin, s_end):
            row_end = s >= 1 and (s - 1) % W == W - 1
            cnt_s = cnt0 + s * L * n * 4
            if self.paper_cache:
                # evict-one-if-full for every layer, then plan, then the layers; nothing happens at row ends
                if s >= 1:
                    B.adsa_compact(tp, seqs0, mb.keep_map, mb.workspace, 0, stream)
                row_end = False
            B.adsa_select(tp, seqs0, sel0, cnt_s, None, B.FLAG_PLAN_APPEND, stream)
            flags = B.FLAG_APPEND | (0 if row_end else B.FLAG_ADVANCE)
            off, q_off = s * self.row_bytes, s * self.q_row_bytes
            for l in range(L):
                B.adsa_attend(lp, seqs0 + l * n * seq_sz, qb[l] + q_off, sel0 + l * n * sel_row, cnt_s + l * n * 4,
                              out0 + l * out_row, lse0 + l * lse_row, mb.layer_workspace, flags,
                              kb[l] + off, vb[l] + off, stream)
            if row_end:
                B.adsa_compact(tp, seqs0, mb.keep_map, mb.workspace, B.FLAG_ADVANCE, stream)
                if on_row_end is not None:
                    on_row_end(s)


def cpu_baseline(wl, n_layers, seconds):
    """The oracle as it stands, one thread, on whole single-(layer, sequence) trajectories."""
    import oracle
    from paper_2506_18226_amd import workloads as WL

    P = wl.prefix_len
    cfg = oracle.make_cfg(n_heads=wl.n_heads, head_dim=wl.head_dim, grid_h=wl.grid_h, grid_w=wl.grid_w,
                          win_rows_back=wl.win_rows_back, win_col_radius=wl.win_col_radius, grid_origin=P,
                          budget=wl.budget if wl.budget_den == 0 else 0, budget_num=wl.budget_num,
                          budget_den=wl.budget_den, score_mode=wl.score_mode, cap=wl.cap(), q_per_kv=wl.q_per_kv)
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
    return {
        "value": seq_layer_steps_per_s / n_layers, "unit": "tokens/s", "cores": 1, "kind": "oracle",
        "sample": f"complete {wl.n_image_tokens}-step trajectories of {seq} of the {wl.n_seq * n_layers} "
                  f"(sequence, layer) caches, {spent:.1f} s of CPU time, scaled by 1/{n_layers} layers",
        "host_cpus": os.cpu_count(),
    }


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
    n_layers = args.layers if args.layers > 0 else wl.n_layers
    t_setup = time.perf_counter()
    job = Job(wl, n_layers, device, paper_cache=args.paper_cache, two_pass_vcos=args.two_pass_vcos)
    torch.cuda.synchronize()
    t_setup = time.perf_counter() - t_setup
    S = job.n_steps_total
    K = S if args.steps <= 0 else min(args.steps, S)
    Wm = max(0, args.warmup)

    # warm-up: Wm steps, then (whole-trajectory runs) start again from the prefix-only cache;
    # shorter runs time the LAST K steps of the trajectory, the deepest contexts.
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
    cnt_log = job.sel_cnt_log.cpu().numpy().astype(np.int64)           # [S][layers * n_seq]
    tau = wl.token_bytes
    tokens = wl.n_seq * K
    result = {
        "metric": "adsa_decode_tokens_per_s", "value": tokens / elapsed, "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": 1e3 * elapsed / K,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if wl.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {
            "workload": f"{wl.name}: {n_layers} layers x {wl.n_seq} sequences, {wl.n_heads} heads x {wl.head_dim}"
                        + (f" with {wl.q_per_kv} query heads each" if wl.q_per_kv > 1 else "") + f", "
                        f"{wl.dtype}, prefix {wl.prefix_len} + {wl.grid_h}x{wl.grid_w} grid, window R={wl.win_rows_back} "
                        f"w={wl.win_col_radius}, budget "
                        + (f"{wl.budget}" if wl.budget_den == 0 else f"{wl.budget_num}/{wl.budget_den} of context")
                        + (", ranking=accumulated attention mass, row-end eviction" if not args.paper_cache else
                           f"; PAPER CACHE POLICY: capacity {job.layer_params.cap}, V-cosine ranking "
                           + ("(two passes over V per step)" if args.two_pass_vcos else "(fused into the attention launch)") +
                           f", evict one when "
                           f"full (the incoming token takes its slot), 1-D window of {job.layer_params.win_recent_m}, "
                           f"attention over everything resident"),
            "decode_steps_timed": [s0, S], "global_batch": wl.n_seq, "layers": n_layers,
            "setup_seconds": round(t_setup, 1),
        },
    }
    # classifier-free guidance runs two sequences (conditional / unconditional, separate caches) per image
    result["image_tokens_per_s_under_cfg_pairing"] = tokens / elapsed / 2.0
    timed_attended = int(cnt_log[s0:S].sum())
    result["selected_kv_gb_per_step"] = timed_attended * tau / K / 1e9
    result["selected_kv_gbs_whole_path"] = timed_attended * tau / elapsed / 1e9

    # ---- roofline of the dominant kernel: same trajectory again with HIP events around k_attend
    if not args.no_roofline_pass:
        job.reset()
        if s0 > 0:
            job.run(0, s0)
        torch.cuda.synchronize()
        n_after = []
        B.adsa_profile_enable(True)
        job.run(s0, S, on_row_end=lambda s: n_after.append((s, [int(x) for x in job.mb.read_seqs()["n_res"]])))
        torch.cuda.synchronize()
        n_launch, att_ms = B.adsa_profile_read()
        B.adsa_profile_enable(False)
        cnt2 = job.sel_cnt_log.cpu().numpy().astype(np.int64)
        att_bytes = int(cnt2[s0:S].sum()) * tau
        achieved = att_bytes / (att_ms * 1e-3) / 1e9
        ratio = measured_traffic_ratio(wl.name)
        result["roofline"] = {
            "kernel": "k_attend" if wl.q_per_kv == 1 else "k_attend_gqa", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": None if ratio is None else ratio * att_bytes / max(1, n_launch),
            "traffic_source": None if ratio is None else
            f"profiles/{wl.name}_attend_hbm_traffic.txt: measured HBM bytes / algorithmic bytes = {ratio} x this run's bytes per launch",
            "launches": int(n_launch), "avg_launch_us": 1e3 * att_ms / max(1, n_launch),
            "algorithmic_bytes_per_launch": att_bytes / max(1, n_launch),
        }
        if wl.q_per_kv > 1:        # the contraction runs on the matrix cores: 4 flops per (query head, token, column)
            flops = int(cnt2[s0:S].sum()) * 4 * wl.n_heads * wl.q_per_kv * wl.head_dim
            result["roofline"]["mfma_tflops"] = flops / (att_ms * 1e-3) / 1e12
            result["roofline"]["mfma_frac_of_bf16_peak"] = flops / (att_ms * 1e-3) / 2.5e15
        if args.paper_cache:       # fixed-capacity cache: resident = what the sequences hold at the end
            n_end = [int(x) for x in job.mb.read_seqs()["n_res"]]
            dense = (wl.prefix_len + wl.n_image_tokens) * wl.n_seq * n_layers * tau
            result["kv_bytes_resident"] = {"max": sum(n_end) * tau, "dense_cache": dense,
                                           "ratio_max_to_dense": sum(n_end) * tau / dense}
        # KV bytes resident: between row ends n_res grows by one per step
        if n_after:
            W = wl.grid_w
            peaks = [sum(v) + W * len(v) for _, v in n_after]      # a row of appends follows each compaction
            dense = (wl.prefix_len + wl.n_image_tokens) * wl.n_seq * n_layers * tau
            result["kv_bytes_resident"] = {
                "max": max(peaks) * tau, "after_last_compaction": sum(n_after[-1][1]) * tau,
                "dense_cache": dense, "ratio_max_to_dense": max(peaks) * tau / dense,
            }

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, n_layers, args.cpu_seconds)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
