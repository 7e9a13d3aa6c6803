"""Device-memory plumbing for one layer of an ADSA decode batch.

`LayerBatch` owns the torch tensors the C ABI points into (K/V caches, pos, score, the
`adsa_seq` device array, outputs, workspace) and converts host arrays to and from them.
It performs no step of the method: every call below that computes anything goes through
`binding.adsa_*`.
"""
from __future__ import annotations

from typing import Optional

import numpy as np
import torch

from . import binding as B
from .workloads import bf16_bits


def to_device(x: np.ndarray, dtype_code: int, device) -> torch.Tensor:
    """float32 host values (already representable in the storage type) -> device tensor."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype_code == B.F32:
        return torch.from_numpy(x).to(device)
    bits = torch.from_numpy(bf16_bits(x).view(np.int16)).to(device)
    return bits.view(torch.bfloat16)


def to_host(t: torch.Tensor) -> np.ndarray:
    """Device tensor (f32 or bf16) -> float32 numpy array."""
    return t.detach().float().cpu().numpy()


class LayerBatch:
    def __init__(self, params: B.AdsaParams, device: str = "cuda:0", with_outputs: bool = True):
        self.params = params
        self.device = torch.device(device)
        p = params
        self.tdtype = torch.float32 if p.dtype == B.F32 else torch.bfloat16
        n, cap, h, D = p.n_seq, p.cap, p.n_heads, p.head_dim
        if p.kv_slot_stride == D and p.kv_head_stride == cap * D:
            self.head_major = True
        elif p.kv_slot_stride == h * D and p.kv_head_stride == D:
            self.head_major = False
        else:
            raise ValueError("LayerBatch allocates dense [head][slot][D] or [slot][head][D] caches only")
        dev = self.device
        shape = (n, h, cap, D) if self.head_major else (n, cap, h, D)
        self.K = torch.zeros(shape, dtype=self.tdtype, device=dev)
        self.V = torch.zeros(shape, dtype=self.tdtype, device=dev)
        self.pos = torch.zeros((n, cap), dtype=torch.int32, device=dev)
        self.rows = B.score_rows(p)
        self.score = torch.zeros((n, self.rows, cap), dtype=torch.float32, device=dev)
        self.seqs_host = np.zeros(n, dtype=B.SEQ_DTYPE)
        # running V-cosine state of the fused ranking: u [h*D] + 4 tag words per sequence
        self.vcos_u = (torch.zeros((n, h * D + 4), dtype=torch.float32, device=dev)
                       if p.score_mode == B.SCORE_VCOS_FUSED else None)
        elem = self.K.element_size()
        for b in range(n):
            s = self.seqs_host[b]
            s["k"] = self.K.data_ptr() + b * cap * h * D * elem
            s["v"] = self.V.data_ptr() + b * cap * h * D * elem
            s["pos"] = self.pos.data_ptr() + b * cap * 4
            s["score"] = self.score.data_ptr() + b * self.rows * cap * 4
            s["step"] = -1
            s["pending_slot"] = -1
            if self.vcos_u is not None:
                s["vcos_u"] = self.vcos_u.data_ptr() + b * (h * D + 4) * 4
        self.seqs = torch.zeros(n * B.SEQ_DTYPE.itemsize, dtype=torch.uint8, device=dev)
        if with_outputs:
            hq = B.query_heads(p)
            self.out = torch.zeros((n, hq, D), dtype=self.tdtype, device=dev)
            self.lse = torch.zeros((n, hq), dtype=torch.float32, device=dev)
            self.sel_idx = torch.full((n, p.sel_cap), -1, dtype=torch.int32, device=dev)
            self.sel_cnt = torch.zeros(n, dtype=torch.int32, device=dev)
            self.keep_map = torch.full((n, cap), -3, dtype=torch.int32, device=dev)
        ws = B.adsa_workspace_bytes(p)
        if ws == 0:
            raise B.AdsaError(-2, "adsa_workspace_bytes (invalid parameters)")
        self.workspace = torch.empty(ws, dtype=torch.uint8, device=dev)
        B.adsa_workspace_init(p, self.workspace)

    # ---- host -> device
    def set_sequence(self, b: int, *, k: np.ndarray, v: np.ndarray, pos: np.ndarray,
                     score: Optional[np.ndarray], step: int, grid_origin: int,
                     n_keep_prefix: Optional[int] = None, budget: int = 0, budget_num: int = 0,
                     budget_den: int = 0) -> None:
        """k, v: [n][h][D] host rows; score: [n] (goes to score row 0, the other rows are zeroed)
        or [rows][n]."""
        n = len(pos)
        p = self.params
        if n > p.cap:
            raise ValueError("more resident slots than cap")
        if n:
            kd, vd = to_device(k[:n], p.dtype, self.device), to_device(v[:n], p.dtype, self.device)
            if self.head_major:
                self.K[b, :, :n] = kd.transpose(0, 1)
                self.V[b, :, :n] = vd.transpose(0, 1)
            else:
                self.K[b, :n] = kd
                self.V[b, :n] = vd
            self.pos[b, :n] = torch.from_numpy(np.ascontiguousarray(pos[:n], dtype=np.int32)).to(self.device)
            self.score[b].zero_()
            if score is not None:
                sc = np.ascontiguousarray(score, dtype=np.float32)
                if sc.ndim == 1:
                    self.score[b, 0, :n] = torch.from_numpy(sc[:n]).to(self.device)
                else:
                    self.score[b, :, :n] = torch.from_numpy(np.ascontiguousarray(sc[:, :n])).to(self.device)
        s = self.seqs_host[b]
        s["n_res"], s["step"], s["grid_origin"] = n, step, grid_origin
        s["n_keep_prefix"] = grid_origin if n_keep_prefix is None else n_keep_prefix
        s["budget"], s["budget_num"], s["budget_den"] = budget, budget_num, budget_den
        s["status"], s["compacted"], s["pending_slot"], s["hole"] = 0, 0, -1, 0
        if self.vcos_u is not None:
            self.vcos_u[b].zero_()          # the cache was set by hand: the running state starts over

    # ---- device -> host, layout-independent views
    def k_host(self) -> np.ndarray:
        """K as float32 [n_seq][cap][h][D]."""
        k = to_host(self.K)
        return k.transpose(0, 2, 1, 3) if self.head_major else k

    def v_host(self) -> np.ndarray:
        v = to_host(self.V)
        return v.transpose(0, 2, 1, 3) if self.head_major else v

    def upload_seqs(self) -> None:
        raw = torch.from_numpy(self.seqs_host.view(np.uint8).reshape(-1).copy())
        self.seqs.copy_(raw.to(self.device))

    # ---- device -> host
    def read_seqs(self) -> np.ndarray:
        raw = self.seqs.cpu().numpy()
        self.seqs_host = raw.view(B.SEQ_DTYPE).copy()
        return self.seqs_host

    # ---- thin forwards to the C ABI
    def select(self, flags: int = 0, stream=None):
        B.adsa_select(self.params, self.seqs, self.sel_idx, self.sel_cnt, self.workspace, flags, stream)

    def attend(self, q: torch.Tensor, flags: int = 0, k_new=None, v_new=None, stream=None):
        B.adsa_attend(self.params, self.seqs, q, self.sel_idx, self.sel_cnt, self.out, self.lse,
                      self.workspace, flags, k_new, v_new, stream)

    def compact(self, flags: int = 0, stream=None):
        B.adsa_compact(self.params, self.seqs, self.keep_map, self.workspace, flags, stream)

    def step(self, q, k_new, v_new, flags: int = 0, stream=None):
        B.adsa_step(self.params, self.seqs, q, k_new, v_new, self.out, self.lse, self.sel_idx, self.sel_cnt,
                    self.keep_map, self.workspace, flags, stream)


    def step_static(self, q, k_new, v_new, flags: int = 0, stream=None):
        B.adsa_step_static(self.params, self.seqs, q, k_new, v_new, self.out, self.lse, self.sel_idx, self.sel_cnt,
                           self.keep_map, flags, stream)


class ModelBatch(LayerBatch):
    """Caches of ALL layers of a model for one decode batch, laid out as n_layers * n_seq
    independent sequences (layer-major), so that the q-independent phases of a decode step
    (adsa_select, adsa_compact) run once for every layer while adsa_attend runs per layer on
    its slice of the same arrays."""

    def __init__(self, layer_params: B.AdsaParams, n_layers: int, device: str = "cuda:0"):
        import copy
        self.layer_params = layer_params
        self.n_layers = n_layers
        self.n_per_layer = layer_params.n_seq
        total = copy.copy(layer_params)
        total.n_seq = layer_params.n_seq * n_layers
        super().__init__(total, device)
        ws = B.adsa_workspace_bytes(layer_params)
        self.layer_workspace = torch.empty(ws, dtype=torch.uint8, device=self.device)
        B.adsa_workspace_init(layer_params, self.layer_workspace)

    def select_all(self, flags: int = 0, stream=None):
        B.adsa_select(self.params, self.seqs, self.sel_idx, self.sel_cnt, self.workspace, flags, stream)

    def compact_all(self, flags: int = 0, stream=None):
        B.adsa_compact(self.params, self.seqs, self.keep_map, self.workspace, flags, stream)

    def attend_layer(self, layer: int, q, k_new=None, v_new=None, flags: int = 0, stream=None):
        n, p = self.n_per_layer, self.layer_params
        b0 = layer * n
        B.adsa_attend(p, self.seqs.data_ptr() + b0 * B.SEQ_DTYPE.itemsize, q,
                      self.sel_idx.data_ptr() + b0 * p.sel_cap * 4, self.sel_cnt.data_ptr() + b0 * 4,
                      self.out[b0:b0 + n], self.lse[b0:b0 + n], self.layer_workspace, flags, k_new, v_new, stream)
