"""ctypes binding of the ADSA HIP library: same names as include/adsa.h, marshalling only.

Every function takes torch tensors (device memory) or raw integers for pointers, packs the
host parameter struct and calls the C entry point.  No step of the decode path runs here.
The library must be built (paper_2506_18226_amd/build.py) -- there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

from . import build as _build

F32, BF16 = 0, 1
SCORE_ATTN_MASS, SCORE_VCOS, SCORE_EXT_LARGEST, SCORE_EXT_SMALLEST, SCORE_VCOS_FUSED = 0, 1, 2, 3, 4
FLAG_NO_COMPACT, FLAG_NO_ACCUMULATE, FLAG_PLAN_APPEND, FLAG_APPEND, FLAG_ADVANCE, FLAG_NEW_F32 = 1, 2, 4, 8, 16, 32
SEQ_CACHE_FULL, SEQ_BAD_STATE, SEQ_SEL_OVERFLOW = 1, 2, 4
MAX_CAP = 8192
EVICT_ROW_END, EVICT_WHEN_FULL, EVICT_REUSE_SLOT = 0, 1, 2

ERRORS = {0: "ADSA_OK", -1: "ADSA_ERR_NULL", -2: "ADSA_ERR_SHAPE", -3: "ADSA_ERR_DTYPE", -4: "ADSA_ERR_ALIGN",
          -5: "ADSA_ERR_CAPACITY", -6: "ADSA_ERR_WORKSPACE", -7: "ADSA_ERR_LAUNCH", -8: "ADSA_ERR_UNSUPPORTED",
          -9: "ADSA_ERR_STATIC_SCRATCH"}
STATIC_SCRATCH_BYTES = 4 << 20

EXPORTS = ["adsa_workspace_bytes", "adsa_workspace_init", "adsa_select", "adsa_attend", "adsa_compact", "adsa_step",
           "adsa_step_static",
           "adsa_profile_enable", "adsa_profile_read", "adsa_strerror", "adsa_version"]


class AdsaParams(C.Structure):
    """Mirror of `adsa_params` (host struct)."""
    _fields_ = [
        ("n_seq", C.c_int32), ("n_heads", C.c_int32), ("head_dim", C.c_int32),
        ("grid_h", C.c_int32), ("grid_w", C.c_int32),
        ("win_rows_back", C.c_int32), ("win_col_radius", C.c_int32),
        ("sel_groups", C.c_int32), ("dtype", C.c_int32), ("score_mode", C.c_int32),
        ("cap", C.c_int32), ("sel_cap", C.c_int32),
        ("kv_slot_stride", C.c_int64), ("kv_head_stride", C.c_int64),
        ("softmax_scale", C.c_float), ("win_recent_m", C.c_int32), ("evict_policy", C.c_int32),
        ("q_per_kv", C.c_int32),
    ]


# Mirror of `adsa_seq` (device struct array), 96 bytes per entry.
SEQ_DTYPE = np.dtype([
    ("k", np.uint64), ("v", np.uint64), ("pos", np.uint64), ("score", np.uint64),
    ("n_res", np.int32), ("step", np.int32), ("grid_origin", np.int32), ("n_keep_prefix", np.int32),
    ("budget", np.int32), ("budget_num", np.int32), ("budget_den", np.int32), ("status", np.int32),
    ("compacted", np.int32), ("pending_slot", np.int32), ("hole", np.int32), ("reserved", np.int32),
    ("vcos_u", np.uint64), ("reserved2", np.int64),
])
assert SEQ_DTYPE.itemsize == 96


class AdsaError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {ERRORS.get(code, code)} ({strerror(code)})")


_lib = None


def library_path() -> str:
    return _build.LIB_PATH


def load_library() -> C.CDLL:
    """dlopen the built HIP library; raises if it has not been built."""
    global _lib
    if _lib is None:
        path = library_path()
        if not os.path.exists(path):
            raise FileNotFoundError(f"{path} is missing: run `python -m paper_2506_18226_amd.build` "
                                    "(or __graft_entry__.build()) first; there is no fallback path")
        # torch ships its own HIP runtime: bring it in first so that this library binds to the SAME
        # runtime instance that owns the tensors' memory and streams (two runtimes in one process
        # do not see each other's allocations)
        import torch  # noqa: F401
        lib = C.CDLL(path)
        vp, i32p, f32p = C.c_void_p, C.c_void_p, C.c_void_p
        pp = C.POINTER(AdsaParams)
        lib.adsa_workspace_bytes.restype = C.c_size_t
        lib.adsa_workspace_bytes.argtypes = [pp]
        lib.adsa_workspace_init.restype = C.c_int
        lib.adsa_workspace_init.argtypes = [pp, vp, C.c_size_t, vp]
        lib.adsa_select.restype = C.c_int
        lib.adsa_select.argtypes = [pp, vp, i32p, i32p, C.c_uint32, vp, C.c_size_t, vp]
        lib.adsa_attend.restype = C.c_int
        lib.adsa_attend.argtypes = [pp, vp, vp, vp, vp, i32p, i32p, vp, f32p, C.c_uint32, vp, C.c_size_t, vp]
        lib.adsa_compact.restype = C.c_int
        lib.adsa_compact.argtypes = [pp, vp, i32p, C.c_uint32, vp, C.c_size_t, vp]
        lib.adsa_step.restype = C.c_int
        lib.adsa_step.argtypes = [pp, vp, vp, vp, vp, vp, f32p, i32p, i32p, i32p, C.c_uint32, vp, C.c_size_t, vp]
        lib.adsa_step_static.restype = C.c_int
        lib.adsa_step_static.argtypes = [pp, vp, vp, vp, vp, vp, f32p, i32p, i32p, i32p, C.c_uint32, vp]
        lib.adsa_profile_enable.restype = C.c_int
        lib.adsa_profile_enable.argtypes = [C.c_int]
        lib.adsa_profile_read.restype = C.c_int
        lib.adsa_profile_read.argtypes = [C.POINTER(C.c_int64), C.POINTER(C.c_double)]
        lib.adsa_strerror.restype = C.c_char_p
        lib.adsa_strerror.argtypes = [C.c_int]
        lib.adsa_version.restype = C.c_int
        lib.adsa_version.argtypes = []
        _lib = lib
    return _lib


def _ptr(x) -> Optional[int]:
    """Device pointer of a torch tensor, or the integer itself, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _nbytes(x) -> int:
    return 0 if x is None else x.numel() * x.element_size()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise AdsaError(rc, where)


def make_params(*, n_seq, n_heads, head_dim, grid_h, grid_w, win_rows_back, win_col_radius, dtype,
                score_mode, cap, sel_cap=None, sel_groups=1, layout="head_major", kv_slot_stride=None,
                kv_head_stride=None, softmax_scale=0.0, win_recent_m=0, evict_policy=0, q_per_kv=0) -> AdsaParams:
    """Fill `adsa_params`.  layout "head_major" = [head][slot][D] (a head's rows are contiguous: the
    fast path), "slot_major" = [slot][head][D]; explicit strides override it."""
    if kv_head_stride is None:
        kv_head_stride = cap * head_dim if layout == "head_major" else head_dim
    if kv_slot_stride is None:
        kv_slot_stride = head_dim if layout == "head_major" else n_heads * head_dim
    return AdsaParams(n_seq, n_heads, head_dim, grid_h, grid_w, win_rows_back, win_col_radius, sel_groups,
                      dtype, score_mode, cap, cap if sel_cap is None else sel_cap,
                      kv_slot_stride, kv_head_stride, softmax_scale, win_recent_m, evict_policy, q_per_kv)


def score_rows(params: AdsaParams) -> int:
    """Rows of adsa_seq.score: one per head for ATTN_MASS, two per head for VCOS_FUSED, else one.  (With per-head
    attended sets, sel_groups == n_heads, every record describes one head.)"""
    heads = 1 if params.sel_groups == params.n_heads else params.n_heads
    if params.score_mode == SCORE_VCOS_FUSED:
        return 2 * heads
    return heads if params.score_mode == SCORE_ATTN_MASS else 1


def query_heads(params: AdsaParams) -> int:
    """Heads of q / out / lse: n_heads cache heads times q_per_kv query heads each."""
    return params.n_heads * max(params.q_per_kv, 1)


def strerror(code: int) -> str:
    return load_library().adsa_strerror(code).decode()


def adsa_version() -> int:
    return load_library().adsa_version()


def adsa_workspace_bytes(params: AdsaParams) -> int:
    return int(load_library().adsa_workspace_bytes(C.byref(params)))


def adsa_workspace_init(params, workspace, stream=None) -> None:
    _check(load_library().adsa_workspace_init(C.byref(params), _ptr(workspace), _nbytes(workspace),
                                              _stream(stream)), "adsa_workspace_init")


def adsa_select(params, seqs, sel_idx, sel_cnt, workspace=None, flags=0, stream=None) -> None:
    _check(load_library().adsa_select(C.byref(params), _ptr(seqs), _ptr(sel_idx), _ptr(sel_cnt), flags,
                                      _ptr(workspace), _nbytes(workspace), _stream(stream)), "adsa_select")


def adsa_attend(params, seqs, q, sel_idx, sel_cnt, out, lse, workspace, flags=0, k_new=None, v_new=None,
                stream=None) -> None:
    _check(load_library().adsa_attend(C.byref(params), _ptr(seqs), _ptr(q), _ptr(k_new), _ptr(v_new),
                                      _ptr(sel_idx), _ptr(sel_cnt), _ptr(out), _ptr(lse), flags,
                                      _ptr(workspace), _nbytes(workspace), _stream(stream)), "adsa_attend")


def adsa_compact(params, seqs, keep_map, workspace, flags=0, stream=None) -> None:
    _check(load_library().adsa_compact(C.byref(params), _ptr(seqs), _ptr(keep_map), flags, _ptr(workspace),
                                       _nbytes(workspace), _stream(stream)), "adsa_compact")


def adsa_step(params, seqs, q, k_new, v_new, out, lse, sel_idx, sel_cnt, keep_map, workspace,
              flags=0, stream=None) -> None:
    _check(load_library().adsa_step(C.byref(params), _ptr(seqs), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out),
                                    _ptr(lse), _ptr(sel_idx), _ptr(sel_cnt), _ptr(keep_map), flags,
                                    _ptr(workspace), _nbytes(workspace), _stream(stream)), "adsa_step")


def adsa_step_static(params, seqs, q, k_new, v_new, out, lse, sel_idx, sel_cnt, keep_map, flags=0, stream=None) -> None:
    """adsa_step on the library's built-in scratch array: no workspace argument, no allocation."""
    _check(load_library().adsa_step_static(C.byref(params), _ptr(seqs), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out),
                                           _ptr(lse), _ptr(sel_idx), _ptr(sel_cnt), _ptr(keep_map), flags,
                                           _stream(stream)), "adsa_step_static")


def adsa_profile_enable(on: bool) -> None:
    _check(load_library().adsa_profile_enable(1 if on else 0), "adsa_profile_enable")


def adsa_profile_read():
    """(number of bracketed attention launches, their summed duration in ms)."""
    n, ms = C.c_int64(0), C.c_double(0.0)
    _check(load_library().adsa_profile_read(C.byref(n), C.byref(ms)), "adsa_profile_read")
    return n.value, ms.value
