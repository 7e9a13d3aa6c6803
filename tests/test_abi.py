"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before anything is launched."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2506_18226_amd import binding as B
from paper_2506_18226_amd import build as BLD

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(BLD.LIB_PATH):
        BLD.build_library()
    return B.load_library()


def header_functions():
    text = open(os.path.join(ROOT, "include", "adsa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(adsa_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = header_functions()
    assert sorted(names) == sorted(B.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n
    assert B.adsa_version() == 1


def test_struct_mirrors_match_the_header():
    assert C.sizeof(B.AdsaParams) == 12 * 4 + 2 * 8 + 4 + 3 * 4
    assert B.SEQ_DTYPE.itemsize == 96 and B.SEQ_DTYPE.fields["vcos_u"][1] == 80
    assert B.SEQ_DTYPE.fields["n_res"][1] == 32 and B.SEQ_DTYPE.fields["status"][1] == 60
    assert B.SEQ_DTYPE.fields["pending_slot"][1] == 68 and B.SEQ_DTYPE.fields["hole"][1] == 72


def good(**kw):
    base = dict(n_seq=2, n_heads=4, head_dim=64, grid_h=8, grid_w=8, win_rows_back=1, win_col_radius=2,
                dtype=B.BF16, score_mode=B.SCORE_ATTN_MASS, cap=128, sel_cap=128, layout="slot_major")
    base.update(kw)
    return B.make_params(**base)


def test_workspace_size_is_positive_and_monotone(lib):
    a = B.adsa_workspace_bytes(good())
    b = B.adsa_workspace_bytes(good(n_seq=8))
    assert a > 0 and b > a and a % 256 == 0
    assert B.adsa_workspace_bytes(good(layout="head_major")) > 0
    # head-major rows of different heads must not overlap: head stride >= cap * slot stride
    assert B.adsa_workspace_bytes(good(layout="head_major", kv_head_stride=127 * 64)) == 0


@pytest.mark.parametrize("kw,code", [
    (dict(dtype=7), -3), (dict(score_mode=9), -3), (dict(n_seq=0), -2), (dict(n_heads=0), -2),
    (dict(n_heads=300), -2), (dict(head_dim=96), -2), (dict(grid_w=0), -2), (dict(win_rows_back=-1), -2),
    (dict(cap=0), -5), (dict(cap=B.MAX_CAP + 1, sel_cap=16), -5), (dict(sel_cap=0), -5), (dict(sel_cap=129), -5),
    (dict(sel_groups=3), -8), (dict(sel_groups=0), -8), (dict(sel_groups=4, n_seq=20000), -2), (dict(kv_slot_stride=4 * 64 + 4), -4), (dict(kv_head_stride=32), -2),
    (dict(kv_slot_stride=64), -2), (dict(softmax_scale=-1.0), -2),
    (dict(score_mode=B.SCORE_VCOS, n_heads=128, head_dim=128), -8),
    (dict(win_recent_m=-1), -2), (dict(evict_policy=5), -3), (dict(evict_policy=B.EVICT_WHEN_FULL), -8),
    (dict(evict_policy=B.EVICT_REUSE_SLOT), -8), (dict(q_per_kv=-1), -2), (dict(q_per_kv=17), -2), (dict(q_per_kv=4, dtype=B.F32), -8),
])
def test_bad_parameters_are_rejected_before_any_launch(lib, kw, code):
    p = good(**kw)
    fake = 0x1000   # never dereferenced: validation fails first
    rc = lib.adsa_select(C.byref(p), fake, fake, fake, 0, fake, 1 << 30, None)
    assert rc == code, B.strerror(rc)
    assert B.adsa_workspace_bytes(p) == 0
    rc = lib.adsa_step(C.byref(p), fake, fake, fake, fake, fake, fake, fake, fake, fake, 0, fake, 1 << 30, None)
    assert rc == code
    assert len(B.strerror(rc)) > 3


def test_per_head_attended_sets_are_an_abi_value(lib):
    """sel_groups == n_heads: every (sequence, head) is a one-head sequence; the workspace is the one of
    n_seq * n_heads single-head sequences, for either nesting of the caller's cache."""
    one_head = good(n_seq=2 * 4, n_heads=1, layout="head_major")
    for layout in ("slot_major", "head_major"):
        per_head = good(sel_groups=4, layout=layout)
        assert B.adsa_workspace_bytes(per_head) == B.adsa_workspace_bytes(one_head) > 0
        assert B.score_rows(per_head) == 1
    assert B.adsa_workspace_bytes(good(sel_groups=4, q_per_kv=4)) > 0
    assert B.query_heads(good(sel_groups=4, q_per_kv=4)) == 16


def test_grouped_query_parameters(lib):
    """q_per_kv 0 and 1 are the multi-head case; 2..16 need bf16; lists whose logits do not fit in LDS are split."""
    assert B.adsa_workspace_bytes(good(q_per_kv=0)) == B.adsa_workspace_bytes(good(q_per_kv=1)) > 0
    assert B.adsa_workspace_bytes(good(q_per_kv=8, dtype=B.BF16)) > 0
    assert B.query_heads(good(q_per_kv=8, dtype=B.BF16)) == 8 * good().n_heads
    big = dict(dtype=B.BF16, cap=B.MAX_CAP, sel_cap=B.MAX_CAP, kv_slot_stride=None, kv_head_stride=None)
    assert B.adsa_workspace_bytes(good(q_per_kv=2, **big)) > 0            # 3 x 8.2k x 4 B of logits: fits
    assert B.adsa_workspace_bytes(good(q_per_kv=16, **big)) > 0           # 17 x 8.2k x 4 B: does not, so the list is split
    # a head's rows are addressed with 32-bit byte offsets: padded strides that push them past 4 GiB are refused
    wide = dict(dtype=B.BF16, cap=8192, sel_cap=128, kv_slot_stride=1 << 18, kv_head_stride=64)
    assert B.adsa_workspace_bytes(good(q_per_kv=1, **wide)) > 0
    assert B.adsa_workspace_bytes(good(q_per_kv=2, **wide)) == 0


def test_fused_vcos_parameters(lib):
    """ADSA_SCORE_VCOS_FUSED: slot-reuse policy, [head][slot][D] caches, one query head per cache head."""
    ok = dict(score_mode=B.SCORE_VCOS_FUSED, evict_policy=B.EVICT_REUSE_SLOT, win_recent_m=9, layout="head_major")
    assert B.adsa_workspace_bytes(good(**ok)) > 0
    assert B.score_rows(good(**ok)) == 2 * good().n_heads
    for bad in (dict(ok, layout="slot_major"), dict(ok, evict_policy=B.EVICT_WHEN_FULL),
                dict(ok, evict_policy=B.EVICT_ROW_END, win_recent_m=0), dict(ok, q_per_kv=2),
                dict(ok, win_recent_m=1),                             # the running sum needs the m - 1 >= 1 newest tokens local
                dict(ok, n_heads=64, head_dim=64, cap=128)):          # 16 * h * D bytes of LDS do not fit
        p = good(**bad)
        assert B.adsa_workspace_bytes(p) == 0, bad
        assert lib.adsa_compact(C.byref(p), 0x1000, 0x1000, 0, 0x1000, 1 << 30, None) == -8, bad


def test_null_alignment_and_workspace_errors(lib):
    p = good()
    ok = 0x1000
    need = B.adsa_workspace_bytes(p)
    assert lib.adsa_select(C.byref(p), None, ok, ok, 0, ok, need, None) == -1
    assert lib.adsa_select(None, ok, ok, ok, 0, ok, need, None) == -1
    assert lib.adsa_attend(C.byref(p), ok, ok, None, None, ok, ok, None, ok, 0, ok, need, None) == -1
    assert lib.adsa_attend(C.byref(p), ok, ok + 4, None, None, ok, ok, ok, ok, 0, ok, need, None) == -4
    assert lib.adsa_attend(C.byref(p), ok, ok, None, None, ok, ok, ok, ok, 0, None, need, None) == -6
    assert lib.adsa_attend(C.byref(p), ok, ok, None, None, ok, ok, ok, ok, 0, ok, need - 1, None) == -6
    assert lib.adsa_attend(C.byref(p), ok, ok, None, None, ok, ok, ok, ok, 0, ok + 16, need, None) == -4
    # appending needs the new rows
    assert lib.adsa_attend(C.byref(p), ok, ok, None, ok, ok, ok, ok, ok, B.FLAG_APPEND, ok, need, None) == -1
    assert lib.adsa_attend(C.byref(p), ok, ok, ok + 2, ok, ok, ok, ok, ok, B.FLAG_APPEND, ok, need, None) == -4
    assert lib.adsa_compact(C.byref(p), ok, None, 0, ok, need, None) == -1
    assert lib.adsa_compact(C.byref(p), ok, ok, 0, ok, 0, None) == -6
    assert lib.adsa_workspace_init(C.byref(p), None, need, None) == -6
    assert lib.adsa_workspace_init(C.byref(p), ok, need - 1, None) == -6
    assert lib.adsa_workspace_init(C.byref(p), ok + 8, need, None) == -4
    # keep_map may be NULL only when the caller rules compaction out
    assert lib.adsa_step(C.byref(p), ok, ok, ok, ok, ok, ok, ok, ok, None, 0, ok, need, None) == -1
    assert lib.adsa_step(C.byref(p), ok, ok, ok, ok + 8, ok, ok, ok, ok, ok, 0, ok, need, None) == -4
    n, ms = C.c_int64(), C.c_double()
    assert lib.adsa_profile_read(None, C.byref(ms)) == -1
    assert lib.adsa_profile_read(C.byref(n), C.byref(ms)) == 0 and n.value == 0


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(BLD, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(FileNotFoundError):
        B.load_library()
    with pytest.raises(FileNotFoundError):
        B.adsa_version()


def test_product_package_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2506_18226_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
                assert "adsa_oracle" not in text, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c", ".h")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2506_18226_amd" not in text and "adsa.h" not in text, f


def test_static_scratch_entry_point_checks_its_arguments_on_the_host(lib):
    """adsa_step_static validates like adsa_step and refuses parameter sets that need more scratch than its
    built-in array, before touching the GPU."""
    ok = 0x1000
    p = good()
    assert B.adsa_workspace_bytes(p) <= B.STATIC_SCRATCH_BYTES
    assert lib.adsa_step_static(C.byref(p), None, ok, ok, ok, ok, ok, ok, ok, ok, 0, None) == -1
    assert lib.adsa_step_static(C.byref(p), ok, ok + 4, ok, ok, ok, ok, ok, ok, ok, 0, None) == -4
    assert lib.adsa_step_static(C.byref(good(head_dim=96)), ok, ok, ok, ok, ok, ok, ok, ok, ok, 0, None) == -2
    big = good(n_seq=4096, n_heads=32, head_dim=128, cap=4096, sel_cap=4096, score_mode=B.SCORE_VCOS, layout="head_major")
    assert B.adsa_workspace_bytes(big) > B.STATIC_SCRATCH_BYTES
    rc = lib.adsa_step_static(C.byref(big), ok, ok, ok, ok, ok, ok, ok, ok, ok, 0, None)
    assert rc == -9 and "built-in" in B.strerror(rc)
