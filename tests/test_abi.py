"""CPU-only checks of the C boundary: the library loads, exports every declared symbol, and
rejects bad arguments before touching a device."""
import ctypes as C
import math
import os
import re

import pytest

import paper_2605_30010_amd as et
from paper_2605_30010_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "earlytom.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(et_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = et.load_library()
    names = _declared_functions()
    assert len(names) >= 19 and "et_encode_clip" in names and "et_merge_select" in names
    for n in names:
        assert hasattr(lib, n), "libearlytom.so does not export " + n


def test_keep_count_rule():
    assert et.et_keep_count(64, 0.5) == 32
    assert et.et_keep_count(729, 0.5) == 364
    assert et.et_keep_count(729, 0.25) == 182
    assert et.et_keep_count(729, 0.3) == 218
    assert et.et_keep_count(10, 0.7) == 7
    assert et.et_keep_count(729, 1.0) == 729
    assert et.et_keep_count(729, 1e-9) == 1
    for bad in (0.0, -0.5, 1.5, math.nan):
        assert et.et_keep_count(729, bad) == 0
    assert et.et_keep_count(0, 0.5) == 0


def test_keep_count_matches_oracle_rule():
    from oracle import earlytom_oracle as O
    import numpy as np
    for L in (1, 7, 64, 729, 1000):
        for r in (0.01, 0.1, 0.25, 0.3, 0.5, 0.7, 0.9, 1.0):
            assert et.et_keep_count(L, r) == O.keep_count(L, np.float32(r))


def test_kernel_names_and_workspace_size():
    assert et.et_kernel_name(0) == "im2col" and et.et_kernel_name(99) == "?"
    assert [et.et_kernel_name(i) for i in range(B.ET_K_COUNT)] == B.KERNEL_KINDS
    assert et.et_merge_workspace_bytes(0, 729, 1152) == 0
    need = et.et_merge_workspace_bytes(64, 729, 1152)
    assert need >= 64 * 729 * 1152 * 2 + (2 * 64 - 1) * 729 * 4
    assert need % 256 == 0


def test_merge_select_rejects_bad_arguments_before_device_work():
    lib = et.load_library()
    out = B._Output()
    fake = C.c_void_p(4096)          # never dereferenced: validation fails first
    out.tokens_dev = out.kept_idx_dev = out.cu_tokens_dev = out.seg_start_dev = 4096
    call = lambda x, T, L, D, tau, r, ws, wsb, o: lib.et_merge_select(x, T, L, D, tau, r, ws, wsb, None, o)
    assert call(None, 4, 8, 64, 0.9, 0.5, fake, 1 << 30, C.byref(out)) == -1
    assert "x_dev" in et.et_last_error()
    assert call(fake, 0, 8, 64, 0.9, 0.5, fake, 1 << 30, C.byref(out)) == -1
    assert call(fake, 4, 8, 60, 0.9, 0.5, fake, 1 << 30, C.byref(out)) == -1
    assert "multiple of 8" in et.et_last_error()
    assert call(fake, 4, 8, 64, math.nan, 0.5, fake, 1 << 30, C.byref(out)) == -1
    assert call(fake, 4, 8, 64, 0.9, 0.0, fake, 1 << 30, C.byref(out)) == -1
    assert call(fake, 4, 8, 64, 0.9, 1.5, fake, 1 << 30, C.byref(out)) == -1
    assert "keep_ratio" in et.et_last_error()
    assert call(fake, 4, 8, 64, 0.9, 0.5, None, 1 << 30, C.byref(out)) == -1
    assert call(fake, 4, 8, 64, 0.9, 0.5, fake, 16, C.byref(out)) == -2
    assert "workspace" in et.et_last_error()
    assert call(fake, 4, 8, 8192, 0.9, 0.5, fake, 1 << 40, C.byref(out)) == -5
    bad = B._Output()
    assert call(fake, 4, 8, 64, 0.9, 0.5, fake, 1 << 30, C.byref(bad)) == -1
    assert "output buffer" in et.et_last_error()
    assert call(fake, 4, 8, 64, 0.9, 0.5, fake, 1 << 30, None) == -1


def test_static_scratch_entry_point_rejects_bad_arguments_and_oversized_shapes():
    """The entry point without a workspace argument validates like et_merge_select and refuses, before
    any device work, shapes whose scratch would not fit its fixed buffer."""
    lib = et.load_library()
    out = B._Output()
    fake = C.c_void_p(4096)
    out.tokens_dev = out.kept_idx_dev = out.cu_tokens_dev = out.seg_start_dev = 4096
    call = lambda x, T, L, D, tau, r, o: lib.et_merge_select_static(x, T, L, D, tau, r, None, o)
    assert call(None, 4, 8, 64, 0.9, 0.5, C.byref(out)) == -1
    assert call(fake, 4, 8, 60, 0.9, 0.5, C.byref(out)) == -1
    assert call(fake, 4, 8, 64, math.nan, 0.5, C.byref(out)) == -1
    assert call(fake, 4, 8, 64, 0.9, 0.0, C.byref(out)) == -1
    assert call(fake, 4, 8, 64, 0.9, 0.5, None) == -1
    limit = 64 << 20
    assert et.et_merge_workspace_bytes(39, 729, 1152) <= limit < et.et_merge_workspace_bytes(40, 729, 1152)
    assert call(fake, 40, 729, 1152, 0.9, 0.5, C.byref(out)) == -2
    assert "static buffer" in et.et_last_error() and str(limit) in et.et_last_error()
    assert call(fake, 64, 729, 1152, 0.9, 0.5, C.byref(out)) == -2


def test_encoder_entry_points_reject_bad_arguments():
    lib = et.load_library()
    handle = C.c_void_p()
    cfg = B._Config(n_layers=1, d_model=64, n_heads=4, d_mlp=256, patch=14, image_h=112, image_w=112,
                    channels=3, ln_eps=1e-6, has_final_ln=1)
    w = B._Weights()
    assert lib.et_encoder_create(None, C.byref(w), 8, C.byref(handle)) == -1
    assert lib.et_encoder_create(C.byref(cfg), C.byref(w), 8, C.byref(handle)) == -1   # NULL weights
    assert "NULL" in et.et_last_error()
    cfg2 = B._Config(n_layers=1, d_model=64, n_heads=5, d_mlp=256, patch=14, image_h=112, image_w=112,
                     channels=3, ln_eps=1e-6, has_final_ln=1)
    assert lib.et_encoder_create(C.byref(cfg2), C.byref(w), 8, C.byref(handle)) == -1
    assert "n_heads" in et.et_last_error()
    cfg3 = B._Config(n_layers=1, d_model=64, n_heads=4, d_mlp=256, patch=14, image_h=10, image_w=112,
                     channels=3, ln_eps=1e-6, has_final_ln=1)
    assert lib.et_encoder_create(C.byref(cfg3), C.byref(w), 8, C.byref(handle)) == -1
    assert "patch" in et.et_last_error()
    assert lib.et_encoder_create(C.byref(cfg), C.byref(w), 0, C.byref(handle)) == -1
    assert lib.et_encode_clip(None, None, 1, 0, 0.9, 0.5, None, 0, None, None) == -1
    assert lib.et_workspace_bytes(None, 4) == 0
    lib.et_encoder_destroy(None)
    assert lib.et_profile_enable(None, 1) == -1
    fake = C.c_void_p(4096)
    assert lib.et_encoder_block_qkv(None, 0, fake, 4, fake, fake, None) == -1


def test_single_step_entry_points_reject_bad_arguments():
    lib = et.load_library()
    fake = C.c_void_p(4096)
    assert lib.et_topk_select(fake, 2, 8, 9, fake, None) == -1          # k > L
    assert lib.et_topk_select(fake, 2, 8, 0, fake, None) == -1
    assert lib.et_topk_select(None, 2, 8, 4, fake, None) == -1
    assert lib.et_topk_select(fake, 2, 20000, 4, fake, None) == -5
    assert lib.et_frame_similarity(fake, 2, 8, 12, fake, fake, None) == -1
    assert lib.et_segment_scan(None, 4, 0.9, fake, fake, None) == -1
    assert lib.et_segment_scan(fake, 4, math.nan, fake, fake, None) == -1
    assert lib.et_compact_tokens(fake, fake, 2, 8, 64, 9, fake, None) == -1
    assert lib.et_layernorm(fake, fake, fake, 1e-6, 4, 12, fake, None) == -1
    assert lib.et_gemm_bf16(fake, fake, fake, None, 4, 64, 64, 2, -1, fake, None) == -1   # residual missing
    assert lib.et_gemm_bf16(fake, fake, fake, None, 4, 60, 64, 0, -1, fake, None) == -1
    assert lib.et_gemm_bf16(fake, fake, fake, None, 4, 64, 64, 0, 99, fake, None) == -1
    assert lib.et_attention(fake, fake, 2, 8, 4, 20, fake, None) == -5
    assert lib.et_attention(None, fake, 2, 8, 4, 16, fake, None) == -1


def test_no_cpu_fallback_when_library_missing(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "_LIB_PATH", str(tmp_path / "absent.so"))
    with pytest.raises(ImportError):
        B.load_library()


def test_policy_entry_points_reject_bad_arguments():
    lib = et.load_library()
    fake = C.c_void_p(4096)
    out = B._Output()
    out.tokens_dev = out.kept_idx_dev = out.cu_tokens_dev = out.seg_start_dev = 4096
    good = B._Policy(merge_mode=1, select_mode=1, alpha=0.9, tau_seg=0.8, tau_merge=0.8, ratio=0.2)
    call = lambda pol: lib.et_merge_select_policy(fake, 4, 8, 64, pol, fake, 1 << 30, None, C.byref(out), None)
    assert call(None) == -1 and "policy" in et.et_last_error()
    for field, bad in (("merge_mode", 7), ("select_mode", -1), ("alpha", 0.0), ("alpha", 1.5),
                       ("tau_seg", math.nan), ("tau_merge", math.nan), ("ratio", 0.0), ("ratio", 2.0)):
        pol = B._Policy(merge_mode=1, select_mode=1, alpha=0.9, tau_seg=0.8, tau_merge=0.8, ratio=0.2)
        setattr(pol, field, bad)
        assert call(C.byref(pol)) == -1, field
    assert lib.et_merge_select_policy(None, 4, 8, 64, C.byref(good), fake, 1 << 30, None, C.byref(out), None) == -1
    assert lib.et_merge_select_policy(fake, 4, 8, 64, C.byref(good), fake, 16, None, C.byref(out), None) == -2
    assert lib.et_encode_clip_policy(None, fake, 4, 2, C.byref(good), fake, 1 << 30, None, C.byref(out), None) == -1
    layers = (C.c_int32 * 2)(1, 2)
    assert lib.et_encode_clip_multi(None, fake, 4, layers, 2, 3, C.byref(good), fake, 1 << 30, None,
                                    C.byref(out), None) == -1
    assert "encoder" in et.et_last_error()
