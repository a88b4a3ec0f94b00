"""CPU-only checks of the C-ABI boundary: the library loads, exports every symbol the header declares,
and rejects bad arguments on the host (no kernel is launched, no GPU is needed)."""
import ctypes
import os
import re

import pytest

from paper_2605_21649_amd import binding as ekv

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_symbols():
    text = open(os.path.join(ROOT, "include", "entmaxkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ekv_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = ekv.load_library()
    syms = header_symbols()
    assert set(syms) == set(ekv.EXPORTS)
    for s in syms:
        assert hasattr(lib, s), s
    assert lib.ekv_version() >= 100
    assert lib.ekv_status_string(0) == b"EKV_OK"
    assert lib.ekv_status_string(3) == b"EKV_ERR_WORKSPACE"


def good_cfg(**kw):
    base = dict(batch=1, n_q_heads=32, n_kv_heads=8, head_dim=128, page_size=16, kv_dtype="bf16", alpha=1.5,
                scale=0.088, max_pages_per_seq=65536, max_sel_pages=2622)
    base.update(kw)
    return ekv.make_config(**base)


def test_workspace_sizes():
    cfg = good_cfg()
    sparse = ekv.ekv_workspace_bytes(cfg, ekv.EKV_OP_DECODE_SPARSE)
    full = ekv.ekv_workspace_bytes(cfg, ekv.EKV_OP_DECODE_FULL)
    # scores: 4 B per candidate token and query head, plus one maximum per 64 tokens; rows that can exceed the
    # solve's 4096-entry list add an overflow list of min(row, 65536) (value, position) entries per head; rows of more
    # than 262144 tokens add the filter lists (32 KiB per 32768-token slice and head)
    scores, spill = 32 * 2622 * 16 * 4, 32 * 2622 * 16 * 8
    assert scores + spill <= sparse < 1.1 * scores + spill
    spill = 32 * 65536 * 8
    assert full >= 32 * 65536 * 16 * 4 + spill and full < 1.3 * 32 * 65536 * 16 * 4 + spill
    assert ekv.ekv_workspace_bytes(cfg, ekv.EKV_OP_SELECT_GAUSS) > 0


@pytest.mark.parametrize("kw,code", [
    (dict(head_dim=64), 2), (dict(page_size=10), 2), (dict(n_q_heads=24, n_kv_heads=8), 2),
    (dict(n_q_heads=30), 1), (dict(alpha=1.0), 1), (dict(scale=0.0), 1), (dict(batch=0), 1),
    (dict(kv_dtype=7), 2), (dict(max_sel_pages=70000), 1),
    (dict(pool_kv_heads=4), 1), (dict(pool_kv_heads=-1), 1),          # fewer pool heads than the config covers
])
def test_bad_config_is_rejected(kw, code):
    lib = ekv.load_library()
    cfg = good_cfg(**kw)
    n = ctypes.c_size_t(0)
    assert lib.ekv_workspace_bytes(ctypes.byref(cfg), ekv.EKV_OP_DECODE_FULL, ctypes.byref(n)) == code


def test_null_and_misaligned_pointers_are_rejected_before_any_launch():
    lib = ekv.load_library()
    cfg = good_cfg()
    cache = ekv.ekv_cache_view(None, None, None, None, 0)
    stats = ekv.ekv_stats_view(None, None)
    assert lib.ekv_stats_build(ctypes.byref(cfg), ctypes.byref(cache), ctypes.byref(stats), None) == 1
    assert lib.ekv_stats_build(None, ctypes.byref(cache), ctypes.byref(stats), None) == 1
    cache = ekv.ekv_cache_view(0x1008, 0x2000, 0x3000, 0x4000, 4)      # k_pool not 16-byte aligned
    stats = ekv.ekv_stats_view(0x5000, 0x6000)
    assert lib.ekv_stats_build(ctypes.byref(cfg), ctypes.byref(cache), ctypes.byref(stats), None) == 1
    assert lib.ekv_score_pages(ctypes.byref(cfg), 0x1000, ctypes.byref(stats), 0x4000, 0, 0x7000, None, None,
                               None) == 1                               # mode 0
    assert lib.ekv_select_topk(ctypes.byref(cfg), 0x1000, 0x2000, 0, 0x3000, 0x4000, None, 0, None) == 1
    assert lib.ekv_select_topk(ctypes.byref(cfg), 0x1000, 0x2000, 5000, 0x3000, 0x4000, None, 0, None) == 1
    # workspace too small / missing
    cache = ekv.ekv_cache_view(0x1000, 0x2000, 0x3000, 0x4000, 4)
    assert lib.ekv_decode_full(ctypes.byref(cfg), 0x1000, ctypes.byref(cache), 0x5000, 0x6000, 0x7000, None,
                               None, 0, None) == 3
    assert lib.ekv_decode_sparse(ctypes.byref(cfg), 0x1000, ctypes.byref(cache), 0x8000, 0x9000, 0x5000, 0x6000,
                                 0x7000, None, 0xA000, 1024, None) == 3
    # Gaussian selector: q_page outside (0,1); non-integer beta
    assert lib.ekv_select_gauss(ctypes.byref(cfg), 0x1000, 0x2000, 0x3000, 1.5, 0.0, 0x4000, 0x5000, 0x6000, 0x7000,
                                0x8000, 4096, None) == 1
    cfg17 = good_cfg(alpha=1.7)
    assert lib.ekv_select_gauss(ctypes.byref(cfg17), 0x1000, 0x2000, 0x3000, 0.9, 0.0, 0x4000, 0x5000, 0x6000,
                                0x7000, 0x8000, 4096, None) == 2


def test_binding_raises_without_fallback(monkeypatch):
    monkeypatch.setattr(ekv, "_lib", None)
    monkeypatch.setattr(ekv, "LIB_PATH", "/nonexistent/libentmaxkv.so")
    with pytest.raises(ekv.EkvError):
        ekv.load_library()


def test_new_entry_points_validate_their_arguments():
    lib = ekv.load_library()
    cfg = good_cfg()
    # box-threshold selection: missing outputs, list given without its length, workspace too small
    assert lib.ekv_select_box_threshold(ctypes.byref(cfg), 0x1000, 0x2000, 0x3000, None, None, None, 0x5000, 0x6000,
                                        0x7000, 0x8000, 1 << 30, None) == 1
    assert lib.ekv_select_box_threshold(ctypes.byref(cfg), 0x1000, 0x2000, 0x3000, 0x4000, None, 0x4000, 0x5000,
                                        0x6000, 0x7000, 0x8000, 1 << 30, None) == 1
    assert lib.ekv_select_box_threshold(ctypes.byref(cfg), 0x1000, 0x2000, 0x3000, None, None, 0x4000, 0x5000,
                                        0x6000, 0x7000, 0x8000, 16, None) == 3
    assert ekv.ekv_workspace_bytes(cfg, ekv.EKV_OP_SELECT_BOX_THRESHOLD) >= 32 * 16 * 4096 * 4
    # group maximum only combines with the box score
    stats = ekv.ekv_stats_view(0x5000, 0x6000)
    bad_mode = ekv.EKV_SCORE_GAUSS | ekv.EKV_SCORE_GROUP_MAX
    assert lib.ekv_score_pages(ctypes.byref(cfg), 0x1000, ctypes.byref(stats), 0x4000, bad_mode, 0x7000, 0x8000,
                               0x9000, None) == 1
    # grouped decode: same checks as the per-head decode
    cache = ekv.ekv_cache_view(0x1000, 0x2000, 0x3000, 0x4000, 4)
    assert lib.ekv_decode_sparse_group(ctypes.byref(cfg), 0x1000, ctypes.byref(cache), None, 0x9000, 0x5000, 0x6000,
                                       0x7000, None, 0xA000, 1 << 40, None) == 1
    assert lib.ekv_decode_sparse_group(ctypes.byref(cfg), 0x1000, ctypes.byref(cache), 0x8000, 0x9000, 0x5000,
                                       0x6000, 0x7000, None, 0xA000, 1024, None) == 3


def test_eight_bit_bounds_are_validated_before_any_launch():
    lib = ekv.load_library()
    cfg = good_cfg()
    mode8 = ekv.EKV_SCORE_BOX8
    # the mode needs the buffer; it does not combine with the cache-dtype box score or the Gaussian moments
    no8 = ekv.ekv_stats_view(0x5000, 0x6000, None)
    assert lib.ekv_score_pages(ctypes.byref(cfg), 0x1000, ctypes.byref(no8), 0x4000, mode8, 0x7000, None, None,
                               None) == 1
    with8 = ekv.ekv_stats_view(0x5000, 0x6000, 0x9000)
    for bad in (mode8 | ekv.EKV_SCORE_BOX, mode8 | ekv.EKV_SCORE_GAUSS, 16):
        assert lib.ekv_score_pages(ctypes.byref(cfg), 0x1000, ctypes.byref(with8), 0x4000, bad, 0x7000, 0x8000,
                                   0xA000, None) == 1
    assert lib.ekv_score_pages(ctypes.byref(cfg), 0x1000, ctypes.byref(with8), 0x4000, mode8, None, None, None,
                               None) == 1                               # no output
    # 16-byte units
    odd = ekv.ekv_stats_view(0x5000, 0x6000, 0x9004)
    cache = ekv.ekv_cache_view(0x1000, 0x2000, 0x3000, 0x4000, 4)
    assert lib.ekv_stats_build(ctypes.byref(cfg), ctypes.byref(cache), ctypes.byref(odd), None) == 1
    assert lib.ekv_stats_append(ctypes.byref(cfg), ctypes.byref(cache), ctypes.byref(odd), 0x7000, None, None) == 1
    # bf16 caches only
    cfg32 = good_cfg(kv_dtype=ekv.EKV_F32)
    assert lib.ekv_stats_build(ctypes.byref(cfg32), ctypes.byref(cache), ctypes.byref(with8), None) == 2
    assert lib.ekv_score_pages(ctypes.byref(cfg32), 0x1000, ctypes.byref(with8), 0x4000, mode8, 0x7000, None, None,
                               None) == 2
    assert lib.ekv_append_score_pages(ctypes.byref(cfg32), ctypes.byref(cache), ctypes.byref(with8), 0x7000, None,
                                      0x1000, mode8, 0x8000, None, None, None) == 2


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    """ekv_decode_sparse_static has a fixed scratch array: a configuration whose decode workspace is larger is
    refused with EKV_ERR_WORKSPACE on the host, before any pointer is looked at or anything is launched."""
    lib = ekv.load_library()
    big = good_cfg(batch=8, max_sel_pages=8192)
    assert ekv.ekv_workspace_bytes(big, ekv.EKV_OP_DECODE_SPARSE) > ekv.EKV_STATIC_SCRATCH_BYTES
    assert lib.ekv_decode_sparse_static(ctypes.byref(big), None, None, None, None, None, None, None, None, None) == 3
    assert lib.ekv_decode_sparse_static(None, None, None, None, None, None, None, None, None, None) == 1
    header = open(os.path.join(ROOT, "include", "entmaxkv.h")).read()
    assert re.search(r"#define\s+EKV_STATIC_SCRATCH_BYTES\s+\(32u\s*<<\s*20\)", header)
    assert ekv.EKV_STATIC_SCRATCH_BYTES == 32 << 20
