"""ctypes binding over the C ABI in include/entmaxkv.h -- argument marshalling only.

Every function has the name of the C entry point it calls and takes torch tensors (device memory
owned by the caller) where the C call takes device pointers.  No step of the method runs in Python.
The shared library is loaded on first use and its absence is an error: there is no fallback path.
"""
import ctypes
import os
from ctypes import c_float, c_int32, c_size_t, c_void_p, POINTER, byref

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libentmaxkv.so")

EKV_OK = 0
EKV_F32, EKV_BF16 = 0, 1
EKV_SCORE_BOX, EKV_SCORE_GAUSS, EKV_SCORE_BOTH, EKV_SCORE_GROUP_MAX, EKV_SCORE_BOX8 = 1, 2, 3, 4, 8
EKV_STATIC_SCRATCH_BYTES = 32 << 20
EKV_OP_SELECT_TOPK, EKV_OP_SELECT_GAUSS, EKV_OP_DECODE_SPARSE, EKV_OP_DECODE_FULL, \
    EKV_OP_DECODE_SPARSE_SOFTMAX, EKV_OP_SELECT_BOX_THRESHOLD = range(6)

# every symbol the header declares
EXPORTS = ["ekv_stats_build", "ekv_stats_append", "ekv_score_pages", "ekv_append_score_pages", "ekv_select_topk",
           "ekv_select_gauss",
           "ekv_select_box_threshold", "ekv_decode_sparse", "ekv_decode_sparse_group", "ekv_decode_full",
           "ekv_decode_sparse_softmax", "ekv_workspace_bytes", "ekv_probe_read", "ekv_decode_sparse_static",
           "ekv_probe_handoff", "ekv_status_string", "ekv_last_hip_error", "ekv_version"]
_STATUS_CALLS = EXPORTS[:15]      # entry points that return ekv_status


class ekv_config(ctypes.Structure):
    _fields_ = [("batch", c_int32), ("n_q_heads", c_int32), ("n_kv_heads", c_int32), ("head_dim", c_int32),
                ("page_size", c_int32), ("kv_dtype", c_int32), ("alpha", c_float), ("scale", c_float),
                ("max_pages_per_seq", c_int32), ("max_sel_pages", c_int32), ("pool_kv_heads", c_int32)]


class ekv_cache_view(ctypes.Structure):
    _fields_ = [("k_pool", c_void_p), ("v_pool", c_void_p), ("block_table", c_void_p), ("seq_lens", c_void_p),
                ("n_phys_pages", c_int32)]


class ekv_stats_view(ctypes.Structure):
    _fields_ = [("box", c_void_p), ("gauss", c_void_p), ("box8", c_void_p)]


class ekv_decode_extras(ctypes.Structure):
    _fields_ = [("support_tokens", c_void_p), ("support_cap", c_int32), ("tau_ref", c_void_p),
                ("kept_mass_ref", c_void_p), ("kept_supp_ref", c_void_p), ("lse", c_void_p),
                ("tau_seed", c_void_p), ("solve_evals", c_void_p), ("score_pass_only", c_int32)]


class EkvError(RuntimeError):
    pass


_lib = None


def load_library():
    """Load libentmaxkv.so (built in-tree by paper_2605_21649_amd.build).  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise EkvError(f"HIP library not built: {LIB_PATH} (run `python -m paper_2605_21649_amd.build`)")
    lib = ctypes.CDLL(LIB_PATH)
    P = POINTER
    lib.ekv_stats_build.argtypes = [P(ekv_config), P(ekv_cache_view), P(ekv_stats_view), c_void_p]
    lib.ekv_stats_append.argtypes = [P(ekv_config), P(ekv_cache_view), P(ekv_stats_view), c_void_p, c_void_p,
                                     c_void_p]
    lib.ekv_score_pages.argtypes = [P(ekv_config), c_void_p, P(ekv_stats_view), c_void_p, c_int32, c_void_p,
                                    c_void_p, c_void_p, c_void_p]
    lib.ekv_append_score_pages.argtypes = [P(ekv_config), P(ekv_cache_view), P(ekv_stats_view), c_void_p, c_void_p,
                                           c_void_p, c_int32, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.ekv_select_topk.argtypes = [P(ekv_config), c_void_p, c_void_p, c_int32, c_void_p, c_void_p, c_void_p,
                                    c_size_t, c_void_p]
    lib.ekv_select_gauss.argtypes = [P(ekv_config), c_void_p, c_void_p, c_void_p, c_float, c_float, c_void_p,
                                     c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    lib.ekv_decode_sparse.argtypes = [P(ekv_config), c_void_p, P(ekv_cache_view), c_void_p, c_void_p, c_void_p,
                                      c_void_p, c_void_p, P(ekv_decode_extras), c_void_p, c_size_t, c_void_p]
    lib.ekv_decode_sparse_group.argtypes = lib.ekv_decode_sparse.argtypes
    lib.ekv_decode_sparse_static.argtypes = [P(ekv_config), c_void_p, P(ekv_cache_view), c_void_p, c_void_p, c_void_p,
                                             c_void_p, c_void_p, P(ekv_decode_extras), c_void_p]
    lib.ekv_decode_full.argtypes = [P(ekv_config), c_void_p, P(ekv_cache_view), c_void_p, c_void_p, c_void_p,
                                    P(ekv_decode_extras), c_void_p, c_size_t, c_void_p]
    lib.ekv_decode_sparse_softmax.argtypes = [P(ekv_config), c_void_p, P(ekv_cache_view), c_void_p, c_void_p,
                                              c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    lib.ekv_workspace_bytes.argtypes = [P(ekv_config), c_int32, P(c_size_t)]
    lib.ekv_status_string.argtypes = [c_int32]
    lib.ekv_status_string.restype = ctypes.c_char_p
    lib.ekv_last_hip_error.restype = c_int32
    lib.ekv_version.restype = c_int32
    lib.ekv_select_box_threshold.argtypes = [P(ekv_config), c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                             c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    lib.ekv_probe_read.argtypes = [c_void_p, c_void_p, c_void_p, c_int32, c_int32, c_void_p, c_void_p, c_void_p]
    lib.ekv_probe_handoff.argtypes = [c_void_p, c_void_p, c_void_p, c_int32, c_int32, c_void_p]
    for name in _STATUS_CALLS:
        getattr(lib, name).restype = c_int32
    _lib = lib
    return lib


def _check(status):
    if status != EKV_OK:
        lib = load_library()
        raise EkvError(f"{lib.ekv_status_string(status).decode()} (hip error {lib.ekv_last_hip_error()})")


def _ptr(t):
    if t is None:
        return None
    assert t.is_contiguous(), "tensors passed to the C ABI must be contiguous"
    return t.data_ptr()


def _stream(stream):
    if stream is not None:
        return stream
    return torch.cuda.current_stream().cuda_stream


def make_config(batch, n_q_heads, n_kv_heads, head_dim, page_size, kv_dtype, alpha, scale, max_pages_per_seq,
                max_sel_pages, pool_kv_heads=0):
    dt = {"f32": EKV_F32, "bf16": EKV_BF16}.get(kv_dtype, kv_dtype)
    return ekv_config(batch, n_q_heads, n_kv_heads, head_dim, page_size, dt, alpha, scale, max_pages_per_seq,
                      max_sel_pages, pool_kv_heads)


def cache_view(k_pool, v_pool, block_table, seq_lens):
    return ekv_cache_view(_ptr(k_pool), _ptr(v_pool), _ptr(block_table), _ptr(seq_lens), k_pool.shape[0])


def cache_view_heads(k_pool, v_pool, block_table, seq_lens, first_kv_head):
    """Cache view of the KV heads from `first_kv_head` on (pools [n_phys][Hkv][P][d]): the pool pointers are
    advanced to that head; use it with a config whose pool_kv_heads is the cache's head count."""
    off = first_kv_head * k_pool.shape[2] * k_pool.shape[3] * k_pool.element_size()
    assert k_pool.is_contiguous() and v_pool.is_contiguous()
    return ekv_cache_view(k_pool.data_ptr() + off, v_pool.data_ptr() + off, _ptr(block_table), _ptr(seq_lens),
                          k_pool.shape[0])


def stats_view(box, gauss, box8=None):
    return ekv_stats_view(_ptr(box), _ptr(gauss), _ptr(box8))


def decode_extras(support_tokens=None, tau_ref=None, kept_mass_ref=None, kept_supp_ref=None, lse=None,
                  tau_seed=None, solve_evals=None, score_pass_only=False):
    cap = support_tokens.shape[-1] if support_tokens is not None else 0
    return ekv_decode_extras(_ptr(support_tokens), cap, _ptr(tau_ref), _ptr(kept_mass_ref), _ptr(kept_supp_ref),
                             _ptr(lse), _ptr(tau_seed), _ptr(solve_evals), 1 if score_pass_only else 0)


def ekv_workspace_bytes(cfg, op):
    n = c_size_t(0)
    _check(load_library().ekv_workspace_bytes(byref(cfg), op, byref(n)))
    return n.value


def ekv_stats_build(cfg, cache, stats, stream=None):
    _check(load_library().ekv_stats_build(byref(cfg), byref(cache), byref(stats), _stream(stream)))


def ekv_stats_append(cfg, cache, stats, k_new, v_new=None, stream=None):
    _check(load_library().ekv_stats_append(byref(cfg), byref(cache), byref(stats), _ptr(k_new), _ptr(v_new),
                                           _stream(stream)))


def ekv_score_pages(cfg, q, stats, seq_lens, mode, box=None, mu=None, sigma=None, stream=None):
    _check(load_library().ekv_score_pages(byref(cfg), _ptr(q), byref(stats), _ptr(seq_lens), mode, _ptr(box),
                                          _ptr(mu), _ptr(sigma), _stream(stream)))


def ekv_append_score_pages(cfg, cache, stats, k_new, v_new, q, mode, box=None, mu=None, sigma=None, stream=None):
    _check(load_library().ekv_append_score_pages(byref(cfg), byref(cache), byref(stats), _ptr(k_new), _ptr(v_new),
                                                 _ptr(q), mode, _ptr(box), _ptr(mu), _ptr(sigma), _stream(stream)))


def ekv_select_topk(cfg, box, seq_lens, k_pages, page_idx, n_sel, workspace, stream=None):
    nbytes = workspace.numel() * workspace.element_size()
    _check(load_library().ekv_select_topk(byref(cfg), _ptr(box), _ptr(seq_lens), k_pages, _ptr(page_idx),
                                          _ptr(n_sel), _ptr(workspace), nbytes, _stream(stream)))


def ekv_select_gauss(cfg, mu, sigma, seq_lens, q_page, margin, tau_hat, page_idx, n_sel, overflow, workspace,
                     stream=None):
    nbytes = workspace.numel() * workspace.element_size()
    _check(load_library().ekv_select_gauss(byref(cfg), _ptr(mu), _ptr(sigma), _ptr(seq_lens), q_page, margin,
                                           _ptr(tau_hat), _ptr(page_idx), _ptr(n_sel), _ptr(overflow),
                                           _ptr(workspace), nbytes, _stream(stream)))


def ekv_select_box_threshold(cfg, box, seq_lens, tau_lo, page_idx_in, n_sel_in, page_idx_out, n_sel_out, n_added,
                             overflow, workspace, stream=None):
    nbytes = workspace.numel() * workspace.element_size()
    _check(load_library().ekv_select_box_threshold(byref(cfg), _ptr(box), _ptr(seq_lens), _ptr(tau_lo),
                                                   _ptr(page_idx_in), _ptr(n_sel_in), _ptr(page_idx_out),
                                                   _ptr(n_sel_out), _ptr(n_added), _ptr(overflow), _ptr(workspace),
                                                   nbytes, _stream(stream)))


def ekv_decode_sparse(cfg, q, cache, page_idx, n_sel, out, tau, supp, workspace, extras=None, stream=None):
    nbytes = workspace.numel() * workspace.element_size()
    ex = byref(extras) if extras is not None else None
    _check(load_library().ekv_decode_sparse(byref(cfg), _ptr(q), byref(cache), _ptr(page_idx), _ptr(n_sel),
                                            _ptr(out), _ptr(tau), _ptr(supp), ex, _ptr(workspace), nbytes,
                                            _stream(stream)))


def ekv_decode_sparse_group(cfg, q, cache, page_idx, n_sel, out, tau, supp, workspace, extras=None, stream=None):
    nbytes = workspace.numel() * workspace.element_size()
    ex = byref(extras) if extras is not None else None
    _check(load_library().ekv_decode_sparse_group(byref(cfg), _ptr(q), byref(cache), _ptr(page_idx), _ptr(n_sel),
                                                  _ptr(out), _ptr(tau), _ptr(supp), ex, _ptr(workspace), nbytes,
                                                  _stream(stream)))


def ekv_decode_full(cfg, q, cache, out, tau, supp, workspace, extras=None, stream=None):
    nbytes = workspace.numel() * workspace.element_size()
    ex = byref(extras) if extras is not None else None
    _check(load_library().ekv_decode_full(byref(cfg), _ptr(q), byref(cache), _ptr(out), _ptr(tau), _ptr(supp), ex,
                                          _ptr(workspace), nbytes, _stream(stream)))


def ekv_decode_sparse_softmax(cfg, q, cache, page_idx, n_sel, out, lse_sel, workspace, stream=None):
    nbytes = workspace.numel() * workspace.element_size()
    _check(load_library().ekv_decode_sparse_softmax(byref(cfg), _ptr(q), byref(cache), _ptr(page_idx),
                                                    _ptr(n_sel), _ptr(out), _ptr(lse_sel), _ptr(workspace), nbytes,
                                                    _stream(stream)))


def ekv_probe_read(base, page_ids, n_pages, page_bytes, sink, lookup=None, out=None, stream=None):
    _check(load_library().ekv_probe_read(_ptr(base), _ptr(page_ids), _ptr(lookup), n_pages, page_bytes, _ptr(out),
                                         _ptr(sink), _stream(stream)))


def ekv_decode_sparse_static(cfg, q, cache, page_idx, n_sel, out, tau, supp, extras=None, stream=None):
    ex = byref(extras) if extras is not None else None
    _check(load_library().ekv_decode_sparse_static(byref(cfg), _ptr(q), byref(cache), _ptr(page_idx), _ptr(n_sel),
                                                   _ptr(out), _ptr(tau), _ptr(supp), ex, _stream(stream)))


def ekv_probe_handoff(data, counter, out, n_workgroups, mode, stream=None):
    _check(load_library().ekv_probe_handoff(_ptr(data), _ptr(counter), _ptr(out), n_workgroups, mode, _stream(stream)))
