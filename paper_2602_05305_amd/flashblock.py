"""Thin ctypes binding over libflashblock.so (contract: include/flashblock.h, measurement hooks:
include/flashblock_prof.h).

Argument marshalling only: every function here has the name of the C entry point it calls,
takes torch tensors for device buffers (PyTorch is used for device memory and streams, nothing
else) and raises FlashBlockError on a non-zero status.  No arithmetic of the method happens in
Python, and there is no fallback: if the HIP library is not built, loading fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, Structure, c_char_p, c_float, c_int, c_int32, c_size_t, c_uint32, c_void_p

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libflashblock.so")

FB_OK, FB_ERR_NULL, FB_ERR_SHAPE, FB_ERR_DTYPE, FB_ERR_ALIGN, FB_ERR_WORKSPACE, FB_ERR_UNSUPPORTED, FB_ERR_HIP = range(8)
FB_F32, FB_BF16 = 0, 1
FB_SPARSE_REFRESH, FB_SPARSE_REUSE, FB_SPARSE_REUSE_SAME_SELECTION = 0, 1, 2
FB_MAX_SPLITS = 256


class fb_shape(Structure):
    _fields_ = [("struct_size", c_uint32), ("batch", c_int32), ("n_q_heads", c_int32),
                ("n_kv_heads", c_int32), ("head_dim", c_int32), ("block_len", c_int32),
                ("prefix_len", c_int32), ("dtype", c_int32), ("scale", c_float)]


class fb_paged_kv(Structure):
    _fields_ = [("struct_size", c_uint32), ("num_pages", c_int32), ("page_size", c_int32), ("max_pages", c_int32),
                ("k_pool", c_void_p), ("v_pool", c_void_p), ("block_table", c_void_p), ("prefix_lens", c_void_p)]


class FlashBlockError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str = ""):
        self.status = status
        super().__init__(f"{where}: status {status} ({detail})")


_lib = None

_SIGNATURES = {
    "fb_version": (c_int, []),
    "fb_status_string": (c_char_p, [c_int]),
    "fb_last_hip_error": (c_char_p, []),
    "fb_check_shape": (c_int, [POINTER(fb_shape)]),
    "fb_external_splits": (c_int32, [POINTER(fb_shape)]),
    "fb_external_kernel_name": (c_char_p, [POINTER(fb_shape)]),
    "fb_workspace_bytes": (c_size_t, [POINTER(fb_shape), c_int32, c_int32, c_int32]),
    "fb_external_partial": (c_int, [POINTER(fb_shape)] + [c_void_p] * 7 + [c_size_t, c_void_p]),
    "fb_external_partial_ex": (c_int, [POINTER(fb_shape)] + [c_void_p] * 6 + [c_int32, c_void_p, c_size_t, c_void_p]),
    "fb_external_partial_prof": (c_int, [POINTER(fb_shape)] + [c_void_p] * 6 + [c_int32, c_void_p, c_size_t] + [c_void_p] * 4),
    "fb_builtin_workspace_bytes": (c_size_t, []),
    "fb_external_partial_builtin_ws": (c_int, [POINTER(fb_shape)] + [c_void_p] * 7),
    "fb_external_heads_splits": (c_int32, [POINTER(fb_shape), c_int32]),
    "fb_external_partial_heads": (c_int, [POINTER(fb_shape)] + [c_void_p] * 4 + [c_int32] + [c_void_p] * 4
                                  + [c_size_t, c_void_p]),
    "fb_paged_splits": (c_int32, [POINTER(fb_shape)]),
    "fb_external_partial_paged": (c_int, [POINTER(fb_shape), c_void_p, POINTER(fb_paged_kv)] + [c_void_p] * 3
                                  + [c_int32, c_void_p, c_size_t, c_void_p]),
    "fb_refresh_step_paged": (c_int, [POINTER(fb_shape), c_void_p, POINTER(fb_paged_kv)] + [c_void_p] * 7
                              + [c_int32, c_void_p, c_size_t, c_void_p]),
    "fb_head_similarity": (c_int, [POINTER(fb_shape)] + [c_void_p] * 4),
    "fb_internal_merge": (c_int, [POINTER(fb_shape)] + [c_void_p] * 9),
    "fb_refresh_step": (c_int, [POINTER(fb_shape)] + [c_void_p] * 11 + [c_size_t, c_void_p]),
    "fb_refresh_step_prof": (c_int, [POINTER(fb_shape)] + [c_void_p] * 11 + [c_size_t] + [c_void_p] * 4),
    "fb_pool_keys": (c_int, [POINTER(fb_shape), c_void_p, c_int32, c_void_p, c_void_p]),
    "fb_select_workspace_bytes": (c_size_t, [POINTER(fb_shape), c_int32]),
    "fb_select_topk": (c_int, [POINTER(fb_shape), c_void_p, c_void_p, c_int32, c_int32, c_void_p, c_void_p, c_size_t,
                               c_void_p]),
    "fb_select_mass_workspace_bytes": (c_size_t, [POINTER(fb_shape), c_int32]),
    "fb_select_topk_mass": (c_int, [POINTER(fb_shape), c_void_p, c_void_p, c_void_p, c_int32, c_int32, c_void_p,
                                    c_void_p, c_void_p, c_size_t, c_void_p]),
    "fb_sparse_external_residual": (c_int, [POINTER(fb_shape), c_int32, c_void_p, c_void_p, c_void_p, c_int32,
                                            c_int32] + [c_void_p] * 8 + [c_size_t, c_void_p]),
}


def load_library():
    """Load libflashblock.so (built by `python -m paper_2602_05305_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2602_05305_amd.build` "
                               "(there is no CPU fallback)")
        # PyTorch ships its own copy of the HIP runtime; the library must bind to that same copy (device memory and
        # streams come from torch), so torch is loaded first: whichever libamdhip64 is in the process first serves both.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def exported_symbols():
    return sorted(_SIGNATURES)


def make_shape(batch, n_q_heads, n_kv_heads, head_dim, block_len, prefix_len, dtype, scale=0.0) -> fb_shape:
    code = {"f32": FB_F32, "bf16": FB_BF16}.get(dtype, dtype)
    return fb_shape(ctypes.sizeof(fb_shape), batch, n_q_heads, n_kv_heads, head_dim, block_len, prefix_len,
                    int(code), float(scale))


def _ptr(t):
    return None if t is None else c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return c_void_p(stream.cuda_stream) if hasattr(stream, "cuda_stream") else c_void_p(stream)


def _check(status, where):
    if status != FB_OK:
        lib = load_library()
        detail = lib.fb_status_string(status).decode()
        if status == FB_ERR_HIP:
            detail += ": " + lib.fb_last_hip_error().decode()
        raise FlashBlockError(status, where, detail)


def fb_version() -> int:
    return load_library().fb_version()


def fb_check_shape(shape: fb_shape) -> int:
    return load_library().fb_check_shape(ctypes.byref(shape))


def fb_external_splits(shape: fb_shape) -> int:
    return load_library().fb_external_splits(ctypes.byref(shape))


def fb_external_kernel_name(shape: fb_shape) -> str:
    return load_library().fb_external_kernel_name(ctypes.byref(shape)).decode()


def fb_workspace_bytes(shape: fb_shape, key_block: int = 0, topk: int = 0, n_splits: int = 0) -> int:
    return load_library().fb_workspace_bytes(ctypes.byref(shape), key_block, topk, n_splits)


def fb_external_partial(shape, q, k_prefix, v_prefix, o_part, m_part, lse_part, workspace, stream=None):
    st = load_library().fb_external_partial(ctypes.byref(shape), _ptr(q), _ptr(k_prefix), _ptr(v_prefix),
                                            _ptr(o_part), _ptr(m_part), _ptr(lse_part), _ptr(workspace),
                                            workspace.numel() * workspace.element_size(), _stream(stream))
    _check(st, "fb_external_partial")


def fb_external_partial_ex(shape, q, k_prefix, v_prefix, o_part, m_part, lse_part, n_splits, workspace, stream=None):
    st = load_library().fb_external_partial_ex(ctypes.byref(shape), _ptr(q), _ptr(k_prefix), _ptr(v_prefix),
                                               _ptr(o_part), _ptr(m_part), _ptr(lse_part), n_splits, _ptr(workspace),
                                               workspace.numel() * workspace.element_size(), _stream(stream))
    _check(st, "fb_external_partial_ex")


def fb_external_partial_prof(shape, q, k_prefix, v_prefix, o_part, m_part, lse_part, n_splits, workspace,
                             ev_begin, ev_attn_end, ev_end, stream=None):
    """ev_*: raw hipEvent_t handles (ints / c_void_p) or None."""
    st = load_library().fb_external_partial_prof(ctypes.byref(shape), _ptr(q), _ptr(k_prefix), _ptr(v_prefix),
                                                 _ptr(o_part), _ptr(m_part), _ptr(lse_part), n_splits, _ptr(workspace),
                                                 workspace.numel() * workspace.element_size(), ev_begin, ev_attn_end,
                                                 ev_end, _stream(stream))
    _check(st, "fb_external_partial_prof")


def fb_builtin_workspace_bytes() -> int:
    return int(load_library().fb_builtin_workspace_bytes())


def fb_external_partial_builtin_ws(shape, q, k_prefix, v_prefix, o_part, m_part, lse_part, stream=None):
    st = load_library().fb_external_partial_builtin_ws(ctypes.byref(shape), _ptr(q), _ptr(k_prefix), _ptr(v_prefix),
                                                       _ptr(o_part), _ptr(m_part), _ptr(lse_part), _stream(stream))
    _check(st, "fb_external_partial_builtin_ws")


def fb_external_heads_splits(shape, n_active_heads) -> int:
    return int(load_library().fb_external_heads_splits(ctypes.byref(shape), n_active_heads))


def fb_external_partial_heads(shape, q, k_prefix, v_prefix, head_mask, o_part, m_part, lse_part, workspace,
                              n_active_heads=0, stream=None):
    st = load_library().fb_external_partial_heads(ctypes.byref(shape), _ptr(q), _ptr(k_prefix), _ptr(v_prefix),
                                                  _ptr(head_mask), n_active_heads, _ptr(o_part), _ptr(m_part),
                                                  _ptr(lse_part),
                                                  _ptr(workspace), workspace.numel() * workspace.element_size(),
                                                  _stream(stream))
    _check(st, "fb_external_partial_heads")


def make_paged_kv(k_pool, v_pool, block_table, prefix_lens) -> fb_paged_kv:
    """k_pool / v_pool: [num_pages, Hkv, page_size, d]; block_table int32 [B, max_pages]; prefix_lens int32 [B].
    The struct holds raw device addresses only: the caller keeps the four tensors alive while it is in use."""
    return fb_paged_kv(ctypes.sizeof(fb_paged_kv), k_pool.shape[0], k_pool.shape[2], block_table.shape[1],
                       k_pool.data_ptr(), v_pool.data_ptr(), block_table.data_ptr(), prefix_lens.data_ptr())


def fb_paged_splits(shape) -> int:
    return int(load_library().fb_paged_splits(ctypes.byref(shape)))


def fb_external_partial_paged(shape, q, kv, o_part, m_part, lse_part, workspace, n_splits=0, stream=None):
    st = load_library().fb_external_partial_paged(ctypes.byref(shape), _ptr(q), ctypes.byref(kv), _ptr(o_part),
                                                  _ptr(m_part), _ptr(lse_part), n_splits, _ptr(workspace),
                                                  workspace.numel() * workspace.element_size(), _stream(stream))
    _check(st, "fb_external_partial_paged")


def fb_refresh_step_paged(shape, q, kv, k_block, v_block, o_part, m_part, lse_part, out, lse_out, workspace,
                          n_splits=0, stream=None):
    st = load_library().fb_refresh_step_paged(ctypes.byref(shape), _ptr(q), ctypes.byref(kv), _ptr(k_block),
                                              _ptr(v_block), _ptr(o_part), _ptr(m_part), _ptr(lse_part), _ptr(out),
                                              _ptr(lse_out), n_splits, _ptr(workspace),
                                              workspace.numel() * workspace.element_size(), _stream(stream))
    _check(st, "fb_refresh_step_paged")


def fb_head_similarity(shape, o_a, o_b, sim, stream=None):
    st = load_library().fb_head_similarity(ctypes.byref(shape), _ptr(o_a), _ptr(o_b), _ptr(sim), _stream(stream))
    _check(st, "fb_head_similarity")


def fb_internal_merge(shape, q, k_block, v_block, o_part, m_part, lse_part, out, lse_out=None, stream=None):
    st = load_library().fb_internal_merge(ctypes.byref(shape), _ptr(q), _ptr(k_block), _ptr(v_block), _ptr(o_part),
                                          _ptr(m_part), _ptr(lse_part), _ptr(out), _ptr(lse_out), _stream(stream))
    _check(st, "fb_internal_merge")


def fb_refresh_step(shape, q, k_prefix, v_prefix, k_block, v_block, o_part, m_part, lse_part, out, lse_out,
                    workspace, stream=None):
    st = load_library().fb_refresh_step(ctypes.byref(shape), _ptr(q), _ptr(k_prefix), _ptr(v_prefix), _ptr(k_block),
                                        _ptr(v_block), _ptr(o_part), _ptr(m_part), _ptr(lse_part), _ptr(out),
                                        _ptr(lse_out), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                        _stream(stream))
    _check(st, "fb_refresh_step")


def fb_refresh_step_prof(shape, q, k_prefix, v_prefix, k_block, v_block, o_part, m_part, lse_part, out, lse_out,
                         workspace, ev_begin, ev_attn_end, ev_end, stream=None):
    st = load_library().fb_refresh_step_prof(ctypes.byref(shape), _ptr(q), _ptr(k_prefix), _ptr(v_prefix),
                                             _ptr(k_block), _ptr(v_block), _ptr(o_part), _ptr(m_part),
                                             _ptr(lse_part), _ptr(out), _ptr(lse_out), _ptr(workspace),
                                             workspace.numel() * workspace.element_size(),
                                             ev_begin, ev_attn_end, ev_end, _stream(stream))
    _check(st, "fb_refresh_step_prof")


def fb_pool_keys(shape, k_prefix, key_block, k_pooled, stream=None):
    st = load_library().fb_pool_keys(ctypes.byref(shape), _ptr(k_prefix), key_block, _ptr(k_pooled), _stream(stream))
    _check(st, "fb_pool_keys")


def fb_select_workspace_bytes(shape, key_block) -> int:
    return int(load_library().fb_select_workspace_bytes(ctypes.byref(shape), key_block))


def fb_select_topk(shape, q, k_pooled, key_block, topk, sel_idx, workspace=None, stream=None):
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = load_library().fb_select_topk(ctypes.byref(shape), _ptr(q), _ptr(k_pooled), key_block, topk, _ptr(sel_idx),
                                       _ptr(workspace), nbytes, _stream(stream))
    _check(st, "fb_select_topk")


def fb_select_mass_workspace_bytes(shape, key_block) -> int:
    return int(load_library().fb_select_mass_workspace_bytes(ctypes.byref(shape), key_block))


def fb_select_topk_mass(shape, q, k_prefix, lse_part, key_block, topk, sel_idx, mass_out, workspace, stream=None):
    st = load_library().fb_select_topk_mass(ctypes.byref(shape), _ptr(q), _ptr(k_prefix), _ptr(lse_part), key_block,
                                            topk, _ptr(sel_idx), _ptr(mass_out), _ptr(workspace),
                                            workspace.numel() * workspace.element_size(), _stream(stream))
    _check(st, "fb_select_topk_mass")


def fb_sparse_external_residual(shape, mode, q, k_prefix, v_prefix, key_block, topk, sel_idx, res_o, res_m, res_lse,
                                o_part, m_part, lse_part, workspace, stream=None):
    st = load_library().fb_sparse_external_residual(
        ctypes.byref(shape), mode, _ptr(q), _ptr(k_prefix), _ptr(v_prefix), key_block, topk, _ptr(sel_idx),
        _ptr(res_o), _ptr(res_m), _ptr(res_lse), _ptr(o_part), _ptr(m_part), _ptr(lse_part), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream))
    _check(st, "fb_sparse_external_residual")
