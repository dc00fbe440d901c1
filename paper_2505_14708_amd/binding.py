"""Thin ctypes binding over the C-ABI library (include/da.h).

Argument marshalling only: every step of the path runs in the HIP kernels of the library.
PyTorch is used for device memory and streams.  If the library has not been built, loading
fails loudly; there is no fallback.
"""
from __future__ import annotations

import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "lib", "libdraftattn.so")

DA_F32, DA_BF16 = 0, 1
DA_REORDER_ROWS, DA_REORDER_VT, DA_RESTORE, DA_REORDER_VOP = 0, 1, 2, 3


def v_layout(dtype: int) -> int:
    """The da_permute mode that writes V the way da_sparse_attn wants it for this dtype."""
    return DA_REORDER_VOP if dtype == DA_BF16 else DA_REORDER_VT
DA_POOL_AVG, DA_POOL_MAX = 0, 1
DA_OK = 0
DA_STATIC_SCRATCH_BYTES = 32 << 20

EXPORTS = ["da_derive", "da_workspace_size", "da_build_perm", "da_draft_map", "da_select_blocks",
           "da_permute", "da_sparse_attn", "da_forward", "da_forward_ex", "da_global_sizes", "da_select_blocks_global",
           "da_sparse_attn_lists", "da_forward_global", "da_sparse_attn_ex", "da_wait_failures",
           "da_select_blocks_global_static", "da_status_string"]


class da_problem(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("T", ctypes.c_int32), ("fh", ctypes.c_int32),
                ("fw", ctypes.c_int32), ("d", ctypes.c_int32), ("ph", ctypes.c_int32), ("pw", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("keep_blocks", ctypes.c_int32), ("sparsity", ctypes.c_double),
                ("pool", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class da_dims(ctypes.Structure):
    _fields_ = [("gh", ctypes.c_int32), ("gw", ctypes.c_int32), ("g", ctypes.c_int32), ("block", ctypes.c_int32),
                ("k", ctypes.c_int32), ("reserved", ctypes.c_int32), ("n", ctypes.c_int64), ("n_pad", ctypes.c_int64)]


class da_global_dims(ctypes.Structure):
    _fields_ = [("budget", ctypes.c_int64), ("cap", ctypes.c_int64), ("select_ws", ctypes.c_size_t),
                ("forward_ws", ctypes.c_size_t)]


class da_layout(ctypes.Structure):
    _fields_ = [("stride_b", ctypes.c_int64), ("stride_h", ctypes.c_int64), ("stride_n", ctypes.c_int64)]


class DaError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: status {status} ({status_string(status)})")
        self.status = status


_lib = None


def lib() -> ctypes.CDLL:
    """Load the library once.  Raises if it is missing: the product path has no CPU fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built; run `python -m paper_2505_14708_amd.build` "
                               "(or __graft_entry__.build()) first")
        L = ctypes.CDLL(LIB_PATH)
        P, V = ctypes.POINTER(da_problem), ctypes.c_void_p
        L.da_derive.argtypes = [P, ctypes.POINTER(da_dims)]
        L.da_workspace_size.argtypes = [P, ctypes.POINTER(ctypes.c_size_t)]
        L.da_build_perm.argtypes = [P, V, V, V, V]
        L.da_draft_map.argtypes = [P, V, V, V, V, V, V, V]
        L.da_select_blocks.argtypes = [P, V, V, V, V]
        L.da_permute.argtypes = [P, V, V, ctypes.c_int, V]
        L.da_sparse_attn.argtypes = [P, V, V, V, V, V, V, V]
        L.da_forward.argtypes = [P, V, V, V, V, V, V, ctypes.c_size_t, V]
        L.da_forward_ex.argtypes = [P, ctypes.POINTER(da_layout), ctypes.POINTER(da_layout), ctypes.c_int, V, V, V, V, V, V,
                                    ctypes.c_size_t, V]
        L.da_global_sizes.argtypes = [P, ctypes.POINTER(da_global_dims)]
        L.da_select_blocks_global.argtypes = [P, V, V, V, V, V, ctypes.c_size_t, V]
        L.da_select_blocks_global_static.argtypes = [P, V, V, V, V, V]
        L.da_sparse_attn_lists.argtypes = [P, V, V, V, V, V, ctypes.c_int64, V, V, V]
        L.da_forward_global.argtypes = [P, V, V, V, V, V, V, V, ctypes.c_size_t, V]
        L.da_sparse_attn_ex.argtypes = [P, V, V, V, V, V, V, ctypes.c_int, V, V]
        L.da_wait_failures.argtypes = [ctypes.POINTER(ctypes.c_uint64)]
        L.da_status_string.argtypes = [ctypes.c_int]
        L.da_status_string.restype = ctypes.c_char_p
        for name in EXPORTS[:-1]:
            getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().da_status_string(int(status)).decode()


def problem(B, H, T, fh, fw, d, ph=8, pw=8, dtype=DA_BF16, sparsity=0.0, keep_blocks=0, pool=DA_POOL_AVG) -> da_problem:
    return da_problem(B, H, T, fh, fw, d, ph, pw, dtype, keep_blocks, float(sparsity), int(pool), 0)


def problem_of(w) -> da_problem:
    """da_problem for a workloads.Workload."""
    return problem(w.B, w.H, w.T, w.fh, w.fw, w.d, w.ph, w.pw, w.dtype, w.sparsity)


def _check(status: int, what: str):
    if status != DA_OK:
        raise DaError(status, what)


def _ptr(t):
    """Device (or NULL) pointer of a torch tensor / None / raw int."""
    if t is None:
        return None
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def da_derive(p: da_problem) -> da_dims:
    out = da_dims()
    _check(lib().da_derive(ctypes.byref(p), ctypes.byref(out)), "da_derive")
    return out


def da_workspace_size(p: da_problem) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().da_workspace_size(ctypes.byref(p), ctypes.byref(n)), "da_workspace_size")
    return int(n.value)


def da_build_perm(p, perm=None, inv=None, valid=None, stream=None):
    _check(lib().da_build_perm(ctypes.byref(p), _ptr(perm), _ptr(inv), _ptr(valid), _stream(stream)), "da_build_perm")


def da_draft_map(p, Q, K, q_pool, k_pool, logits=None, draft=None, stream=None):
    _check(lib().da_draft_map(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(q_pool), _ptr(k_pool), _ptr(logits),
                              _ptr(draft), _stream(stream)), "da_draft_map")


def da_select_blocks(p, scores, idx, mask=None, stream=None):
    _check(lib().da_select_blocks(ctypes.byref(p), _ptr(scores), _ptr(idx), _ptr(mask), _stream(stream)),
           "da_select_blocks")


def da_permute(p, X, Y, mode, stream=None):
    _check(lib().da_permute(ctypes.byref(p), _ptr(X), _ptr(Y), int(mode), _stream(stream)), "da_permute")


def da_sparse_attn(p, Qp, Kp, Vt, idx, Op, lse=None, stream=None):
    _check(lib().da_sparse_attn(ctypes.byref(p), _ptr(Qp), _ptr(Kp), _ptr(Vt), _ptr(idx), _ptr(Op), _ptr(lse),
                                _stream(stream)), "da_sparse_attn")


def da_forward(p, Q, K, V, O, ws, idx_out=None, stream=None):
    nbytes = ws.numel() * ws.element_size()
    _check(lib().da_forward(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(idx_out), _ptr(ws),
                            ctypes.c_size_t(nbytes), _stream(stream)), "da_forward")


def layout_of(t) -> da_layout:
    """da_layout of a torch tensor viewed as [B, H, rows, d] (any strides, d contiguous)."""
    assert t.dim() == 4 and t.stride(3) == 1
    return da_layout(t.stride(0), t.stride(1), t.stride(2))


def da_forward_ex(p, Q, K, V, O, ws, layout_in=None, layout_out=None, reordered=0, idx_out=None, stream=None):
    nbytes = ws.numel() * ws.element_size()
    li = ctypes.byref(layout_in) if layout_in is not None else None
    lo = ctypes.byref(layout_out) if layout_out is not None else None
    _check(lib().da_forward_ex(ctypes.byref(p), li, lo, int(reordered), _ptr(Q), _ptr(K), _ptr(V), _ptr(O),
                               _ptr(idx_out), _ptr(ws), ctypes.c_size_t(nbytes), _stream(stream)), "da_forward_ex")


def da_global_sizes(p: da_problem) -> da_global_dims:
    out = da_global_dims()
    _check(lib().da_global_sizes(ctypes.byref(p), ctypes.byref(out)), "da_global_sizes")
    return out


def da_select_blocks_global(p, scores, row_ptr, cols, ws, mask=None, stream=None):
    nbytes = ws.numel() * ws.element_size()
    _check(lib().da_select_blocks_global(ctypes.byref(p), _ptr(scores), _ptr(row_ptr), _ptr(cols), _ptr(mask), _ptr(ws),
                                         ctypes.c_size_t(nbytes), _stream(stream)), "da_select_blocks_global")


def da_select_blocks_global_static(p, scores, row_ptr, cols, mask=None, stream=None):
    _check(lib().da_select_blocks_global_static(ctypes.byref(p), _ptr(scores), _ptr(row_ptr), _ptr(cols), _ptr(mask),
                                                _stream(stream)), "da_select_blocks_global_static")


def da_sparse_attn_lists(p, Qp, Kp, Vt, row_ptr, cols, cap, Op, lse=None, stream=None):
    _check(lib().da_sparse_attn_lists(ctypes.byref(p), _ptr(Qp), _ptr(Kp), _ptr(Vt), _ptr(row_ptr), _ptr(cols),
                                      ctypes.c_int64(int(cap)), _ptr(Op), _ptr(lse), _stream(stream)),
           "da_sparse_attn_lists")


def da_forward_global(p, Q, K, V, O, ws, row_ptr_out=None, cols_out=None, stream=None):
    nbytes = ws.numel() * ws.element_size()
    _check(lib().da_forward_global(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(row_ptr_out),
                                   _ptr(cols_out), _ptr(ws), ctypes.c_size_t(nbytes), _stream(stream)),
           "da_forward_global")


def da_sparse_attn_ex(p, Q, Kp, Vt, idx, O, lse=None, original_order=0, tile_counts=None, stream=None):
    _check(lib().da_sparse_attn_ex(ctypes.byref(p), _ptr(Q), _ptr(Kp), _ptr(Vt), _ptr(idx), _ptr(O), _ptr(lse),
                                   int(original_order), _ptr(tile_counts), _stream(stream)), "da_sparse_attn_ex")


def da_wait_failures() -> int:
    """Waves of the bf16 attention kernel that gave up waiting for a tile (synchronises the device)."""
    n = ctypes.c_uint64(0)
    _check(lib().da_wait_failures(ctypes.byref(n)), "da_wait_failures")
    return int(n.value)
