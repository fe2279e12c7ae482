"""Bi-Mask N:M sparse-training hot path for AMD MI355X (gfx950).

Thin Python binding over the C-ABI library `libbimask.so` (declared in
`include/bimask.h`).  The functions here only marshal arguments -- every step
of the path runs in the library's HIP kernels.  PyTorch is used for device
memory and streams only.  There is no CPU fallback: if the library is missing
or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

F32, BF16 = 0, 1
WS_PERM_SEARCH, WS_GEMM_FWD, WS_GEMM_BWD = 0, 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbimask.so")
_lib = None

_I64, _INT, _PTR, _SZ = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
_SIGNATURES = {
    "bimask_forward_mask": (_INT, [_PTR, _I64, _I64, _I64, _INT, _INT, _INT, _PTR, _PTR]),
    "bimask_forward_mask_compress": (_INT, [_PTR, _I64, _I64, _I64, _INT, _INT, _INT, _PTR, _PTR, _PTR, _PTR]),
    "bimask_perm_search": (_INT, [_PTR, _I64, _I64, _INT, _INT, _PTR, _INT, _PTR, _PTR, _PTR, _PTR, _SZ, _PTR]),
    "bimask_perm_search_static": (_INT, [_PTR, _I64, _I64, _INT, _INT, _PTR, _INT, _PTR, _PTR, _PTR, _PTR]),
    "bimask_check_perms": (_INT, [_PTR, _INT, _I64, _PTR, _PTR]),
    "bimask_perm_refine": (_INT, [_PTR, _I64, _I64, _INT, _INT, _PTR, _PTR, _I64, _PTR, _PTR, _PTR]),
    "bimask_backward_mask": (_INT, [_PTR, _I64, _I64, _I64, _INT, _INT, _INT, _PTR, _PTR, _PTR, _PTR]),
    "bimask_backward_mask_compress": (_INT, [_PTR, _I64, _I64, _I64, _INT, _INT, _INT, _PTR, _PTR, _PTR, _PTR, _PTR, _PTR]),
    "bimask_compress_nm": (_INT, [_PTR, _I64, _I64, _I64, _INT, _INT, _INT, _PTR, _PTR, _INT, _PTR, _PTR, _PTR]),
    "bimask_sparse_gemm_fwd": (_INT, [_PTR, _I64, _I64, _PTR, _PTR, _I64, _I64, _INT, _INT, _INT, _PTR, _I64, _PTR, _SZ, _PTR]),
    "bimask_sparse_gemm_bwd": (_INT, [_PTR, _I64, _I64, _PTR, _PTR, _PTR, _I64, _I64, _INT, _INT, _INT, _PTR, _I64, _PTR, _SZ, _PTR]),
    "bimask_forward_mask_compress_group": (_INT, [_PTR, _INT, _INT, _INT, _INT, _PTR]),
    "bimask_perm_search_group": (_INT, [_PTR, _INT, _INT, _INT, _INT, _PTR]),
    "bimask_backward_mask_compress_group": (_INT, [_PTR, _INT, _INT, _INT, _INT, _PTR]),
    "bimask_perm_refine_group": (_INT, [_PTR, _INT, _INT, _INT, _PTR]),
    "bimask_operand_elems": (_I64, [_I64, _I64, _INT, _INT]),
    "bimask_operand_index_words": (_I64, [_I64, _I64, _INT, _INT]),
    "bimask_workspace_bytes": (_SZ, [_INT, _I64, _I64, _I64, _INT, _INT, _INT, _INT]),
    "bimask_status_string": (ctypes.c_char_p, [_INT]),
}
EXPORTS = tuple(_SIGNATURES)


class BimaskError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        super().__init__(f"{fn} failed with status {status}: {status_string(status)}")


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2302_06058_amd.build` "
                "(there is no CPU fallback)")
        l = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(l, name)
            fn.restype, fn.argtypes = res, args
        _lib = l
    return _lib


def status_string(status: int) -> str:
    return lib().bimask_status_string(int(status)).decode()


def _check(fn: str, status: int) -> None:
    if status != 0:
        raise BimaskError(fn, status)


# -- tensor helpers (device memory and streams only) ---------------------------------
def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _need_cuda(*ts):
    for t in ts:
        if t is not None and not t.is_cuda:
            raise ValueError("all tensors must live on the GPU")


def _rowmajor(t):
    if t.dim() != 2 or t.stride(1) != 1:
        raise ValueError("expected a 2-D tensor with unit stride along its last dimension")
    return t.stride(0)


def mask_words(cols: int) -> int:
    return (cols + 31) // 32


def workspace_bytes(kind: int, I: int, J: int, T: int, K: int, dtype: int, N: int, M: int) -> int:
    return int(lib().bimask_workspace_bytes(kind, I, J, T, K, dtype, N, M))


def _empty(shape, dtype, like):
    import torch
    return torch.empty(shape, dtype=dtype, device=like.device)


def operand_elems(rows: int, cols: int, N: int, M: int) -> int:
    return int(lib().bimask_operand_elems(rows, cols, N, M))


def operand_index_words(rows: int, cols: int, N: int, M: int) -> int:
    return int(lib().bimask_operand_index_words(rows, cols, N, M))


def _values_shape(rows: int, cols: int, N: int, M: int):
    """Flat fragment-major buffer (see include/bimask.h): 2-of-4 compressed for N <= 2, dense masked for N > 2."""
    return (operand_elems(rows, cols, N, M),)


def _index_shape(rows: int, cols: int, N: int, M: int):
    return (operand_index_words(rows, cols, N, M),)


def prepare(name: str, *args):
    """Bind one call of include/bimask.h to already marshalled arguments.

    `args` are exactly the C arguments, in order; tensors are replaced by their device
    addresses once, here.  The returned callable issues the C call and checks its status,
    nothing else: for launch-bound loops where the per-call marshalling of the wrappers
    below (shape checks, pointer and stream look-ups) would cost more than the kernels.
    The caller keeps the tensors alive and passes the stream handle explicitly."""
    fn = getattr(lib(), name)
    cargs = tuple(a.data_ptr() if hasattr(a, "data_ptr") else a for a in args)

    def call():
        st = fn(*cargs)
        if st:
            raise BimaskError(name, st)
    return call


# -- the calls of include/bimask.h -----------------------------------------------------
def bimask_forward_mask(W, N: int, M: int, B_bits=None):
    import torch
    _need_cuda(W, B_bits)
    I, J = W.shape
    ldw = _rowmajor(W)
    if B_bits is None:
        B_bits = _empty((I, mask_words(J)), torch.int32, W)
    _check("bimask_forward_mask",
           lib().bimask_forward_mask(_ptr(W), I, J, ldw, _dtype_code(W), N, M, _ptr(B_bits), _stream()))
    return B_bits


def bimask_forward_mask_compress(W, N: int, M: int, B_bits=None, values=None, index=None):
    import torch
    _need_cuda(W, B_bits, values, index)
    I, J = W.shape
    ldw = _rowmajor(W)
    if B_bits is None:
        B_bits = _empty((I, mask_words(J)), torch.int32, W)
    if values is None:
        values = _empty(_values_shape(I, J, N, M), W.dtype, W)
    if index is None and N <= 2:
        index = _empty(_index_shape(I, J, N, M), torch.int32, W)
    _check("bimask_forward_mask_compress",
           lib().bimask_forward_mask_compress(_ptr(W), I, J, ldw, _dtype_code(W), N, M, _ptr(B_bits),
                                              _ptr(values), _ptr(index), _stream()))
    return B_bits, values, index


def bimask_perm_search(B_bits, I: int, J: int, N: int, M: int, perms, scores=None, best=None,
                       best_perm=None, workspace=None, want_best_perm: bool = True):
    import torch
    _need_cuda(B_bits, perms, scores, best, best_perm, workspace)
    K = perms.shape[0]
    if perms.dtype != torch.int32 or not perms.is_contiguous() or perms.shape[1] != I:
        raise ValueError("perms must be a contiguous K x I int32 tensor")
    if scores is None:
        scores = _empty((K,), torch.int32, perms)
    if best is None:
        best = _empty((1,), torch.int32, perms)
    if best_perm is None and want_best_perm:
        best_perm = _empty((I,), torch.int32, perms)
    need = workspace_bytes(WS_PERM_SEARCH, I, J, 0, K, BF16, N, M)
    if workspace is None:
        workspace = _empty((max(need, 16),), torch.uint8, perms)
    _check("bimask_perm_search",
           lib().bimask_perm_search(_ptr(B_bits), I, J, N, M, _ptr(perms), K, _ptr(scores), _ptr(best),
                                    _ptr(best_perm), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                    _stream()))
    return scores, best, best_perm


def bimask_perm_search_static(B_bits, I: int, J: int, N: int, M: int, perms, scores, best, best_perm=None):
    """bimask_perm_search without a workspace and without any allocation: every output is the caller's."""
    import torch
    _need_cuda(B_bits, perms, scores, best, best_perm)
    K = perms.shape[0]
    if perms.dtype != torch.int32 or not perms.is_contiguous() or perms.shape[1] != I:
        raise ValueError("perms must be a contiguous K x I int32 tensor")
    _check("bimask_perm_search_static",
           lib().bimask_perm_search_static(_ptr(B_bits), I, J, N, M, _ptr(perms), K, _ptr(scores), _ptr(best),
                                           _ptr(best_perm), _stream()))
    return scores, best, best_perm


def bimask_check_perms(perms, ok=None):
    """Debug helper: int32[K] of flags, 1 where the candidate is a permutation of 0 .. I-1."""
    import torch
    _need_cuda(perms, ok)
    if perms.dtype != torch.int32 or not perms.is_contiguous() or perms.dim() != 2:
        raise ValueError("perms must be a contiguous K x I int32 tensor")
    K, I = perms.shape
    if ok is None:
        ok = _empty((K,), torch.int32, perms)
    _check("bimask_check_perms", lib().bimask_check_perms(_ptr(perms), K, I, _ptr(ok), _stream()))
    return ok


def bimask_perm_refine(B_bits, I: int, J: int, N: int, M: int, swaps, perm=None, perm_out=None, result=None):
    """Hill climbing over proposed exchanges of two positions; returns (perm_out, result) with
    result = [gain in eligible blocks, proposals kept]."""
    import torch
    _need_cuda(B_bits, swaps, perm, perm_out, result)
    if swaps.dtype != torch.int32 or not swaps.is_contiguous() or swaps.dim() != 2 or swaps.shape[1] != 2:
        raise ValueError("swaps must be a contiguous S x 2 int32 tensor")
    if perm is not None and (perm.dtype != torch.int32 or not perm.is_contiguous() or perm.numel() != I):
        raise ValueError("perm must be a contiguous int32 tensor of I entries")
    if perm_out is None:
        perm_out = _empty((I,), torch.int32, B_bits)
    if result is None:
        result = _empty((2,), torch.int32, B_bits)
    _check("bimask_perm_refine",
           lib().bimask_perm_refine(_ptr(B_bits), I, J, N, M, _ptr(perm), _ptr(swaps) if swaps.shape[0] else None,
                                    swaps.shape[0], _ptr(perm_out), _ptr(result), _stream()))
    return perm_out, result


def bimask_backward_mask(W, N: int, M: int, B_bits, perm=None, Bbar_bits=None):
    import torch
    _need_cuda(W, B_bits, perm, Bbar_bits)
    I, J = W.shape
    ldw = _rowmajor(W)
    if Bbar_bits is None:
        Bbar_bits = _empty((I, mask_words(J)), torch.int32, W)
    _check("bimask_backward_mask",
           lib().bimask_backward_mask(_ptr(W), I, J, ldw, _dtype_code(W), N, M, _ptr(B_bits), _ptr(perm),
                                      _ptr(Bbar_bits), _stream()))
    return Bbar_bits


def bimask_backward_mask_compress(W, N: int, M: int, B_bits, perm=None, Bbar_bits=None, values=None, index=None):
    import torch
    _need_cuda(W, B_bits, perm, Bbar_bits, values, index)
    I, J = W.shape
    ldw = _rowmajor(W)
    if Bbar_bits is None:
        Bbar_bits = _empty((I, mask_words(J)), torch.int32, W)
    if values is None:
        values = _empty(_values_shape(J, I, N, M), W.dtype, W)
    if index is None and N <= 2:
        index = _empty(_index_shape(J, I, N, M), torch.int32, W)
    _check("bimask_backward_mask_compress",
           lib().bimask_backward_mask_compress(_ptr(W), I, J, ldw, _dtype_code(W), N, M, _ptr(B_bits), _ptr(perm),
                                               _ptr(Bbar_bits), _ptr(values), _ptr(index), _stream()))
    return Bbar_bits, values, index


def bimask_compress_nm(W, N: int, M: int, mask_bits, perm=None, transposed: int = 0, values=None, index=None):
    import torch
    _need_cuda(W, mask_bits, perm, values, index)
    I, J = W.shape
    ldw = _rowmajor(W)
    rows, cols = (J, I) if transposed else (I, J)
    if values is None:
        values = _empty(_values_shape(rows, cols, N, M), W.dtype, W)
    if index is None and N <= 2:
        index = _empty(_index_shape(rows, cols, N, M), torch.int32, W)
    _check("bimask_compress_nm",
           lib().bimask_compress_nm(_ptr(W), I, J, ldw, _dtype_code(W), N, M, _ptr(mask_bits), _ptr(perm),
                                    int(transposed), _ptr(values), _ptr(index), _stream()))
    return values, index


def bimask_sparse_gemm_fwd(X, Wf_values, Wf_index, I: int, J: int, N: int, M: int, Y=None, workspace=None):
    _need_cuda(X, Wf_values, Wf_index, Y, workspace)
    T = X.shape[0]
    ldx = _rowmajor(X)
    if Y is None:
        Y = _empty((T, I), X.dtype, X)
    ldy = _rowmajor(Y)
    wsb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check("bimask_sparse_gemm_fwd",
           lib().bimask_sparse_gemm_fwd(_ptr(X), T, ldx, _ptr(Wf_values), _ptr(Wf_index), I, J, _dtype_code(X),
                                        N, M, _ptr(Y), ldy, _ptr(workspace), wsb, _stream()))
    return Y


def bimask_sparse_gemm_bwd(dY, perm, Wb_values, Wb_index, I: int, J: int, N: int, M: int, dX=None, workspace=None):
    import torch
    _need_cuda(dY, perm, Wb_values, Wb_index, dX, workspace)
    T = dY.shape[0]
    lddy = _rowmajor(dY)
    if dX is None:
        dX = _empty((T, J), dY.dtype, dY)
    lddx = _rowmajor(dX)
    if workspace is None and perm is not None:
        need = workspace_bytes(WS_GEMM_BWD, I, J, T, 0, _dtype_code(dY), N, M)
        workspace = _empty((max(need, 16),), torch.uint8, dY)
    wsb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check("bimask_sparse_gemm_bwd",
           lib().bimask_sparse_gemm_bwd(_ptr(dY), T, lddy, _ptr(perm), _ptr(Wb_values), _ptr(Wb_index), I, J,
                                        _dtype_code(dY), N, M, _ptr(dX), lddx, _ptr(workspace), wsb, _stream()))
    return dX


# -- grouped calls: the mask / search steps of several independent layers in a few launches -------
class GroupLayer(ctypes.Structure):
    """Mirror of `bimask_group_layer` (include/bimask.h): one layer of a grouped call."""
    _fields_ = [("W", _PTR), ("I", _I64), ("J", _I64), ("ldw", _I64), ("B_bits", _PTR), ("Wf_values", _PTR),
                ("Wf_index", _PTR), ("perms", _PTR), ("scores", _PTR), ("best", _PTR), ("best_perm", _PTR),
                ("workspace", _PTR), ("workspace_bytes", _SZ), ("Bbar_bits", _PTR), ("Wb_values", _PTR),
                ("Wb_index", _PTR), ("swaps", _PTR), ("n_swaps", _I64), ("refine_result", _PTR)]


def group_layers(entries):
    """A host array of `bimask_group_layer` from dicts of tensors / ints (argument marshalling only).
    Keys: W (2-D tensor), B_bits, Wf_values, Wf_index, perms, scores, best, best_perm, workspace, Bbar_bits,
    Wb_values, Wb_index, swaps (S x 2 int32), refine_result -- absent keys stay NULL.  The tensors must outlive
    the calls that use the array."""
    arr = (GroupLayer * len(entries))()
    for g, e in zip(arr, entries):
        W = e["W"]
        _need_cuda(*[v for v in e.values() if hasattr(v, "is_cuda")])
        g.W, g.I, g.J, g.ldw = W.data_ptr(), W.shape[0], W.shape[1], _rowmajor(W)
        for key in ("B_bits", "Wf_values", "Wf_index", "perms", "scores", "best", "best_perm", "Bbar_bits",
                    "Wb_values", "Wb_index", "swaps", "refine_result"):
            setattr(g, key, _ptr(e.get(key)))
        g.n_swaps = 0 if e.get("swaps") is None else e["swaps"].shape[0]
        ws = e.get("workspace")
        g.workspace = _ptr(ws)
        g.workspace_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    return arr


def bimask_forward_mask_compress_group(layers, dtype: int, N: int, M: int) -> None:
    _check("bimask_forward_mask_compress_group",
           lib().bimask_forward_mask_compress_group(ctypes.cast(layers, _PTR), len(layers), dtype, N, M, _stream()))


def bimask_perm_search_group(layers, N: int, M: int, K: int) -> None:
    _check("bimask_perm_search_group",
           lib().bimask_perm_search_group(ctypes.cast(layers, _PTR), len(layers), N, M, K, _stream()))


def bimask_perm_refine_group(layers, N: int, M: int) -> None:
    _check("bimask_perm_refine_group",
           lib().bimask_perm_refine_group(ctypes.cast(layers, _PTR), len(layers), N, M, _stream()))


def bimask_backward_mask_compress_group(layers, dtype: int, N: int, M: int) -> None:
    _check("bimask_backward_mask_compress_group",
           lib().bimask_backward_mask_compress_group(ctypes.cast(layers, _PTR), len(layers), dtype, N, M, _stream()))
