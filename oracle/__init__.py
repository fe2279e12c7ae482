"""CPU oracle for the Bi-Mask hot path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over `bimask_oracle.c` (plain C loops in double precision)
plus float64 numpy matmuls for full-size GEMM references.  Only tests, the
smoke check and the benchmark's cpu_baseline leg may import this package; the
product (`paper_2302_06058_amd`) never does, and nothing here imports it.

All arrays are host numpy arrays:
  W, X, dY : float64 (the exact values of the stored bf16 / fp32 numbers)
  masks    : uint8 0/1, shape I x J
  perms    : int32, shape K x I (gather form: permuted row r = original row P[r])
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bimask_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()                                   # compiles when the library is missing or older than its source
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_argmax.restype = ctypes.c_int
        _lib.oracle_relative_gap.restype = ctypes.c_double
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _u8(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.uint8)


def _i32(a) -> Optional[np.ndarray]:
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _i64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int64)


def _check_nm(I: int, J: int, N: int, M: int, cols_grouped: bool = True, rows_grouped: bool = False):
    assert 1 <= N < M <= 64
    if cols_grouped:
        assert J % M == 0, "J must be a multiple of M"
    if rows_grouped:
        assert I % M == 0, "I must be a multiple of M"


# ---------------------------------------------------------------- masks
def forward_mask(W, N: int, M: int) -> np.ndarray:
    """Eq. (4): top-N magnitudes in every group of M consecutive columns."""
    W = _f64(W)
    I, J = W.shape
    _check_nm(I, J, N, M)
    B = np.empty((I, J), dtype=np.uint8)
    _load().oracle_forward_mask(_p(W), ctypes.c_int64(I), ctypes.c_int64(J), N, M, _p(B))
    return B


def perm_scores(B, perms, N: int, M: int) -> np.ndarray:
    """Sec. 3.3 / Alg. 1: eligible N:M column blocks of (B.*W)[P,:] per candidate."""
    B = _u8(B)
    perms = _i32(np.atleast_2d(perms))
    I, J = B.shape
    K = perms.shape[0]
    assert perms.shape[1] == I
    _check_nm(I, J, N, M, cols_grouped=False, rows_grouped=True)
    scores = np.empty(K, dtype=np.int64)
    _load().oracle_perm_scores(_p(B), ctypes.c_int64(I), ctypes.c_int64(J), N, M, _p(perms), K, _p(scores))
    return scores


def is_permutation(perms) -> np.ndarray:
    """Sec. 3.3: P is a permutation of the I row indices.  One flag per candidate row (plain definition:
    sorted, the row reads 0, 1, ..., I-1)."""
    perms = np.atleast_2d(np.asarray(perms))
    I = perms.shape[1]
    return (np.sort(perms, axis=1) == np.arange(I)[None, :]).all(axis=1).astype(np.int32)


def perm_refine(B, P, swaps, N: int, M: int):
    """Limitations (future work): hill climbing on Sec. 3.3's objective by proposed exchanges of two
    positions of P, each kept iff the eligible-block count grows.  Returns (P', score before,
    score after, proposals kept)."""
    B = _u8(B)
    I, J = B.shape
    _check_nm(I, J, N, M, cols_grouped=False, rows_grouped=True)
    P = np.arange(I, dtype=np.int32) if P is None else np.array(P, dtype=np.int32, copy=True)
    assert P.shape == (I,)
    swaps = np.ascontiguousarray(np.asarray(swaps, dtype=np.int32).reshape(-1, 2))
    score = np.zeros(2, dtype=np.int64)
    acc = np.zeros(1, dtype=np.int64)
    _load().oracle_perm_refine(_p(B), ctypes.c_int64(I), ctypes.c_int64(J), N, M, _p(P), _p(swaps),
                               ctypes.c_int64(swaps.shape[0]), _p(score), _p(acc))
    return P, int(score[0]), int(score[1]), int(acc[0])


def argmax_first(scores) -> int:
    """Alg. 1: best candidate, first among equals."""
    scores = _i64(scores)
    return int(_load().oracle_argmax(_p(scores), int(scores.shape[0])))


def backward_mask(W, B, P, N: int, M: int) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. (11) (Eq. (9) for P=None).  Returns (Bbar, sel) in permuted row
    coordinates; `sel` is the selection before AND-ing with the forward mask."""
    W, B, P = _f64(W), _u8(B), _i32(P)
    I, J = W.shape
    _check_nm(I, J, N, M, cols_grouped=False, rows_grouped=True)
    Bbar = np.empty((I, J), dtype=np.uint8)
    sel = np.empty((I, J), dtype=np.uint8)
    _load().oracle_backward_mask(_p(W), _p(B), ctypes.c_int64(I), ctypes.c_int64(J), N, M,
                                 _p(P), _p(Bbar), _p(sel))
    return Bbar, sel


# ---------------------------------------------------------------- compression
def compress_fwd(W, B, N: int, M: int) -> Tuple[np.ndarray, np.ndarray]:
    """Kept values and their in-group positions, I x (J/M*N) each."""
    W, B = _f64(W), _u8(B)
    I, J = W.shape
    _check_nm(I, J, N, M)
    S = J // M * N
    val = np.empty((I, S), dtype=np.float64)
    idx = np.empty((I, S), dtype=np.uint8)
    _load().oracle_compress_fwd(_p(W), _p(B), ctypes.c_int64(I), ctypes.c_int64(J), N, M, _p(val), _p(idx))
    return val, idx


def compress_bwd(W, B, P, N: int, M: int) -> Tuple[np.ndarray, np.ndarray]:
    """Transposed compressed backward operand, J x (I/M*N) each."""
    W, B, P = _f64(W), _u8(B), _i32(P)
    I, J = W.shape
    _check_nm(I, J, N, M, cols_grouped=False, rows_grouped=True)
    S = I // M * N
    val = np.empty((J, S), dtype=np.float64)
    idx = np.empty((J, S), dtype=np.uint8)
    _load().oracle_compress_bwd(_p(W), _p(B), _p(P), ctypes.c_int64(I), ctypes.c_int64(J), N, M,
                                _p(val), _p(idx))
    return val, idx


def pack_bits(bits) -> np.ndarray:
    """0/1 bytes -> uint32 words, entry j = bit j%32 of word j//32."""
    bits = _u8(bits)
    R, C = bits.shape
    words = np.empty((R, (C + 31) // 32), dtype=np.uint32)
    _load().oracle_pack_bits(_p(bits), ctypes.c_int64(R), ctypes.c_int64(C), _p(words))
    return words


def pack_index(idx, M: int) -> np.ndarray:
    """Position indices -> log2(M)-bit fields, little-endian in uint32 words."""
    idx = _u8(idx)
    R, S = idx.shape
    b = (M - 1).bit_length()
    words = np.empty((R, (S * b + 31) // 32), dtype=np.uint32)
    _load().oracle_pack_index(_p(idx), ctypes.c_int64(R), ctypes.c_int64(S), M, _p(words))
    return words


# ---------------------------------------------------------------- GEMMs
def gemm_fwd_loops(X, W, B) -> np.ndarray:
    """Eq. (3), triple loop.  Small sizes only."""
    X, W, B = _f64(X), _f64(W), _u8(B)
    T, J = X.shape
    I = W.shape[0]
    Y = np.empty((T, I), dtype=np.float64)
    _load().oracle_gemm_fwd(_p(X), _p(W), _p(B), ctypes.c_int64(T), ctypes.c_int64(I), ctypes.c_int64(J), _p(Y))
    return Y


def gemm_bwd_loops(dY, W, Bbar, P) -> np.ndarray:
    """Eq. (10), triple loop.  Small sizes only."""
    dY, W, Bbar, P = _f64(dY), _f64(W), _u8(Bbar), _i32(P)
    T, I = dY.shape
    J = W.shape[1]
    dX = np.empty((T, J), dtype=np.float64)
    _load().oracle_gemm_bwd(_p(dY), _p(W), _p(Bbar), _p(P), ctypes.c_int64(T), ctypes.c_int64(I),
                            ctypes.c_int64(J), _p(dX))
    return dX


def gemm_fwd_at(X, W, B, ts, is_) -> np.ndarray:
    """Eq. (3) at listed (t, i) output coordinates."""
    X, W, B, ts, is_ = _f64(X), _f64(W), _u8(B), _i64(ts), _i64(is_)
    I, J = W.shape
    out = np.empty(ts.shape[0], dtype=np.float64)
    _load().oracle_gemm_fwd_at(_p(X), _p(W), _p(B), ctypes.c_int64(I), ctypes.c_int64(J),
                               _p(ts), _p(is_), ctypes.c_int64(ts.shape[0]), _p(out))
    return out


def gemm_bwd_at(dY, W, Bbar, P, ts, js) -> np.ndarray:
    """Eq. (10) at listed (t, j) output coordinates."""
    dY, W, Bbar, P, ts, js = _f64(dY), _f64(W), _u8(Bbar), _i32(P), _i64(ts), _i64(js)
    I, J = W.shape
    out = np.empty(ts.shape[0], dtype=np.float64)
    _load().oracle_gemm_bwd_at(_p(dY), _p(W), _p(Bbar), _p(P), ctypes.c_int64(I), ctypes.c_int64(J),
                               _p(ts), _p(js), ctypes.c_int64(ts.shape[0]), _p(out))
    return out


def gemm_fwd(X, W, B) -> np.ndarray:
    """Eq. (3) as a float64 library matmul on the dense masked weights."""
    return _f64(X) @ (_f64(W) * _u8(B)).T


def gemm_bwd(dY, W, Bbar, P) -> np.ndarray:
    """Eq. (10) as a float64 library matmul: dY[:,P] @ (Bbar .* W[P,:])."""
    dY, W, Bbar = _f64(dY), _f64(W), _u8(Bbar)
    if P is None:
        return dY @ (W * Bbar)
    P = np.asarray(P, dtype=np.int64)
    return dY[:, P] @ (W[P, :] * Bbar)


# ---------------------------------------------------------------- gradient gap (Eq. 5 vs Eq. 10)
def grad_exact_loops(dY, W, B) -> np.ndarray:
    """Eq. (5): g(X) = g(Y) (B .* W), triple loop.  Small sizes only."""
    dY, W, B = _f64(dY), _f64(W), _u8(B)
    T, I = dY.shape
    J = W.shape[1]
    gX = np.empty((T, J), dtype=np.float64)
    _load().oracle_grad_exact(_p(dY), _p(W), _p(B), ctypes.c_int64(T), ctypes.c_int64(I), ctypes.c_int64(J), _p(gX))
    return gX


def grad_exact(dY, W, B) -> np.ndarray:
    """Eq. (5) as a float64 library matmul on the dense forward-masked weights."""
    return _f64(dY) @ (_f64(W) * _u8(B))


def relative_gap(approx, exact) -> float:
    """||approx - exact||_F / ||exact||_F for two T x J gradients (Sec. 3.3's gradient gap)."""
    approx, exact = _f64(approx), _f64(exact)
    assert approx.shape == exact.shape
    return float(_load().oracle_relative_gap(_p(approx), _p(exact), ctypes.c_int64(approx.size)))


def gradient_gap(dY, W, B, P, N: int, M: int) -> float:
    """Gap between Eq. (10)'s g-bar(X), with the backward mask of Eq. (11) for permutation P (None =
    identity: Eq. (8) with Eq. (9)), and Eq. (5)'s g(X)."""
    Bbar, _ = backward_mask(W, B, P, N, M)
    return relative_gap(gemm_bwd(dY, W, Bbar, P), grad_exact(dY, W, B))


# ---------------------------------------------------------------- whole step
def bimask_step(W, X, dY, perms, N: int, M: int):
    """One Bi-Mask step of Alg. 1 for one layer (search included)."""
    B = forward_mask(W, N, M)
    Y = gemm_fwd(X, W, B)
    scores = perm_scores(B, perms, N, M)
    best = argmax_first(scores)
    P = np.asarray(perms)[best]
    Bbar, sel = backward_mask(W, B, P, N, M)
    dX = gemm_bwd(dY, W, Bbar, P)
    return dict(B=B, Y=Y, scores=scores, best=best, P=P, Bbar=Bbar, sel=sel, dX=dX)
