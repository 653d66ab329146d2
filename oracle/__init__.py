"""CPU oracle: SpMM / SDDMM by definition (C, fp64) and the reference format converter (numpy).

TEST INFRASTRUCTURE ONLY.  Imported by ``tests/``, by the smoke check and by
the ``cpu_baseline`` leg of the benchmark; never by the product package.  It
shares no code with the HIP library and does not import it.

Pins (what ties each function to something other than itself) live in
``tests/test_oracle_*.py``:
  * ``spmm`` / ``sddmm``: dense brute force in numpy fp64, scipy's CSR product,
    identity and all-ones special cases, algebraic invariants, a hand-worked
    golden example.
  * ``convert_ref``: a hand-worked golden example, a per-element brute force
    over a dense occupancy mask, round trip back to CSR, closed-form counts for
    the stencil, structural invariants.
  * ``edge_softmax_backward``: a hand-worked golden example, the definition as
    plain loops, central differences of the (separately pinned) forward softmax
    on rows with dyadic probabilities, the closed form of two-entry rows, and
    the invariants of a softmax Jacobian (zero row sums, constants map to zero).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

from .convert_ref import FormatRef, convert_ref, issued_mac_ratio, pack_ref, padded_format_bytes  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fs_oracle.c")
_SO = os.path.join(_HERE, "libfs_oracle.so")
_DT = {"f16": 0, "bf16": 1}
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP).  Returns the path of the shared object."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, p = ctypes.c_int64, ctypes.c_void_p
        lib.oracle_spmm.restype = ctypes.c_int
        lib.oracle_spmm.argtypes = [i64, i64, i64, p, p, p, p, i64, ctypes.c_int, p, i64, p, p]
        lib.oracle_sddmm.restype = ctypes.c_int
        lib.oracle_sddmm.argtypes = [i64, i64, i64, p, p, p, i64, p, i64, ctypes.c_int, p, i64, p, p]
        lib.oracle_edge_softmax.restype = ctypes.c_int
        lib.oracle_edge_softmax.argtypes = [i64, p, p, ctypes.c_int, ctypes.c_double, p, i64, p]
        lib.oracle_attention.restype = ctypes.c_int
        lib.oracle_attention.argtypes = [i64, i64, p, p, p, i64, p, i64, i64, ctypes.c_int, ctypes.c_double,
                                         p, i64, i64, p, i64, p, p]
        lib.oracle_csr_transpose.restype = ctypes.c_int
        lib.oracle_csr_transpose.argtypes = [i64, i64, p, p, p, p, p]
        lib.oracle_threads.restype = ctypes.c_int
        lib.oracle_widen.restype = ctypes.c_double
        lib.oracle_widen.argtypes = [ctypes.c_uint16, ctypes.c_int]
        _lib = lib
    return _lib


def threads() -> int:
    """Number of OpenMP threads the oracle will use."""
    return int(_load().oracle_threads())


def widen(bits: int, dtype: str) -> float:
    return float(_load().oracle_widen(int(bits), _DT[dtype]))


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check_csr(rowptr, colidx, M):
    assert rowptr.dtype == np.int32 and colidx.dtype == np.int32
    assert rowptr.shape == (M + 1,) and rowptr.flags.c_contiguous and colidx.flags.c_contiguous


def spmm(M: int, K: int, rowptr: np.ndarray, colidx: np.ndarray, vals_bits: np.ndarray,
         B_bits: np.ndarray, dtype: str, rows: Optional[np.ndarray] = None,
         want_scale: bool = True) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """C = A @ B in fp64 (paper Section 2.2).  Returns (C, S) with S = sum |a||b|.

    ``rows`` (int64 array) restricts the computation to those rows of A.
    """
    _check_csr(rowptr, colidx, M)
    assert vals_bits.dtype == np.uint16 and B_bits.dtype == np.uint16 and B_bits.ndim == 2
    assert B_bits.shape[0] == K and B_bits.strides[1] == 2
    N = B_bits.shape[1]
    ldb = B_bits.strides[0] // 2
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
    n_rows = M if rows is None else rows.shape[0]
    C = np.empty((n_rows, N), dtype=np.float64)
    S = np.empty((n_rows, N), dtype=np.float64) if want_scale else None
    rc = _load().oracle_spmm(M, K, N, _ptr(rowptr), _ptr(colidx), _ptr(np.ascontiguousarray(vals_bits)),
                             _ptr(B_bits), ldb, _DT[dtype], _ptr(rows), n_rows, _ptr(C), _ptr(S))
    if rc:
        raise ValueError("oracle_spmm: index out of range")
    return C, S


def sddmm(M: int, K: int, rowptr: np.ndarray, colidx: np.ndarray, X_bits: np.ndarray,
          Y_bits: np.ndarray, dtype: str, rows: Optional[np.ndarray] = None,
          want_scale: bool = True) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """out[p] = <X[i,:], Y[col[p],:]> for each stored entry p of row i, fp64 (paper Section 3.4).

    Returns (out, S) indexed by CSR position.  With ``rows`` given, positions
    of other rows are left as NaN.
    """
    _check_csr(rowptr, colidx, M)
    assert X_bits.dtype == np.uint16 and Y_bits.dtype == np.uint16
    assert X_bits.shape[0] == M and Y_bits.shape[0] == K and X_bits.shape[1] == Y_bits.shape[1]
    assert X_bits.strides[1] == 2 and Y_bits.strides[1] == 2
    d = X_bits.shape[1]
    nnz = colidx.shape[0]
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
    n_rows = M if rows is None else rows.shape[0]
    out = np.full(nnz, np.nan, dtype=np.float64)
    S = np.full(nnz, np.nan, dtype=np.float64) if want_scale else None
    rc = _load().oracle_sddmm(M, K, d, _ptr(rowptr), _ptr(colidx), _ptr(X_bits), X_bits.strides[0] // 2,
                              _ptr(Y_bits), Y_bits.strides[0] // 2, _DT[dtype], _ptr(rows), n_rows,
                              _ptr(out), _ptr(S))
    if rc:
        raise ValueError("oracle_sddmm: index out of range")
    return out, S


def edge_softmax(M: int, rowptr: np.ndarray, vals_bits: np.ndarray, dtype: str, scale: float = 1.0,
                 rows: Optional[np.ndarray] = None) -> np.ndarray:
    """Softmax of scale * value over the stored entries of each row, fp64 (the softmax layer of the
    attention GNN in the paper's Section 4.4).  Indexed by CSR position; with ``rows`` given,
    positions of other rows are left as NaN."""
    assert rowptr.dtype == np.int32 and rowptr.shape == (M + 1,) and vals_bits.dtype == np.uint16
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
    n_rows = M if rows is None else rows.shape[0]
    out = np.full(vals_bits.shape[0], np.nan, dtype=np.float64)
    rc = _load().oracle_edge_softmax(M, _ptr(np.ascontiguousarray(rowptr)), _ptr(np.ascontiguousarray(vals_bits)),
                                     _DT[dtype], float(scale), _ptr(rows), n_rows, _ptr(out))
    if rc:
        raise ValueError("oracle_edge_softmax: row out of range")
    return out


def edge_softmax_backward(M: int, rowptr: np.ndarray, p_bits: np.ndarray, g_bits: np.ndarray, dtype: str,
                          scale: float = 1.0) -> Tuple[np.ndarray, np.ndarray]:
    """Gradient of the row softmax with respect to its input scores, fp64, by its definition: with
    p = softmax_row(scale * s) and g the gradient that arrives at p (both indexed by CSR position),

        ds[q] = scale * p[q] * (g[q] - sum over the row of p[r] * g[r]).

    What the training pass of the attention GNN of the paper's Section 4.4 needs between the two sparse
    products of its backward pass.  p and g are 16-bit values (widened exactly); the sum runs over the stored
    entries of the row of q, in CSR order.  Returns (ds, S) with S = |scale| |p[q]| (|g[q]| + sum |p[r] g[r]|),
    the magnitude errors are measured against."""
    assert rowptr.dtype == np.int32 and rowptr.shape == (M + 1,)
    assert p_bits.dtype == np.uint16 and g_bits.dtype == np.uint16 and p_bits.shape == g_bits.shape == (int(rowptr[M]),)
    p, g = _widen_all(p_bits, dtype), _widen_all(g_bits, dtype)
    row = np.repeat(np.arange(M), np.diff(rowptr))               # the row of every stored entry
    dot = np.bincount(row, weights=p * g, minlength=M)           # sum over each row of p * g, in CSR order
    mag = np.bincount(row, weights=np.abs(p * g), minlength=M)
    ds = scale * p * (g - dot[row])
    S = abs(scale) * np.abs(p) * (np.abs(g) + mag[row])
    return ds, S


def _widen_all(bits: np.ndarray, dtype: str) -> np.ndarray:
    """Every 16-bit pattern of an array widened exactly to fp64 (numpy's own conversions: fp16 -> fp64, and
    bf16 as the upper half of an fp32)."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    with np.errstate(invalid="ignore"):  # signalling NaN patterns stay NaN
        if dtype == "f16":
            return bits.view(np.float16).astype(np.float64)
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def attention(M: int, K: int, rowptr: np.ndarray, colidx: np.ndarray, X_bits: np.ndarray, Y_bits: np.ndarray,
              H_bits: np.ndarray, dtype: str, scale: float = 1.0,
              rows: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Sparse attention softmax_row(scale * (X Y^T) at A's pattern) * H in fp64, nothing rounded in between
    (the SDDMM -> softmax -> SpMM chain of the paper's Section 4.4 attention GNN as one definition).
    Returns (out, S) with S = sum a |h| the matching magnitude; rows of A without entries give zeros."""
    _check_csr(rowptr, colidx, M)
    for a in (X_bits, Y_bits, H_bits):
        assert a.dtype == np.uint16 and a.ndim == 2 and a.flags.c_contiguous
    d, N = X_bits.shape[1], H_bits.shape[1]
    assert X_bits.shape[0] == M and Y_bits.shape == (K, d) and H_bits.shape[0] == K
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
    n_rows = M if rows is None else rows.shape[0]
    out = np.empty((n_rows, N), dtype=np.float64)
    S = np.empty((n_rows, N), dtype=np.float64)
    rc = _load().oracle_attention(M, K, _ptr(rowptr), _ptr(colidx), _ptr(X_bits), d, _ptr(Y_bits), d, d, _DT[dtype],
                                  float(scale), _ptr(H_bits), N, N, _ptr(rows), n_rows, _ptr(out), _ptr(S))
    if rc:
        raise ValueError("oracle_attention: index out of range")
    return out, S


def csr_transpose(M: int, K: int, rowptr: np.ndarray, colidx: np.ndarray):
    """CSR of the transposed matrix and the permutation of the stored entries: returns
    (rowptr_t[K+1], colidx_t[nnz], perm[nnz]) with perm[q] = position in A's CSR order of entry q of
    A^T's CSR order (for the A^T * dC of a backward pass, Section 4.4)."""
    _check_csr(rowptr, colidx, M)
    nnz = colidx.shape[0]
    rowptr_t = np.empty(K + 1, dtype=np.int32)
    colidx_t = np.empty(nnz, dtype=np.int32)
    perm = np.empty(nnz, dtype=np.int32)
    rc = _load().oracle_csr_transpose(M, K, _ptr(rowptr), _ptr(colidx), _ptr(rowptr_t), _ptr(colidx_t), _ptr(perm))
    if rc:
        raise ValueError("oracle_csr_transpose: column out of range")
    return rowptr_t, colidx_t, perm


def round_f64_to_bits(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp64 values to the 16-bit storage type, nearest-even, in one step (for the SDDMM->SpMM chain)."""
    x = np.asarray(x, dtype=np.float64)
    if dtype == "f16":
        return x.astype(np.float16).view(np.uint16)
    # bf16: round the double directly to 8 significant bits.  Going through
    # float32 first could round twice, so do it on the exact value instead.
    m, e = np.frexp(x)  # x = m * 2**e, 0.5 <= |m| < 1
    q = np.rint(m * 256.0) / 256.0  # 8 significant bits, ties to even
    y = np.ldexp(q, e).astype(np.float32)  # exactly representable (normal range)
    return (y.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
