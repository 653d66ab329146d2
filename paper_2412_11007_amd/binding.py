"""ctypes binding of the C ABI in ``include/flashsparse.h``.

Same names as the C entry points.  Argument marshalling only: every step of the
computation runs in the HIP library; torch supplies device memory and the
current stream.  There is no fallback: if the shared library is missing the
first call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
# FLASHSPARSE_LIB points at an alternative build of the same library (e.g. one compiled with other -D flags)
_LIB_PATH = os.environ.get("FLASHSPARSE_LIB") or os.path.join(_HERE, "libflashsparse_hip.so")
_lib = None

FS_F16, FS_BF16 = 0, 1


class FsError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = int(code)
        super().__init__("%s failed: %s (status %d)" % (where, fs_status_string(code), code))


class _FsFormatStruct(ctypes.Structure):
    _fields_ = [
        ("M", ctypes.c_int64), ("K", ctypes.c_int64), ("nnz", ctypes.c_int64), ("nvec", ctypes.c_int64),
        ("W", ctypes.c_int64),
        ("V", ctypes.c_int32), ("KB", ctypes.c_int32), ("dtype", ctypes.c_int32), ("chunk", ctypes.c_int32),
        ("n_items", ctypes.c_int64), ("n_split_items", ctypes.c_int64), ("n_split_windows", ctypes.c_int64),
        ("win_ptr", ctypes.c_void_p), ("vec_col", ctypes.c_void_p), ("vec_mask", ctypes.c_void_p),
        ("csr_to_slot", ctypes.c_void_p), ("vals_blk", ctypes.c_void_p), ("blk_desc", ctypes.c_void_p),
        ("n_blocks", ctypes.c_int64), ("items", ctypes.c_void_p),
        ("split_windows", ctypes.c_void_p),
        ("n_cut_items", ctypes.c_int64),
        ("item_order", ctypes.c_void_p),
        ("items_by_cost", ctypes.c_void_p),
        ("blk_row_base", ctypes.c_void_p),
        ("packed", ctypes.c_void_p),
        ("slot_range", ctypes.c_void_p),
        ("arena_used", ctypes.c_size_t),
    ]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load the HIP library; raises (never falls back) when it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    import torch  # noqa: F401  (first, so that this library binds to the HIP runtime torch has loaded)
    if not os.path.exists(_LIB_PATH):
        raise ImportError("%s is missing: build it with `python -m paper_2412_11007_amd.build`" % _LIB_PATH)
    lib = ctypes.CDLL(_LIB_PATH)
    i32, i64, vp, sz = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t
    fmtp = ctypes.POINTER(_FsFormatStruct)
    szp = ctypes.POINTER(ctypes.c_size_t)
    lib.fs_version.restype = ctypes.c_int
    lib.fs_version.argtypes = []
    lib.fs_status_string.restype = ctypes.c_char_p
    lib.fs_status_string.argtypes = [ctypes.c_int]
    lib.fs_format_bytes.restype = ctypes.c_int
    lib.fs_format_bytes.argtypes = [i64, i64, i32, i32, ctypes.c_int, szp, szp]
    lib.fs_convert.restype = ctypes.c_int
    lib.fs_convert.argtypes = [i64, i64, i64, vp, vp, vp, ctypes.c_int, i32, i32, i32, vp, sz, vp, sz, vp, fmtp]
    lib.fs_spmm_workspace_bytes.restype = ctypes.c_int
    lib.fs_spmm_workspace_bytes.argtypes = [fmtp, i64, szp]
    lib.fs_spmm.restype = ctypes.c_int
    lib.fs_spmm.argtypes = [fmtp, vp, vp, i64, i64, vp, i64, vp, sz, vp]
    lib.fs_spmm_static.restype = ctypes.c_int
    lib.fs_spmm_static.argtypes = [fmtp, vp, vp, i64, i64, vp, i64, vp]
    lib.fs_spmm_timed.restype = ctypes.c_int
    lib.fs_spmm_timed.argtypes = [fmtp, vp, vp, i64, i64, vp, i64, vp, sz, vp, vp, vp]
    lib.fs_sddmm.restype = ctypes.c_int
    lib.fs_sddmm.argtypes = [fmtp, vp, i64, vp, i64, i64, vp, vp, vp]
    lib.fs_edge_softmax_workspace_bytes.restype = ctypes.c_int
    lib.fs_edge_softmax_workspace_bytes.argtypes = [fmtp, szp]
    lib.fs_pack_bytes.restype = ctypes.c_int
    lib.fs_pack_bytes.argtypes = [fmtp, szp]
    lib.fs_pack_values.restype = ctypes.c_int
    lib.fs_pack_values.argtypes = [fmtp, vp, vp, sz, vp]
    lib.fs_spmm_packed.restype = ctypes.c_int
    lib.fs_spmm_packed.argtypes = [fmtp, vp, vp, i64, i64, vp, i64, vp, sz, vp]
    lib.fs_attention_workspace_bytes.restype = ctypes.c_int
    lib.fs_attention_workspace_bytes.argtypes = [fmtp, i64, szp]
    lib.fs_attention.restype = ctypes.c_int
    lib.fs_attention.argtypes = [fmtp, vp, i64, vp, i64, i64, ctypes.c_float, vp, i64, i64, vp, i64, vp, sz, vp]
    lib.fs_sddmm_spmm.restype = ctypes.c_int
    lib.fs_sddmm_spmm.argtypes = lib.fs_attention.argtypes
    lib.fs_edge_softmax.restype = ctypes.c_int
    lib.fs_edge_softmax.argtypes = [fmtp, vp, vp, ctypes.c_float, vp, sz, vp]
    lib.fs_edge_softmax_backward.restype = ctypes.c_int
    lib.fs_edge_softmax_backward.argtypes = [fmtp, vp, vp, ctypes.c_float, vp, vp, sz, vp]
    lib.fs_blk_to_csr.restype = ctypes.c_int
    lib.fs_blk_to_csr.argtypes = [fmtp, vp, vp, vp]
    lib.fs_csr_to_blk.restype = ctypes.c_int
    lib.fs_csr_to_blk.argtypes = [fmtp, vp, vp, vp]
    lib.fs_csr_transpose_bytes.restype = ctypes.c_int
    lib.fs_csr_transpose_bytes.argtypes = [i64, i64, i64, ctypes.POINTER(sz)]
    lib.fs_csr_transpose.restype = ctypes.c_int
    lib.fs_csr_transpose.argtypes = [i64, i64, i64, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.fs_gather16.restype = ctypes.c_int
    lib.fs_gather16.argtypes = [vp, vp, i64, vp, vp]
    lib.fs_gather_probe.restype = ctypes.c_int
    lib.fs_gather_probe.argtypes = [fmtp, vp, i64, i64, vp, sz, vp]
    lib.fs_read_bytes.restype = ctypes.c_int
    lib.fs_read_bytes.argtypes = [vp, sz, i32, vp, sz, vp]
    lib.fs_copy_bytes.restype = ctypes.c_int
    lib.fs_copy_bytes.argtypes = [vp, vp, sz, vp]
    _lib = lib
    return lib


def fs_version() -> int:
    return int(load_library().fs_version())


def fs_status_string(code: int) -> str:
    return load_library().fs_status_string(int(code)).decode()


def _dtype_code(torch_dtype) -> int:
    import torch
    if torch_dtype == torch.float16:
        return FS_F16
    if torch_dtype == torch.bfloat16:
        return FS_BF16
    raise TypeError("element type must be torch.float16 or torch.bfloat16")


def _stream_ptr(stream) -> int:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def fs_format_bytes(M: int, nnz: int, V: int = 0, KB: int = 0, dtype: int = FS_F16) -> Tuple[int, int]:
    a, s = ctypes.c_size_t(0), ctypes.c_size_t(0)
    rc = load_library().fs_format_bytes(M, nnz, V, KB, dtype, ctypes.byref(a), ctypes.byref(s))
    if rc:
        raise FsError(rc, "fs_format_bytes")
    return int(a.value), int(s.value)


class FsFormat:
    """Host descriptor + the device arena it points into (kept alive together)."""

    def __init__(self, struct: _FsFormatStruct, arena, torch_dtype):
        self.c = struct
        self.arena = arena
        self.torch_dtype = torch_dtype

    def __getattr__(self, name):
        return getattr(self.c, name)

    def _view(self, ptr: int, nbytes: int, torch_dtype):
        ofs = ptr - self.arena.data_ptr()
        return self.arena[ofs:ofs + nbytes].view(torch_dtype)

    # views of the converted arrays (device tensors sharing the arena's memory)
    def win_ptr_t(self):
        import torch
        return self._view(self.c.win_ptr, 4 * (self.c.W + 1), torch.int32)

    def vec_col_t(self):
        import torch
        return self._view(self.c.vec_col, 4 * self.c.nvec, torch.int32)

    def vec_mask_t(self):
        import torch
        return self._view(self.c.vec_mask, 4 * self.c.nvec, torch.int32)

    def csr_to_slot_t(self):
        import torch
        return self._view(self.c.csr_to_slot, 4 * self.c.nnz, torch.int32)

    def vals_blk_t(self):
        return self._view(self.c.vals_blk, 2 * self.c.V * self.c.nvec, self.torch_dtype)

    def blk_desc_t(self):
        import torch
        return self._view(self.c.blk_desc, 16 * self.c.n_blocks, torch.int32).view(-1, 4)

    def items_t(self):
        import torch
        return self._view(self.c.items, 16 * self.c.n_items, torch.int32).view(-1, 4)

    def item_order_t(self):
        import torch
        return self._view(self.c.item_order, 4 * self.c.n_items, torch.int32)

    def items_by_cost_t(self):
        import torch
        return self._view(self.c.items_by_cost, 16 * self.c.n_items, torch.int32).view(-1, 4)

    def blk_row_base_t(self):
        import torch
        return self._view(self.c.blk_row_base, 4 * self.c.V * self.c.n_blocks, torch.int32).view(-1, self.c.V)

    def split_windows_t(self):
        import torch
        return self._view(self.c.split_windows, 16 * self.c.n_split_windows, torch.int32).view(-1, 4)

    def slot_range_t(self):
        import torch
        return self._view(self.c.slot_range, 8 * self.c.n_split_items, torch.int32).view(-1, 2)


def fs_convert(rowptr, colidx, vals, M: int, K: int, torch_dtype=None, V: int = 0, KB: int = 0, chunk: int = 0,
               stream=None, arena=None, scratch=None) -> FsFormat:
    """CSR (int32 device tensors) -> window format.  ``vals`` may be None (pattern only)."""
    import torch
    lib = load_library()
    nnz = int(colidx.numel())
    if vals is not None:
        torch_dtype = vals.dtype
    if torch_dtype is None:
        torch_dtype = torch.float16
    code = _dtype_code(torch_dtype)
    assert rowptr.dtype == torch.int32 and colidx.dtype == torch.int32 and rowptr.is_cuda and colidx.is_cuda
    assert rowptr.is_contiguous() and colidx.is_contiguous() and rowptr.numel() == M + 1
    assert vals is None or (vals.is_cuda and vals.is_contiguous() and vals.numel() == nnz)
    a_bytes, s_bytes = fs_format_bytes(M, nnz, V, KB, code)
    dev = rowptr.device
    if arena is None:
        arena = torch.empty(a_bytes, dtype=torch.uint8, device=dev)
    if scratch is None:
        scratch = torch.empty(s_bytes, dtype=torch.uint8, device=dev)
    st = _FsFormatStruct()
    rc = lib.fs_convert(M, K, nnz, rowptr.data_ptr(), colidx.data_ptr(), 0 if vals is None else vals.data_ptr(),
                        code, V, KB, chunk, arena.data_ptr(), arena.numel(), scratch.data_ptr(), scratch.numel(),
                        _stream_ptr(stream), ctypes.byref(st))
    if rc:
        raise FsError(rc, "fs_convert")
    return FsFormat(st, arena, torch_dtype)


def fs_spmm_workspace_bytes(fmt: FsFormat, N: int) -> int:
    w = ctypes.c_size_t(0)
    rc = load_library().fs_spmm_workspace_bytes(ctypes.byref(fmt.c), N, ctypes.byref(w))
    if rc:
        raise FsError(rc, "fs_spmm_workspace_bytes")
    return int(w.value)


def fs_spmm(fmt: FsFormat, B, vals=None, out=None, work=None, stream=None, events=None):
    """C = A @ B.  ``vals`` (vals_blk layout) overrides the format's own values.

    ``events`` = (before, after) raw hipEvent_t handles switches to fs_spmm_timed,
    which records them around the main kernel.
    """
    import torch
    K, N = B.shape
    assert B.is_cuda and B.dtype == fmt.torch_dtype and B.stride(1) == 1 and K == fmt.c.K
    if out is None:
        out = torch.empty((fmt.c.M, N), dtype=B.dtype, device=B.device)
    assert out.shape == (fmt.c.M, N) and out.stride(1) == 1 and out.dtype == B.dtype
    need = fs_spmm_workspace_bytes(fmt, N)
    if work is None and need:
        work = torch.empty(need, dtype=torch.uint8, device=B.device)
    args = (ctypes.byref(fmt.c), 0 if vals is None else vals.data_ptr(), B.data_ptr(), N,
            B.stride(0), out.data_ptr(), out.stride(0),
            0 if work is None else work.data_ptr(), 0 if work is None else work.numel(), _stream_ptr(stream))
    if events is None:
        rc = load_library().fs_spmm(*args)
    else:
        rc = load_library().fs_spmm_timed(*args, events[0], events[1])
    if rc:
        raise FsError(rc, "fs_spmm")
    return out


def bind_spmm(fmt: FsFormat, B, out, work=None, vals=None, stream=None):
    """fs_spmm with its arguments checked and marshalled once: returns a callable that only makes the C call
    (for loops that repeat one call and cannot afford the per-call checks of ``fs_spmm``).  The tensors must
    stay alive and unchanged in place; the stream is the one current now unless given."""
    import torch
    K, N = B.shape
    assert B.is_cuda and B.dtype == fmt.torch_dtype and B.stride(1) == 1 and K == fmt.c.K
    assert out.shape == (fmt.c.M, N) and out.stride(1) == 1 and out.dtype == B.dtype
    need = fs_spmm_workspace_bytes(fmt, N)
    if work is None and need:
        work = torch.empty(need, dtype=torch.uint8, device=B.device)
    fn = load_library().fs_spmm
    args = (ctypes.byref(fmt.c), 0 if vals is None else vals.data_ptr(), B.data_ptr(), N, B.stride(0), out.data_ptr(),
            out.stride(0), 0 if work is None else work.data_ptr(), 0 if work is None else work.numel(), _stream_ptr(stream))
    keep = (fmt, B, out, work, vals)

    def call():
        rc = fn(*args)
        if rc:
            raise FsError(rc, "fs_spmm")
        return keep[2]
    return call


def bind_sddmm(fmt: FsFormat, X, Y, out=None, out_csr=None, stream=None):
    """fs_sddmm marshalled once (see bind_spmm); at least one of ``out`` (blocked layout) and ``out_csr``."""
    assert X.is_cuda and Y.is_cuda and X.dtype == fmt.torch_dtype and Y.dtype == fmt.torch_dtype
    assert X.shape[0] == fmt.c.M and Y.shape[0] == fmt.c.K and X.shape[1] == Y.shape[1]
    assert X.stride(1) == 1 and Y.stride(1) == 1 and (out is not None or out_csr is not None)
    assert out is None or (out.numel() == fmt.c.V * fmt.c.nvec and out.is_contiguous() and out.dtype == X.dtype)
    assert out_csr is None or (out_csr.numel() == fmt.c.nnz and out_csr.is_contiguous() and out_csr.dtype == X.dtype)
    fn = load_library().fs_sddmm
    args = (ctypes.byref(fmt.c), X.data_ptr(), X.stride(0), Y.data_ptr(), Y.stride(0), X.shape[1],
            0 if out is None else out.data_ptr(), 0 if out_csr is None else out_csr.data_ptr(), _stream_ptr(stream))
    keep = (fmt, X, Y, out, out_csr)

    def call():
        rc = fn(*args)
        if rc:
            raise FsError(rc, "fs_sddmm")
        return keep[3] if keep[3] is not None else keep[4]
    return call


def fs_spmm_static(fmt: FsFormat, B, out, vals=None, stream=None):
    """C = A @ B into ``out`` with the library's own fixed workspace: the call itself allocates nothing."""
    K, N = B.shape
    assert B.is_cuda and B.dtype == fmt.torch_dtype and B.stride(1) == 1 and K == fmt.c.K
    assert out.shape == (fmt.c.M, N) and out.stride(1) == 1 and out.dtype == B.dtype
    rc = load_library().fs_spmm_static(ctypes.byref(fmt.c), 0 if vals is None else vals.data_ptr(), B.data_ptr(), N,
                                       B.stride(0), out.data_ptr(), out.stride(0), _stream_ptr(stream))
    if rc:
        raise FsError(rc, "fs_spmm_static")
    return out


def fs_sddmm(fmt: FsFormat, X, Y, out=None, stream=None, out_csr=None, blocked=True):
    """Scores (X @ Y^T) at the stored positions of A.  Returns them in the vals_blk layout (V*nvec elements);
    ``out_csr`` (nnz elements) additionally receives them in CSR order from the same kernel.  With
    ``blocked=False`` only ``out_csr`` is written (allocated if not given) and returned."""
    import torch
    assert X.is_cuda and Y.is_cuda and X.dtype == fmt.torch_dtype and Y.dtype == fmt.torch_dtype
    assert X.shape[0] == fmt.c.M and Y.shape[0] == fmt.c.K and X.shape[1] == Y.shape[1]
    assert X.stride(1) == 1 and Y.stride(1) == 1
    if blocked:
        if out is None:
            out = torch.empty(fmt.c.V * fmt.c.nvec, dtype=X.dtype, device=X.device)
        assert out.numel() == fmt.c.V * fmt.c.nvec and out.is_contiguous()
    else:
        out = None
        if out_csr is None:
            out_csr = torch.empty(fmt.c.nnz, dtype=X.dtype, device=X.device)
    if out_csr is not None:
        assert out_csr.numel() == fmt.c.nnz and out_csr.is_contiguous() and out_csr.dtype == X.dtype
    rc = load_library().fs_sddmm(ctypes.byref(fmt.c), X.data_ptr(), X.stride(0), Y.data_ptr(), Y.stride(0),
                                 X.shape[1], 0 if out is None else out.data_ptr(),
                                 0 if out_csr is None else out_csr.data_ptr(), _stream_ptr(stream))
    if rc:
        raise FsError(rc, "fs_sddmm")
    return out if blocked else out_csr


def fs_edge_softmax_workspace_bytes(fmt: FsFormat) -> int:
    n = ctypes.c_size_t(0)
    rc = load_library().fs_edge_softmax_workspace_bytes(ctypes.byref(fmt.c), ctypes.byref(n))
    if rc:
        raise FsError(rc, "fs_edge_softmax_workspace_bytes")
    return int(n.value)


def fs_edge_softmax(fmt: FsFormat, vals, out=None, scale: float = 1.0, work=None, stream=None):
    """Row softmax of scale * value over the stored entries, on vals_blk-layout arrays (out may be vals)."""
    import torch
    assert vals.is_cuda and vals.dtype == fmt.torch_dtype and vals.is_contiguous()
    assert vals.numel() == fmt.c.V * fmt.c.nvec
    if out is None:
        out = torch.empty_like(vals)
    assert out.numel() == vals.numel() and out.dtype == vals.dtype and out.is_contiguous()
    need = fs_edge_softmax_workspace_bytes(fmt)
    if work is None and need > 0:
        work = torch.empty(need, dtype=torch.uint8, device=vals.device)
    rc = load_library().fs_edge_softmax(ctypes.byref(fmt.c), vals.data_ptr(), out.data_ptr(), float(scale),
                                        work.data_ptr() if work is not None else None,
                                        work.numel() * work.element_size() if work is not None else 0,
                                        _stream_ptr(stream))
    if rc:
        raise FsError(rc, "fs_edge_softmax")
    return out


def fs_edge_softmax_backward(fmt: FsFormat, probs, grad, out=None, scale: float = 1.0, work=None, stream=None):
    """Gradient of fs_edge_softmax: scale * p * (g - row sum of p * g), on vals_blk-layout arrays (out may be
    either input)."""
    import torch
    for t in (probs, grad):
        assert t.is_cuda and t.dtype == fmt.torch_dtype and t.is_contiguous() and t.numel() == fmt.c.V * fmt.c.nvec
    if out is None:
        out = torch.empty_like(probs)
    assert out.numel() == probs.numel() and out.dtype == probs.dtype and out.is_contiguous()
    need = fs_edge_softmax_workspace_bytes(fmt)
    if work is None and need > 0:
        work = torch.empty(need, dtype=torch.uint8, device=probs.device)
    rc = load_library().fs_edge_softmax_backward(ctypes.byref(fmt.c), probs.data_ptr(), grad.data_ptr(), float(scale),
                                                 out.data_ptr(), work.data_ptr() if work is not None else None,
                                                 work.numel() * work.element_size() if work is not None else 0,
                                                 _stream_ptr(stream))
    if rc:
        raise FsError(rc, "fs_edge_softmax_backward")
    return out


def fs_pack_values(fmt: FsFormat, vals=None, out=None, stream=None):
    """Bitmap-packed copy of a vals_blk-layout array (default: the format's own values) for fs_spmm_packed."""
    import torch
    lib = load_library()
    n = ctypes.c_size_t(0)
    rc = lib.fs_pack_bytes(ctypes.byref(fmt.c), ctypes.byref(n))
    if rc:
        raise FsError(rc, "fs_pack_bytes")
    if out is None:
        out = torch.empty(n.value, dtype=torch.uint8, device="cuda")
    if vals is not None:
        assert vals.is_cuda and vals.is_contiguous() and vals.numel() == fmt.c.V * fmt.c.nvec and vals.element_size() == 2
    rc = lib.fs_pack_values(ctypes.byref(fmt.c), vals.data_ptr() if vals is not None else None, out.data_ptr(),
                            out.numel(), _stream_ptr(stream))
    if rc:
        raise FsError(rc, "fs_pack_values")
    return out


def fs_spmm_packed(fmt: FsFormat, packed, B, out=None, work=None, stream=None):
    """C = A @ B with A's values taken from a buffer made by fs_pack_values."""
    import torch
    assert B.is_cuda and B.dtype == fmt.torch_dtype and B.dim() == 2 and B.stride(1) == 1 and B.shape[0] == fmt.c.K
    assert packed.is_cuda and packed.dtype == torch.uint8
    N = B.shape[1]
    if out is None:
        out = torch.empty((fmt.c.M, N), dtype=B.dtype, device=B.device)
    assert out.shape == (fmt.c.M, N) and out.dtype == B.dtype and out.stride(1) == 1
    need = fs_spmm_workspace_bytes(fmt, N)
    if work is None and need > 0:
        work = torch.empty(need, dtype=torch.uint8, device=B.device)
    rc = load_library().fs_spmm_packed(ctypes.byref(fmt.c), packed.data_ptr(), B.data_ptr(), N, B.stride(0),
                                       out.data_ptr(), out.stride(0),
                                       work.data_ptr() if work is not None else None,
                                       work.numel() * work.element_size() if work is not None else 0,
                                       _stream_ptr(stream))
    if rc:
        raise FsError(rc, "fs_spmm_packed")
    return out


def fs_attention_workspace_bytes(fmt: FsFormat, N: int) -> int:
    n = ctypes.c_size_t(0)
    rc = load_library().fs_attention_workspace_bytes(ctypes.byref(fmt.c), int(N), ctypes.byref(n))
    if rc:
        raise FsError(rc, "fs_attention_workspace_bytes")
    return int(n.value)


def fs_sddmm_spmm(fmt: FsFormat, X, Y, H, scale: float = 1.0, out=None, work=None, stream=None):
    """((scale * X @ Y.T) at A's stored positions, rounded to the element type) @ H in one kernel: fs_sddmm
    followed by fs_spmm without the score array."""
    return _attention_like("fs_sddmm_spmm", fmt, X, Y, H, scale, out, work, stream)


def fs_attention(fmt: FsFormat, X, Y, H, scale: float = 1.0, out=None, work=None, stream=None):
    """softmax_rows(scale * (X @ Y.T) at A's stored positions) @ H in one kernel (rows without entries: zeros)."""
    return _attention_like("fs_attention", fmt, X, Y, H, scale, out, work, stream)


def _attention_like(name, fmt, X, Y, H, scale, out, work, stream):
    import torch
    for t in (X, Y, H):
        assert t.is_cuda and t.dtype == fmt.torch_dtype and t.dim() == 2 and t.stride(1) == 1
    d, N = X.shape[1], H.shape[1]
    assert X.shape[0] == fmt.c.M and Y.shape == (fmt.c.K, d) and H.shape[0] == fmt.c.K
    if out is None:
        out = torch.empty((fmt.c.M, N), dtype=H.dtype, device=H.device)
    assert out.shape == (fmt.c.M, N) and out.dtype == H.dtype and out.stride(1) == 1
    need = fs_attention_workspace_bytes(fmt, N)
    if work is None and need > 0:
        work = torch.empty(need, dtype=torch.uint8, device=H.device)
    rc = getattr(load_library(), name)(ctypes.byref(fmt.c), X.data_ptr(), X.stride(0), Y.data_ptr(), Y.stride(0), d,
                                     float(scale), H.data_ptr(), N, H.stride(0), out.data_ptr(), out.stride(0),
                                     work.data_ptr() if work is not None else None,
                                     work.numel() * work.element_size() if work is not None else 0,
                                     _stream_ptr(stream))
    if rc:
        raise FsError(rc, name)
    return out


def fs_blk_to_csr(fmt: FsFormat, blk, out=None, stream=None):
    """Reorder a vals_blk-layout array into CSR order."""
    import torch
    if out is None:
        out = torch.empty(fmt.c.nnz, dtype=blk.dtype, device=blk.device)
    rc = load_library().fs_blk_to_csr(ctypes.byref(fmt.c), blk.data_ptr(), out.data_ptr(), _stream_ptr(stream))
    if rc:
        raise FsError(rc, "fs_blk_to_csr")
    return out


def fs_csr_to_blk(fmt: FsFormat, vals_csr, out=None, stream=None):
    """CSR-order values -> vals_blk layout (zeros elsewhere): new values for the same pattern."""
    import torch
    assert vals_csr.is_cuda and vals_csr.dtype == fmt.torch_dtype and vals_csr.is_contiguous()
    assert vals_csr.numel() == fmt.c.nnz
    if out is None:
        out = torch.empty(fmt.c.V * fmt.c.nvec, dtype=vals_csr.dtype, device=vals_csr.device)
    assert out.numel() == fmt.c.V * fmt.c.nvec and out.is_contiguous()
    rc = load_library().fs_csr_to_blk(ctypes.byref(fmt.c), vals_csr.data_ptr(), out.data_ptr(), _stream_ptr(stream))
    if rc:
        raise FsError(rc, "fs_csr_to_blk")
    return out


def fs_csr_transpose(rowptr, colidx, M: int, K: int, stream=None):
    """CSR of A^T on the GPU: returns (rowptr_t[K+1], colidx_t[nnz], perm[nnz]), perm[q] = position in
    A's CSR order of entry q of A^T's.  Convert the result with fs_convert for A^T * dC."""
    import torch
    assert rowptr.is_cuda and colidx.is_cuda and rowptr.dtype == torch.int32 and colidx.dtype == torch.int32
    assert rowptr.is_contiguous() and colidx.is_contiguous() and rowptr.numel() == M + 1
    nnz = colidx.numel()
    lib = load_library()
    need = ctypes.c_size_t(0)
    rc = lib.fs_csr_transpose_bytes(M, K, nnz, ctypes.byref(need))
    if rc:
        raise FsError(rc, "fs_csr_transpose_bytes")
    dev = rowptr.device
    rowptr_t = torch.empty(K + 1, dtype=torch.int32, device=dev)
    colidx_t = torch.empty(nnz, dtype=torch.int32, device=dev)
    perm = torch.empty(nnz, dtype=torch.int32, device=dev)
    scratch = torch.empty(need.value, dtype=torch.uint8, device=dev)
    rc = lib.fs_csr_transpose(M, K, nnz, rowptr.data_ptr(), colidx.data_ptr(), rowptr_t.data_ptr(),
                              colidx_t.data_ptr(), perm.data_ptr(), scratch.data_ptr(), need.value,
                              _stream_ptr(stream))
    if rc:
        raise FsError(rc, "fs_csr_transpose")
    scratch.record_stream(torch.cuda.current_stream() if stream is None else stream)
    return rowptr_t, colidx_t, perm


def fs_gather16(src, idx, out=None, stream=None):
    """out[i] = src[idx[i]] on 16-bit elements (values of A carried into the CSR order of A^T)."""
    import torch
    assert src.is_cuda and idx.is_cuda and idx.dtype == torch.int32 and src.element_size() == 2
    assert src.is_contiguous() and idx.is_contiguous()
    if out is None:
        out = torch.empty(idx.numel(), dtype=src.dtype, device=src.device)
    assert out.numel() == idx.numel() and out.dtype == src.dtype and out.is_contiguous()
    rc = load_library().fs_gather16(src.data_ptr(), idx.data_ptr(), idx.numel(), out.data_ptr(), _stream_ptr(stream))
    if rc:
        raise FsError(rc, "fs_gather16")
    return out


def fs_gather_probe(fmt: FsFormat, B, sink=None, stream=None):
    """Measurement aid: only the gather of fs_spmm (the rows of B named by the format's column indices)."""
    import torch
    assert B.is_cuda and B.dim() == 2 and B.stride(1) == 1 and B.shape[0] == fmt.c.K and B.element_size() == 2
    if sink is None:
        sink = torch.empty(1024 * 256, dtype=torch.int32, device=B.device)
    rc = load_library().fs_gather_probe(ctypes.byref(fmt.c), B.data_ptr(), B.shape[1], B.stride(0), sink.data_ptr(),
                                        sink.numel() * sink.element_size(), _stream_ptr(stream))
    if rc:
        raise FsError(rc, "fs_gather_probe")
    return sink


def fs_read_bytes(src, repeats: int = 1, sink=None, stream=None):
    """Measurement aid: read ``src`` ``repeats`` times in one kernel (L2 bandwidth when it fits the L2s)."""
    import torch
    if sink is None:
        sink = torch.empty(2048 * 256, dtype=torch.int32, device=src.device)
    rc = load_library().fs_read_bytes(src.data_ptr(), src.numel() * src.element_size(), int(repeats), sink.data_ptr(),
                                      sink.numel() * sink.element_size(), _stream_ptr(stream))
    if rc:
        raise FsError(rc, "fs_read_bytes")
    return sink


def fs_copy_bytes(dst, src, stream=None):
    """Plain streaming copy (measurement aid for calibrating byte counters)."""
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    rc = load_library().fs_copy_bytes(dst.data_ptr(), src.data_ptr(), nbytes, _stream_ptr(stream))
    if rc:
        raise FsError(rc, "fs_copy_bytes")
    return dst
