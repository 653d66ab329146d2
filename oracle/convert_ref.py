"""Reference converter: CSR -> vector-blocked row-window format (the paper's ME-BCRS, Section 3.5).

TEST INFRASTRUCTURE ONLY; integer-exact; numpy; shares nothing with the HIP
converter.  The steps follow the paper's description of the format:

* Section 2.2: V consecutive rows form a *window*; a V x 1 column slice of a
  window that holds at least one stored entry is a *nonzero vector*; every KB
  consecutive nonzero vectors of a window form a block, zero-filled where the
  matrix stores nothing.
* Section 3.5: three arrays.  Row pointers give where each window starts in
  the column-index array; the column-index array holds the column of every
  nonzero vector; the value array is laid out block after block, each block
  row-major, and NO padding vectors are stored, so the last block of a window
  is narrower than KB when the window's vector count is not a multiple of KB.

Readings where the paper is silent (the figure that fixes them is not part of
the text): vectors of a window are ordered by ascending column; the pointer
array has one terminating entry (W + 1 values); the row stride of a narrow last
block is its own width kb; a window cut short by the matrix edge keeps V rows in
the value array (the missing rows are zero); "nonzero" means *stored* (an
explicit zero value still marks a vector).

Two arrays are additions for the kernels' benefit and are part of the checked
output: a per-vector row-occupancy bit mask, and the slot of every CSR entry.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass
class FormatRef:
    M: int
    K: int
    nnz: int
    V: int
    KB: int
    W: int
    nvec: int
    win_ptr: np.ndarray  # int32, W+1
    vec_col: np.ndarray  # int32, nvec
    vec_mask: np.ndarray  # uint32, nvec; bit r set iff row w*V+r stores this column
    csr_to_slot: np.ndarray  # int32, nnz
    vals_blk: np.ndarray  # uint16 bits, V*nvec


def convert_ref(M: int, K: int, rowptr: np.ndarray, colidx: np.ndarray, vals_bits, V: int, KB: int) -> FormatRef:
    rowptr = np.asarray(rowptr, dtype=np.int64)
    colidx = np.asarray(colidx, dtype=np.int64)
    nnz = int(colidx.shape[0])
    W = (M + V - 1) // V  # windows; the last may have fewer than V real rows

    row = np.repeat(np.arange(M, dtype=np.int64), np.diff(rowptr))  # row of every stored entry
    win = row // V  # its window
    r = row % V  # its row inside the window

    # nonzero vectors = distinct (window, column) pairs; sorting the pair key
    # orders them by window, then by ascending column inside the window
    pair = win * np.int64(K) + colidx
    uniq, vec_of_entry = np.unique(pair, return_inverse=True)
    vec_of_entry = vec_of_entry.reshape(-1)
    nvec = int(uniq.shape[0])
    vec_win = uniq // K
    vec_col = (uniq % K).astype(np.int32)

    per_window = np.bincount(vec_win, minlength=W)
    win_ptr = np.zeros(W + 1, dtype=np.int64)
    win_ptr[1:] = np.cumsum(per_window)

    # occupancy mask: each (vector, row) pair occurs at most once, so adding the bits is an OR
    vec_mask = np.zeros(nvec, dtype=np.int64)
    np.add.at(vec_mask, vec_of_entry, np.int64(1) << r)

    # slot of entry (row r, vector v of window w):
    #   block b = v div KB, column c = v mod KB, width kb = min(KB, nvec_w - b*KB)
    #   slot = V*(win_ptr[w] + b*KB) + r*kb + c
    v = vec_of_entry - win_ptr[win]
    b = v // KB
    c = v % KB
    nvec_w = per_window[win]
    kb = np.minimum(KB, nvec_w - b * KB)
    slot = V * (win_ptr[win] + b * KB) + r * kb + c

    vals_blk = np.zeros(V * nvec, dtype=np.uint16)
    if vals_bits is not None:
        vals_blk[slot] = np.asarray(vals_bits, dtype=np.uint16)

    assert V * nvec < 2 ** 31
    return FormatRef(M, K, nnz, V, KB, W, nvec, win_ptr.astype(np.int32), vec_col,
                     vec_mask.astype(np.uint32), slot.astype(np.int32), vals_blk)


def pack_ref(fmt: FormatRef, vals_bits) -> tuple:
    """Bitmap-packed value array: the block-row-major value array of Section 3.5 with every position
    that the matrix does not store taken out (the per-vector occupancy masks say which those are).

    Returns (blk_ofs, packed): ``packed`` holds the nnz stored values in slot order, i.e. block after
    block and row-major inside a block; ``blk_ofs[s]`` is the index in it of the first value of block
    slot s (every window owns max(1, ceil(n_w / KB)) slots, numbered window after window), with one
    terminating entry.
    """
    order = np.argsort(fmt.csr_to_slot, kind="stable")
    packed = np.asarray(vals_bits, dtype=np.uint16)[order]
    slots_sorted = fmt.csr_to_slot[order].astype(np.int64)
    n = np.diff(fmt.win_ptr.astype(np.int64))
    nblk = np.maximum(1, (n + fmt.KB - 1) // fmt.KB)
    first_slot = np.concatenate([[0], np.cumsum(nblk)])
    n_blocks = int(first_slot[-1])
    # first vector of every block slot: window start + KB * (index of the slot inside its window)
    win_of_slot = np.repeat(np.arange(fmt.W, dtype=np.int64), nblk)
    idx_in_win = np.arange(n_blocks, dtype=np.int64) - first_slot[win_of_slot]
    first_vec = fmt.win_ptr.astype(np.int64)[win_of_slot] + fmt.KB * idx_in_win
    blk_ofs = np.searchsorted(slots_sorted, fmt.V * first_vec, side="left")
    blk_ofs = np.concatenate([blk_ofs, [fmt.nnz]]).astype(np.int32)
    return blk_ofs, packed


def issued_mac_ratio(win_ptr: np.ndarray, V_issue: int, KB_issue: int, nnz: int) -> float:
    """Redundancy R = multiply-accumulate slots the matrix unit issues / useful ones.

    A window with n vectors issues ceil(n / KB_issue) tile products of
    V_issue x KB_issue slots per output column; the useful work per output
    column is one MAC per stored entry.  (The quantity behind the paper's
    Figure 1 and Table 2.)
    """
    n = np.diff(np.asarray(win_ptr, dtype=np.int64))
    blocks = (n + KB_issue - 1) // KB_issue
    return float(V_issue * KB_issue * blocks.sum()) / float(max(nnz, 1))


def padded_format_bytes(win_ptr: np.ndarray, V: int, KB: int, elem_bytes: int = 2) -> dict:
    """Footprint of this format against the zero-vector-padded layout it replaces (paper Section 3.5, Table 7).

    Padded layout: every window's vector count rounded up to a multiple of KB in
    both the value and the column-index arrays, and two pointers per window.
    """
    n = np.diff(np.asarray(win_ptr, dtype=np.int64))
    W = n.shape[0]
    nvec = int(n.sum())
    padded_vec = int((((n + KB - 1) // KB) * KB).sum())
    ours = 4 * (W + 1) + 4 * nvec + elem_bytes * V * nvec
    padded = 4 * (2 * W) + 4 * padded_vec + elem_bytes * V * padded_vec
    return {"me_bcrs": ours, "padded": padded, "saved_frac": 1.0 - ours / padded if padded else 0.0}
