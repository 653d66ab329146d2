"""Independent decoder of the window format, used to check converters by round trip.

It walks the arrays the way a consumer kernel does (window -> block -> row ->
vector) and never looks at ``csr_to_slot``; it shares no code with either
converter.
"""
import numpy as np


def decode_to_dense(M, K, V, KB, win_ptr, vec_col, vals_blk, vec_mask=None):
    """Rebuild (dense values as uint16 bits, dense occupancy) from the format arrays."""
    dense = np.zeros((M, K), dtype=np.uint16)
    occ = np.zeros((M, K), dtype=bool)
    W = len(win_ptr) - 1
    for w in range(W):
        lo, hi = int(win_ptr[w]), int(win_ptr[w + 1])
        n = hi - lo
        nblk = (n + KB - 1) // KB
        for b in range(nblk):
            kb = min(KB, n - b * KB)
            base = V * (lo + b * KB)
            for r in range(V):
                i = w * V + r
                for c in range(kb):
                    v = lo + b * KB + c
                    bits = vals_blk[base + r * kb + c]
                    present = bool((int(vec_mask[v]) >> r) & 1) if vec_mask is not None else bits != 0
                    if i >= M:
                        assert bits == 0 and not (vec_mask is not None and present)
                        continue
                    if present:
                        dense[i, vec_col[v]] = bits
                        occ[i, vec_col[v]] = True
                    else:
                        assert bits == 0, "slot outside the pattern must hold +0.0"
    return dense, occ
