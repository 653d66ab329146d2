/*
 * flashsparse.h -- C ABI of the MI355X (gfx950) sparse library.
 *
 * Unstructured-sparse SpMM (C = A_sparse * B_dense) and SDDMM
 * (out = (X * Y^T) sampled at the stored positions of A) on the CDNA4 matrix
 * cores, over a vector-blocked row-window format (the paper's ME-BCRS,
 * Section 3.5) produced on the GPU from CSR.
 *
 * Conventions
 *  - Every function returns an fs_status (0 = FS_OK); nothing throws or aborts.
 *  - "d_" arguments are DEVICE pointers, everything else is a HOST pointer or
 *    a value.  The library allocates no device memory and keeps no state: all
 *    buffers belong to the caller and must stay alive until the work queued on
 *    `stream` has finished.  (One exception, fs_spmm_static, owns a fixed
 *    workspace inside the library's device image.)  `stream` is a hipStream_t passed as void*
 *    (NULL = the default stream).
 *  - Dense matrices are row-major with a leading dimension in ELEMENTS.
 *  - Element type is IEEE binary16 (FS_F16) or bfloat16 (FS_BF16); products
 *    are accumulated in fp32 on the matrix cores and rounded to the element
 *    type (nearest even) once, when the result is stored.
 *  - Arguments are checked before anything is launched; a failed check queues
 *    no work.  HIP launch failures are reported as FS_ERR_HIP.
 */
#ifndef FLASHSPARSE_H
#define FLASHSPARSE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FS_OK = 0,
    FS_ERR_INVALID_ARG = 1,      /* NULL pointer, negative size, misaligned pointer or leading dimension */
    FS_ERR_INVALID_CSR = 2,      /* column index out of [0,K) or not strictly ascending inside a row */
    FS_ERR_UNSUPPORTED = 3,      /* (V, KB, dtype, N, d) combination the kernels do not implement */
    FS_ERR_BUFFER_TOO_SMALL = 4, /* arena / scratch / workspace smaller than required */
    FS_ERR_TOO_LARGE = 5,        /* sizes that overflow the 32-bit indices of the format */
    FS_ERR_HIP = 6               /* a HIP runtime call or kernel launch failed */
} fs_status;

typedef enum { FS_F16 = 0, FS_BF16 = 1 } fs_dtype;

/*
 * Descriptor of a converted matrix.  Filled by fs_convert; plain data, lives in
 * host memory, may be copied freely.  All pointers point INTO the caller's
 * device arena.
 *
 * The format (paper Section 2.2 for windows / nonzero vectors / blocks,
 * Section 3.5 for the three arrays):
 *   window w   = rows [w*V, min(M, w*V+V)) of A;  W = ceil(M / V) windows
 *   vector     = a column of a window holding at least one stored entry;
 *                the vectors of a window are ordered by ascending column
 *   win_ptr[w] = index of window w's first vector; win_ptr[W] = nvec
 *   vec_col[v] = column of vector v
 *   vals_blk   = values, window after window, block after block.  Block b of
 *                window w holds vectors [b*KB, b*KB+kb), kb = min(KB, n_w - b*KB),
 *                as a V x kb row-major tile starting at element
 *                V*(win_ptr[w] + b*KB); entry (row r, vector c of the block) is
 *                at  + r*kb + c.  No padding vectors are stored: the array has
 *                exactly V*nvec elements; positions A does not store hold +0.0.
 * Additions used by the kernels (also produced bit-exactly):
 *   vec_mask[v]    bit r set iff row w*V+r stores column vec_col[v]
 *   csr_to_slot[p] element index in vals_blk of CSR entry p
 *   blk_desc       one record of four int32 per block slot.  Every window owns
 *                  max(1, ceil(n_w / KB)) block slots, numbered window after window:
 *                  {first vector, width kb (0 for the slot of an empty window)
 *                   | 256 if it is its window's last block | 512 if it is the first,
 *                   window, 0}
 *   items          work list of fs_spmm, fs_edge_softmax and the fused calls (fs_sddmm walks the block
 *                  slots directly): an item is a run of consecutive block
 *                  slots.  With T = chunk / KB: a window with more than 1.5 T blocks is cut into
 *                  round(blocks / T) parts of equal length (within one block), from its start;
 *                  shorter windows are never cut and are packed whole into items of about
 *                  min(T, 4) blocks.  No item has more than 2 * T + 4 blocks (at most 64).  n_items records of four int32
 *                  {first block slot, number of blocks, first partial slot, first vector}; a
 *                  record with 0 blocks is empty.  An item whose first or last window is only
 *                  partly inside it adds that part into an fp32 partial tile (slots are handed
 *                  out in item order: head first, then tail), n_split_items tiles in total.
 *   item_order     n_items int32: the order in which fs_spmm, fs_attention, fs_sddmm_spmm, fs_edge_softmax and
 *                  fs_edge_softmax_backward take the items, a permutation of
 *                  [0, n_items).  First the n_cut_items items that hold a part of a cut window, by the
 *                  column of their first vector (scaled to 16 bits: floor(column * 65536 / K)), so that
 *                  parts of different hub windows over the same columns run side by side; then the
 *                  others, costliest first (cost = blocks + blocks that end a window, capped at 128);
 *                  empty records last; ties in work-list order.  It only decides which item starts
 *                  when: results do not depend on it
 *   items_by_cost  the item records in that order: record t is items[item_order[t]]
 *   blk_row_base   V int32 per block slot: [x * V + r] = position in CSR order of the first stored entry of
 *                  window row r whose column is not below the column of slot x's first vector (the end of
 *                  the row if there is none).  With the occupancy masks this locates every entry of a
 *                  block in CSR order: fs_sddmm writes CSR-order output with it
 *   split_windows  n_split_windows records of four int32
 *                  {window, first partial slot, number of slots, 0}: the partial
 *                  tiles of a cut window are consecutive slots
 *   slot_range     n_split_items records of two int32, one per partial slot:
 *                  {first partial slot of its window, number of slots of that window}
 *                  (split_windows seen from a slot)
 */
typedef struct fs_format {
    int64_t M, K, nnz, nvec, W;
    int32_t V, KB;
    int32_t dtype; /* fs_dtype */
    int32_t chunk; /* target vectors per part of a cut window (T * KB), a multiple of KB */
    int64_t n_items, n_split_items, n_split_windows;
    const int32_t *win_ptr;       /* W + 1 */
    const int32_t *vec_col;       /* nvec */
    const uint32_t *vec_mask;     /* nvec */
    const int32_t *csr_to_slot;   /* nnz */
    const void *vals_blk;         /* V * nvec elements (all zeros when converted pattern-only) */
    const int32_t *blk_desc;      /* 4 * n_blocks */
    int64_t n_blocks;             /* block slots in total */
    const int32_t *items;         /* 4 * n_items */
    const int32_t *split_windows; /* 4 * n_split_windows */
    int64_t n_cut_items;          /* items that hold a part of a cut window: the first n_cut_items of item_order */
    const int32_t *item_order;    /* n_items */
    const int32_t *items_by_cost; /* 4 * n_items */
    const int32_t *blk_row_base;  /* V * n_blocks */
    const void *packed;           /* the format's own values bitmap-packed (the buffer fs_pack_values makes), or NULL:
                                     built by fs_convert for large matrices with long rows, read by fs_spmm */
    const int32_t *slot_range;    /* 2 * n_split_items: per partial-tile slot {first slot of its window, slots of the window}:
                                     what a part of a cut window needs to find the other parts' statistics (fs_edge_softmax) */
    size_t arena_used;            /* bytes of the arena actually occupied */
} fs_format;

/* Library version: major*10000 + minor*100 + patch. */
int fs_version(void);

/* Static string for a status code (never NULL). */
const char *fs_status_string(fs_status s);

/*
 * Upper bounds, in bytes, of the two device buffers fs_convert needs for a
 * matrix with M rows and nnz stored entries (they assume nvec <= nnz).
 *   arena   : holds the converted format; must outlive every fs_spmm / fs_sddmm on it
 *   scratch : only used during fs_convert
 * V in [1,32], KB in [1,64].  Errors: FS_ERR_INVALID_ARG, FS_ERR_TOO_LARGE.
 */
fs_status fs_format_bytes(int64_t M, int64_t nnz, int32_t V, int32_t KB, fs_dtype dtype,
                          size_t *arena_bytes, size_t *scratch_bytes);

/*
 * CSR -> window format, on the GPU (paper Section 3.1: the translation runs as
 * GPU kernels; Section 3.5: the arrays it produces).  Run once per sparsity
 * pattern.
 *   d_rowptr[M+1], d_colidx[nnz] : int32 CSR; columns strictly ascending in each row, in [0,K)
 *   d_vals[nnz]                  : 16-bit values, or NULL for a pattern-only conversion
 *                                  (vals_blk is then all zeros; use fs_sddmm to fill one)
 *   V   : rows per window, 0 = chosen by the library: 8, except 4 for a matrix that gets packed values (below)
 *         and in whose eight-row windows fewer than one stored entry in twenty shares its vector with another
 *         (counted during the conversion).  KB: vectors per block, 0 = default (32).
 *         Any V in [1,32], KB in [1,64] converts; the compute calls need V in {4,8,16}, KB = 32.
 *   chunk : target vectors per part of a window that is cut across work items (see fs_format.items),
 *           0 = chosen from the matrix; else a positive multiple of KB, at most 32*KB.
 *   d_arena / d_scratch : device buffers of at least the sizes fs_format_bytes reports,
 *                         256-byte aligned.
 * For a matrix with at least 4 Mi stored entries and 12 per row on average (bound by memory traffic), values
 * given and KB = 32, V <= 16, the conversion also stores the values bitmap-packed (fs_format.packed, see
 * fs_pack_values); fs_spmm then reads those instead of vals_blk.  Same results bit for bit.
 * Synchronises `stream` twice (the vector, block and work-item counts come back to the host, then the
 * counts of the cut windows).  On FS_ERR_INVALID_CSR the arena content is unspecified.
 * The CSR check is always on (it costs one comparison per entry).
 * Errors: FS_ERR_INVALID_ARG (a NULL pointer, a misaligned buffer, a chunk that is no multiple of KB or too
 * long, stored entries in a matrix without rows), FS_ERR_BUFFER_TOO_SMALL, FS_ERR_TOO_LARGE (a size or
 * V * nnz at or above 2^31), FS_ERR_INVALID_CSR, FS_ERR_HIP.
 */
fs_status fs_convert(int64_t M, int64_t K, int64_t nnz,
                     const int32_t *d_rowptr, const int32_t *d_colidx, const void *d_vals,
                     fs_dtype dtype, int32_t V, int32_t KB, int32_t chunk,
                     void *d_arena, size_t arena_bytes, void *d_scratch, size_t scratch_bytes,
                     void *stream, fs_format *out);

/*
 * Bytes of device workspace fs_spmm needs for N output columns (fp32 partial
 * tiles of the windows that were cut into several work items; 0 if none).
 */
fs_status fs_spmm_workspace_bytes(const fs_format *fmt, int64_t N, size_t *work_bytes);

/*
 * C = A * B (paper Section 3.3).  A is `fmt`; B is K x N, C is M x N.
 *   d_vals : value array to use, in vals_blk layout (V*nvec elements), or NULL for the format's own
 *            values (fmt->packed where the conversion made it and B spans less than 4 GiB, else
 *            fmt->vals_blk: same result bit for bit).  Passing the d_out_blk of fs_sddmm here chains the two.
 *   N % 8 == 0, ldb % 8 == 0, ldc % 8 == 0, d_B and d_C 16-byte aligned.
 *   d_work : workspace of fs_spmm_workspace_bytes(fmt, N) bytes, 16-byte aligned
 *            (may be NULL when that size is 0).
 * Every element of C's M x N region is overwritten (rows of empty windows get
 * zeros).  Asynchronous on `stream`; deterministic (no atomics).
 * The method multiplies whole V-row vectors: a row of B that any row of a window
 * references meets explicit zeros for the window's other rows, so an infinity or
 * NaN in B reaches all V rows of every window that references that row (0 * inf),
 * where the exact product would only touch the rows that store the column.
 * Finite inputs are unaffected.
 */
fs_status fs_spmm(const fs_format *fmt, const void *d_vals,
                  const void *d_B, int64_t N, int64_t ldb,
                  void *d_C, int64_t ldc,
                  void *d_work, size_t work_bytes, void *stream);

/*
 * fs_spmm for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same computation, same kernels, same
 * result bit for bit; the fp32 partial tiles of cut windows go to a fixed 32 MiB array inside the
 * library's device image (one copy per GPU, held until the process ends) instead of d_work.  The call
 * allocates and frees nothing.
 *   Needs fs_spmm_workspace_bytes(fmt, N) <= 32 MiB (33 554 432), else FS_ERR_TOO_LARGE and nothing is
 *   queued.  The current device must be the one `stream` and the buffers belong to; the array's address on
 *   that device is looked up on the first call there (at most 64 devices, else FS_ERR_UNSUPPORTED).
 *   All calls on one GPU share the array, which keeps the previous call's contents (every partial tile
 *   is written before it is read, so nothing needs clearing): two calls whose work overlaps in time on
 *   one GPU -- different streams, or different host threads' streams -- race and give wrong results;
 *   calls on one stream are ordered and safe.
 * Other arguments, checks and errors as for fs_spmm.
 */
fs_status fs_spmm_static(const fs_format *fmt, const void *d_vals,
                         const void *d_B, int64_t N, int64_t ldb,
                         void *d_C, int64_t ldc, void *stream);

/*
 * Bitmap-packed values.  The value array of Section 3.5 leaves out padding vectors but still stores the
 * zeros inside nonzero vectors (V - 1 of V values where a vector holds one entry).  The packed form takes
 * the same idea one level down: it keeps only the stored values, and the kernel rebuilds each block from
 * the per-vector occupancy masks.
 *   d_packed   : caller's buffer of fs_pack_bytes(fmt) bytes, 256-byte aligned.  fs_pack_values fills it
 *                with, per block slot, the index of its first stored value; the occupancy masks narrowed
 *                to one byte per vector (two for V = 16); and the nnz stored values, block after block,
 *                row-major inside a block.  Part of it serves as scratch during the call.
 *   d_vals_blk : values to pack, in vals_blk layout, or NULL for fmt->vals_blk.
 * fs_spmm_packed is fs_spmm reading that buffer instead of a vals_blk-layout array: same arguments
 * otherwise, same result bit for bit.  B must span less than 4 GiB (else FS_ERR_UNSUPPORTED).
 * It pays on large matrices bound by memory traffic (values shrink from 2V to about 2 bytes per vector;
 * convert those with V = 8); on small ones the decoding costs more than the traffic it saves.
 * Both calls are asynchronous on `stream`.
 */
fs_status fs_pack_bytes(const fs_format *fmt, size_t *packed_bytes);
fs_status fs_pack_values(const fs_format *fmt, const void *d_vals_blk, void *d_packed, size_t packed_bytes,
                         void *stream);
fs_status fs_spmm_packed(const fs_format *fmt, const void *d_packed,
                         const void *d_B, int64_t N, int64_t ldb,
                         void *d_C, int64_t ldc,
                         void *d_work, size_t work_bytes, void *stream);

/*
 * out = (X * Y^T) at the stored positions of A (paper Section 3.4).  A's values are not used.  X is M x d,
 * Y is K x d.  Two output forms, either or both:
 *   d_out_blk : V*nvec elements in the vals_blk layout, so that fs_spmm can consume it directly (the paper's
 *               Algorithm 1 serves the same purpose for its own register layout); positions outside the
 *               pattern get +0.0.  16-byte aligned, or NULL.
 *   d_out_csr : nnz elements in CSR order (entry p of the CSR arrays fs_convert was given), written by the
 *               same kernel -- no second pass over the scores.  2-byte aligned, or NULL.
 *   At least one of the two must be given.  d % 8 == 0, ldx % 8 == 0, ldy % 8 == 0, d_X and d_Y 16-byte aligned.
 * Asynchronous on `stream`; deterministic.
 */
fs_status fs_sddmm(const fs_format *fmt,
                   const void *d_X, int64_t ldx, const void *d_Y, int64_t ldy, int64_t d,
                   void *d_out_blk, void *d_out_csr, void *stream);

/*
 * Bytes of device workspace fs_edge_softmax needs (two floats per row for every part of a
 * window that was cut into several work items; 0 if none).
 */
fs_status fs_edge_softmax_workspace_bytes(const fs_format *fmt, size_t *work_bytes);

/*
 * Edge softmax: for every row i of A and every stored entry p of that row,
 *   out[p] = exp(scale * in[p]) / sum over the stored entries q of row i of exp(scale * in[q]),
 * on value arrays in the vals_blk layout -- the normalisation between fs_sddmm and fs_spmm in an
 * attention GNN (the softmax layer of the paper's Section 4.4 end-to-end model; the paper gives
 * no kernel for it, this is the textbook definition, evaluated in fp32 with the row maximum
 * subtracted first and rounded once to the element type).
 *   d_in_blk, d_out_blk : V*nvec elements each; may be the same buffer.  Positions of d_out_blk
 *                         outside the pattern get +0.0; a row without stored entries gets zeros.
 *   scale               : finite.
 *   d_work              : workspace of fs_edge_softmax_workspace_bytes(fmt) bytes, 4-byte aligned
 *                         (may be NULL when that size is 0).
 * Asynchronous on `stream`; deterministic (no atomics).
 */
fs_status fs_edge_softmax(const fs_format *fmt, const void *d_in_blk, void *d_out_blk, float scale,
                          void *d_work, size_t work_bytes, void *stream);

/*
 * Gradient of fs_edge_softmax with respect to its input, for training the attention GNN of the paper's
 * Section 4.4 (the paper describes no kernel for it; this is the Jacobian of the row softmax applied to a
 * vector): with p = the output of fs_edge_softmax(.., scale, ..) and g the gradient that arrives at p,
 *   out[q] = scale * p[q] * (g[q] - sum over the stored entries r of the row of q of p[r] * g[r]),
 * all three in the vals_blk layout (g is what fs_sddmm(dOut, H) writes; out is what fs_spmm takes as values
 * for the gradients of X and, on the transposed format, of Y).  fp32 arithmetic, one rounding to the element
 * type; positions outside the pattern get +0.0.
 *   d_p_blk, d_g_blk, d_out_blk : V*nvec elements each; d_out_blk may be either input buffer.
 *   scale                       : the scale of the forward call; finite.
 *   d_work                      : workspace of fs_edge_softmax_workspace_bytes(fmt) bytes, 4-byte aligned
 *                                 (may be NULL when that size is 0).
 * Asynchronous on `stream`; deterministic (no atomics).
 */
fs_status fs_edge_softmax_backward(const fs_format *fmt, const void *d_p_blk, const void *d_g_blk, float scale,
                                   void *d_out_blk, void *d_work, size_t work_bytes, void *stream);

/*
 * Sparse attention in one call:
 *   out = softmax_rows(scale * (X * Y^T) at the stored positions of A) * H,
 * i.e. fs_sddmm, fs_edge_softmax and fs_spmm (the chain of the attention GNN in the paper's Section 4.4
 * evaluation) without the scores ever leaving the registers: they are neither rounded to the element
 * type nor written to memory; the probabilities are rounded to the element type relative to the running
 * row maximum, multiplied with H on the matrix cores in fp32, and the sum is divided by the fp32 row
 * total once, at the end.  A's values are not used.  X is M x d, Y is K x d, H is K x N, out is M x N.
 *   d % 8 == 0, d <= 128; N % 8 == 0; leading dimensions % 8 == 0; all four pointers 16-byte aligned.
 *   X, Y and H must each span less than 4 GiB, with fewer than 2^24 rows and a row pitch
 *   below 2^24 bytes (else FS_ERR_UNSUPPORTED: use the three separate calls).
 *   scale  : finite.
 *   d_work : workspace of fs_attention_workspace_bytes(fmt, N) bytes, 16-byte aligned (may be NULL when
 *            that size is 0).
 * Every element of out's M x N region is overwritten; a row without stored entries gets zeros.
 * Asynchronous on `stream`; deterministic (no atomics).
 */
fs_status fs_attention_workspace_bytes(const fs_format *fmt, int64_t N, size_t *work_bytes);

/*
 * The same kernel without the softmax:
 *   out = ((scale * X * Y^T) at the stored positions of A, rounded to the element type) * H,
 * i.e. fs_sddmm followed by fs_spmm on its scores (Sections 3.4 and 3.3 chained, as in the attention GNN
 * of Section 4.4 before normalisation) without the score array ever being written.  With scale = 1 the
 * result is bit-identical to those two calls.  Arguments, limits and workspace as for fs_attention
 * (fs_attention_workspace_bytes covers both).
 */
fs_status fs_sddmm_spmm(const fs_format *fmt,
                        const void *d_X, int64_t ldx, const void *d_Y, int64_t ldy, int64_t d, float scale,
                        const void *d_H, int64_t N, int64_t ldh,
                        void *d_out, int64_t ldo,
                        void *d_work, size_t work_bytes, void *stream);
fs_status fs_attention(const fs_format *fmt,
                       const void *d_X, int64_t ldx, const void *d_Y, int64_t ldy, int64_t d, float scale,
                       const void *d_H, int64_t N, int64_t ldh,
                       void *d_out, int64_t ldo,
                       void *d_work, size_t work_bytes, void *stream);

/*
 * Reorder a value array from the vals_blk layout to CSR order:
 * d_out_csr[p] = d_blk[csr_to_slot[p]] for p in [0, nnz).  Asynchronous.
 */
fs_status fs_blk_to_csr(const fs_format *fmt, const void *d_blk, void *d_out_csr, void *stream);

/*
 * The inverse: place CSR-order values into the vals_blk layout,
 * d_out_blk[csr_to_slot[p]] = d_vals_csr[p], every other position +0.0 -- new values for the same
 * sparsity pattern (edge weights that change between calls) without converting again.
 *   d_out_blk : V*nvec elements, 16-byte aligned.  Pass it to fs_spmm as d_vals.
 * Asynchronous on `stream`.
 */
fs_status fs_csr_to_blk(const fs_format *fmt, const void *d_vals_csr, void *d_out_blk, void *stream);

/*
 * CSR of the transposed matrix, on the GPU -- the index structure behind A^T * dC, the gradient of
 * C = A * B with respect to B in the training workloads of the paper's Section 4.4 (the paper gives
 * no kernel for it).  Convert the result with fs_convert and use fs_spmm on it; the gradient with
 * respect to A's values is fs_sddmm(fmt, dC, B).
 *   d_rowptr[M+1], d_colidx[nnz] : int32 CSR of A (M x K), columns ascending in each row and in
 *                                  [0,K).  Not checked here: fs_convert checks the same arrays.
 *                                  Invalid input gives a meaningless result but no invalid access.
 *   d_rowptr_t[K+1], d_colidx_t[nnz] : CSR of A^T (K x M), columns ascending in each row
 *   d_perm[nnz]                  : d_perm[q] = position in A's CSR order of the entry at position q
 *                                  of A^T's CSR order; fs_gather16 with it carries A's values over
 *   d_scratch                    : fs_csr_transpose_bytes(M, K, nnz) bytes, 256-byte aligned; only
 *                                  used during the call (may be NULL when nnz is 0)
 * Asynchronous on `stream`, no host synchronisation; deterministic (a stable radix sort by column).
 * Errors: FS_ERR_INVALID_ARG, FS_ERR_TOO_LARGE (a size above 2^31 - 4097), FS_ERR_BUFFER_TOO_SMALL.
 */
fs_status fs_csr_transpose_bytes(int64_t M, int64_t K, int64_t nnz, size_t *scratch_bytes);
fs_status fs_csr_transpose(int64_t M, int64_t K, int64_t nnz,
                           const int32_t *d_rowptr, const int32_t *d_colidx,
                           int32_t *d_rowptr_t, int32_t *d_colidx_t, int32_t *d_perm,
                           void *d_scratch, size_t scratch_bytes, void *stream);

/*
 * d_dst[i] = d_src[d_idx[i]] for i in [0, n), 16-bit elements; d_idx values must lie inside d_src.
 * With fs_csr_transpose's d_perm: the values of A in the CSR order of A^T.  Asynchronous.
 */
fs_status fs_gather16(const void *d_src, const int32_t *d_idx, int64_t n, void *d_dst, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* FLASHSPARSE_H */
