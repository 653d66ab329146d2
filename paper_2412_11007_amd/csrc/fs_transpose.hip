// CSR of the transposed matrix, entirely on the GPU and without a host synchronisation.
//
// Training a GNN layer (the paper's Section 4.4 workloads) needs A^T * dC in the backward pass of
// C = A * B.  This library computes it with the same kernels on a second converted format, that of
// A^T; this file produces the CSR that conversion starts from, plus the permutation that carries
// per-entry values (edge weights, attention coefficients) from A's order into A^T's.
//
// The stored entries of A, taken in CSR order, are sorted by (row, column).  A STABLE sort of them by
// column alone therefore leaves them sorted by (column, row): the CSR order of A^T.  The sort is a
// least-significant-digit radix sort on 8-bit digits of the column index, one wavefront per tile:
//   hist     per tile, the number of entries per digit value
//   scan     exclusive prefix sum over (digit value, tile), digit-major: where each tile's entries
//            with a given digit start in the output
//   scatter  each wavefront walks its tile in order, 64 entries at a time; a lane's rank among the
//            lanes of the same digit comes from eight wave-wide ballots, so equal digits keep their
//            input order
// No atomics touch global memory and the result does not depend on scheduling.
#include <algorithm>

#include "fs_common.h"
#include "fs_rows.h"
#include "fs_scan.h"
#include "fs_sort.h"

namespace {

// rowptr_t[k] = number of entries whose column is below k, k in [0, K].
__global__ void k_rowptr_of_sorted(const int32_t *__restrict__ sorted_cols, int32_t n, int64_t K, int32_t *__restrict__ rowptr_t)
{
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k > K) return;
    int32_t lo = 0, hi = n;
    while (lo < hi) {
        const int32_t mid = lo + (hi - lo) / 2;
        if (sorted_cols[mid] < k) lo = mid + 1; else hi = mid;
    }
    rowptr_t[k] = lo;
}

// row_of[p] = the row of A that stores entry p: the last r with rowptr[r] <= p.
__global__ void __launch_bounds__(kEntriesPerGroup) k_row_of_entry(const int32_t *__restrict__ rowptr, int64_t n,
                                                                    const int32_t *__restrict__ group_rows,
                                                                    int32_t *__restrict__ row_of)
{
    __shared__ int32_t sh_ptr[kEntriesPerGroup];
    const int64_t p = (int64_t)blockIdx.x * kEntriesPerGroup + threadIdx.x;
    const int64_t r = group_row_of(rowptr, n, p, group_rows, sh_ptr);
    if (r >= 0) row_of[p] = (int32_t)r;
}

// colidx_t[i] = row_of[perm[i]]
__global__ void k_gather_i32(const int32_t *__restrict__ src, const int32_t *__restrict__ idx, int64_t n, int32_t *__restrict__ dst)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[idx[i]];
}

__global__ void k_fill_i32(int32_t *__restrict__ dst, int64_t n, int32_t v)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = v;
}

__global__ void k_gather16(const uint16_t *__restrict__ src, const int32_t *__restrict__ idx, int64_t n, uint16_t *__restrict__ dst)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[idx[i]];
}

inline unsigned grid_of(int64_t n, int threads) { return (unsigned)((n + threads - 1) / threads); }

// Scratch layout (ints): [keys 0: nnz][keys 1: nnz][payload: nnz][digit counts: 256 * tiles + 1][scan tmp]
struct TransposePlan {
    int64_t ntile;
    size_t key0, key1, val1, hist, tmp, total_ints;
};
TransposePlan plan_transpose(int64_t nnz)
{
    TransposePlan p;
    p.ntile = (nnz + kSortTile - 1) / kSortTile;
    const size_t e = fs_align_up((size_t)nnz, 64);
    size_t o = 0;
    p.key0 = o; o += e;
    p.key1 = o; o += e;
    p.val1 = o; o += e;
    p.hist = o; o += fs_align_up((size_t)kDigits * p.ntile + 1, 64);
    p.tmp = o; o += scan_tmp_ints((int64_t)kDigits * p.ntile);
    p.total_ints = o;
    return p;
}

bool sizes_ok(int64_t M, int64_t K, int64_t nnz) { return M >= 0 && K >= 0 && nnz >= 0; }
bool sizes_fit(int64_t M, int64_t K, int64_t nnz)
{
    const int64_t lim = (int64_t)INT32_MAX - 4096;
    return M <= lim && K <= lim && nnz <= lim;
}

}  // namespace

extern "C" fs_status fs_csr_transpose_bytes(int64_t M, int64_t K, int64_t nnz, size_t *scratch_bytes)
{
    if (!scratch_bytes || !sizes_ok(M, K, nnz)) return FS_ERR_INVALID_ARG;
    if (!sizes_fit(M, K, nnz)) return FS_ERR_TOO_LARGE;
    *scratch_bytes = plan_transpose(nnz).total_ints * sizeof(int) + 256;
    return FS_OK;
}

extern "C" fs_status fs_csr_transpose(int64_t M, int64_t K, int64_t nnz, const int32_t *d_rowptr, const int32_t *d_colidx,
                                      int32_t *d_rowptr_t, int32_t *d_colidx_t, int32_t *d_perm, void *d_scratch,
                                      size_t scratch_bytes, void *stream)
{
    if (!sizes_ok(M, K, nnz) || !d_rowptr || !d_rowptr_t) return FS_ERR_INVALID_ARG;
    if (nnz > 0 && (!d_colidx || !d_colidx_t || !d_perm || !d_scratch || M == 0 || K == 0)) return FS_ERR_INVALID_ARG;
    if (!sizes_fit(M, K, nnz)) return FS_ERR_TOO_LARGE;
    hipStream_t st = (hipStream_t)stream;
    if (nnz == 0) {
        k_fill_i32<<<grid_of(K + 1, 256), 256, 0, st>>>(d_rowptr_t, K + 1, 0);
        FS_LAUNCH_CHECK();
        return FS_OK;
    }
    if ((uintptr_t)d_scratch & 255) return FS_ERR_INVALID_ARG;
    const TransposePlan pl = plan_transpose(nnz);
    if (scratch_bytes < pl.total_ints * sizeof(int)) return FS_ERR_BUFFER_TOO_SMALL;
    int *S = (int *)d_scratch;
    int32_t *key[2] = {S + pl.key0, S + pl.key1};
    int *hist = S + pl.hist, *tmp = S + pl.tmp;

    int bits = 0;
    while (bits < 31 && ((K - 1) >> bits) != 0) bits++;
    const int P = std::max(1, (bits + kDigitBits - 1) / kDigitBits);
    const int32_t *src_key = d_colidx;
    const int32_t *src_val = nullptr;
    for (int p = 0; p < P; p++) {
        const int shift = p * kDigitBits;
        int32_t *dst_key = key[p & 1];
        int32_t *dst_val = ((P - 1 - p) & 1) ? S + pl.val1 : d_perm;  // the last pass writes d_perm
        k_digit_hist<<<(unsigned)pl.ntile, 64, 0, st>>>(src_key, nnz, shift, pl.ntile, hist);
        FS_LAUNCH_CHECK();
        fs_status s = scan_exclusive(hist, (int64_t)kDigits * pl.ntile, tmp, st);
        if (s != FS_OK) return s;
        if (p == 0)
            k_digit_scatter<true><<<(unsigned)((pl.ntile + kScatterWaves - 1) / kScatterWaves), 64 * kScatterWaves, 0, st>>>(src_key, nullptr, nnz, shift, pl.ntile, hist, dst_key, dst_val);
        else
            k_digit_scatter<false><<<(unsigned)((pl.ntile + kScatterWaves - 1) / kScatterWaves), 64 * kScatterWaves, 0, st>>>(src_key, src_val, nnz, shift, pl.ntile, hist, dst_key, dst_val);
        FS_LAUNCH_CHECK();
        src_key = dst_key;
        src_val = dst_val;
    }
    k_rowptr_of_sorted<<<grid_of(K + 1, 256), 256, 0, st>>>(src_key, (int32_t)nnz, K, d_rowptr_t);
    FS_LAUNCH_CHECK();
    int32_t *row_of = key[P & 1];  // the key buffer the last pass did not write
    int32_t *group_rows = hist;  // the digit counts are no longer needed; 256 * tiles + 1 >= nnz / 256 + 2 ints
    const int64_t n_groups = (nnz + kEntriesPerGroup - 1) / kEntriesPerGroup;
    k_group_rows<<<grid_of(n_groups + 1, 256), 256, 0, st>>>(d_rowptr, M, nnz, n_groups, group_rows);
    FS_LAUNCH_CHECK();
    k_row_of_entry<<<(unsigned)n_groups, kEntriesPerGroup, 0, st>>>(d_rowptr, nnz, group_rows, row_of);
    FS_LAUNCH_CHECK();
    k_gather_i32<<<grid_of(nnz, 256), 256, 0, st>>>(row_of, d_perm, nnz, d_colidx_t);
    FS_LAUNCH_CHECK();
    return FS_OK;
}

extern "C" fs_status fs_gather16(const void *d_src, const int32_t *d_idx, int64_t n, void *d_dst, void *stream)
{
    if (n < 0) return FS_ERR_INVALID_ARG;
    if (n == 0) return FS_OK;
    if (!d_src || !d_idx || !d_dst) return FS_ERR_INVALID_ARG;
    k_gather16<<<grid_of(n, 256), 256, 0, (hipStream_t)stream>>>((const uint16_t *)d_src, d_idx, n, (uint16_t *)d_dst);
    FS_LAUNCH_CHECK();
    return FS_OK;
}
