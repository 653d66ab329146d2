// Which row of a CSR matrix stores entry p, for kernels that run one thread per stored entry: shared by the
// translation units that walk a CSR structure entry by entry.  Every translation unit gets its own copy.
//
// The 256 entries of a workgroup lie in consecutive rows.  A small kernel finds the row of every 256th
// entry beforehand (group_rows[b] = row of entry min(256 b, nnz - 1): one full search per workgroup, done
// ahead instead of inside it, where every thread would wait for it); the workgroup copies the row pointers
// between its first row and the next workgroup's into LDS and every thread searches there.  All searches
// stay inside [0, M) whatever rowptr holds, so a malformed rowptr cannot cause an out-of-range read.
#pragma once

#include "fs_common.h"

namespace {

constexpr int kEntriesPerGroup = 256;  // threads (= stored entries) per workgroup of a per-entry kernel

// The last row r in [lo, hi) with rowptr[r] <= p, given rowptr[lo] <= p.
__device__ __forceinline__ int64_t last_row_at_or_before(const int32_t *__restrict__ rowptr, int64_t lo, int64_t hi, int64_t p)
{
    while (hi - lo > 1) {  // invariant: the answer is in [lo, hi)
        const int64_t mid = lo + ((hi - lo) >> 1);
        if (rowptr[mid] <= p) lo = mid; else hi = mid;
    }
    return lo;
}

// group_rows[b] for b in [0, n_groups], n_groups = ceil(nnz / 256); needs M >= 1 and nnz >= 1.
__global__ void k_group_rows(const int32_t *__restrict__ rowptr, int64_t M, int64_t nnz, int64_t n_groups,
                             int32_t *__restrict__ group_rows)
{
    const int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (b > n_groups) return;
    group_rows[b] = (int32_t)last_row_at_or_before(rowptr, 0, M, min(b * kEntriesPerGroup, nnz - 1));
}

// Row of entry p = blockIdx.x * 256 + threadIdx.x, or -1 for p >= nnz.  Every thread of the workgroup must
// call it (it holds a barrier); sh_ptr is LDS for 256 ints.
__device__ __forceinline__ int64_t group_row_of(const int32_t *__restrict__ rowptr, int64_t nnz, int64_t p,
                                                const int32_t *__restrict__ group_rows, int32_t *sh_ptr)
{
    const int64_t r_first = group_rows[blockIdx.x], r_last = group_rows[blockIdx.x + 1];
    const int64_t n = r_last - r_first + 1;  // rows the workgroup's entries may lie in: the same for every thread
    if (n > kEntriesPerGroup) {               // many empty rows in between: search the row pointers in place
        if (p >= nnz) return -1;
        return last_row_at_or_before(rowptr, r_first, r_last + 1, p);
    }
    if ((int64_t)threadIdx.x < n) sh_ptr[threadIdx.x] = rowptr[r_first + threadIdx.x];
    __syncthreads();
    if (p >= nnz) return -1;
    int lo = 0, hi = (int)n;  // invariant: sh_ptr[lo] <= p, the answer is in [lo, hi)
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (sh_ptr[mid] <= p) lo = mid; else hi = mid;
    }
    return r_first + lo;
}

}  // namespace
