// One pass of a stable least-significant-digit radix sort on 8-bit digits of int32 keys, one wavefront per
// tile of 2048 entries, shared by the translation units that sort (the CSR transposition sorts entries by
// column; the conversion orders the work list).  Every translation unit gets its own copy.
//   hist     per tile, the number of entries per digit value
//   scan     (the caller's, fs_scan.h) exclusive prefix sum over (digit value, tile), digit-major: where
//            each tile's entries with a given digit start in the output
//   scatter  each wavefront walks its tile in order, 64 entries at a time; a lane's rank among the lanes
//            of the same digit comes from eight wave-wide ballots, so equal digits keep their input order
// No atomics touch global memory and the result does not depend on scheduling.
#pragma once

#include <algorithm>

#include "fs_common.h"

namespace {

constexpr int kSortTile = 2048;       // entries per wavefront for large sorts
constexpr int kSortTileSmall = 256;   // ... and for sorts of a few thousand entries, where a wavefront's 32 sequential
                                      // rounds per 2048-entry tile would be the whole run time
constexpr int kDigitBits = 8;
constexpr int kDigits = 1 << kDigitBits;

__global__ void __launch_bounds__(64) k_digit_hist(const int32_t *__restrict__ keys, int64_t n, int shift, int64_t ntile,
                                                   int *__restrict__ hist, int tile = kSortTile)
{
    __shared__ int h[kDigits];
    const int lane = threadIdx.x;
#pragma unroll
    for (int i = 0; i < kDigits / 64; i++) h[lane + 64 * i] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * tile;
    const int64_t end = std::min<int64_t>(base + tile, n);
    for (int64_t i = base + lane; i < end; i += 64) atomicAdd(&h[((uint32_t)keys[i] >> shift) & (kDigits - 1)], 1);
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kDigits / 64; i++) {
        const int d = lane + 64 * i;
        hist[(int64_t)d * ntile + blockIdx.x] = h[d];
    }
}

// FIRST: the payload of entry i is i itself (its position in the source CSR order).
template <bool FIRST>
__global__ void __launch_bounds__(64) k_digit_scatter(const int32_t *__restrict__ keys, const int32_t *__restrict__ vals,
                                                      int64_t n, int shift, int64_t ntile, const int *__restrict__ start,
                                                      int32_t *__restrict__ out_keys, int32_t *__restrict__ out_vals,
                                                      int tile = kSortTile)
{
    __shared__ int cur[kDigits];
    const int lane = threadIdx.x;
#pragma unroll
    for (int i = 0; i < kDigits / 64; i++) {
        const int d = lane + 64 * i;
        cur[d] = start[(int64_t)d * ntile + blockIdx.x];
    }
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * tile;
    const int64_t end = std::min<int64_t>(base + tile, n);
    const uint64_t below = ((uint64_t)1 << lane) - 1;
    for (int64_t i0 = base; i0 < end; i0 += 64) {  // the trip count is the same for all lanes
        const int64_t i = i0 + lane;
        const bool valid = i < end;
        const int32_t key = valid ? keys[i] : 0;
        const int32_t val = FIRST ? (int32_t)i : (valid ? vals[i] : 0);
        const int digit = ((uint32_t)key >> shift) & (kDigits - 1);
        uint64_t same = __ballot(valid);
#pragma unroll
        for (int b = 0; b < kDigitBits; b++) {
            const bool bit = (digit >> b) & 1;
            const uint64_t set = __ballot(valid && bit);
            same &= bit ? set : ~set;
        }
        const int rank = __popcll(same & below), cnt = __popcll(same);
        if (valid) {
            const int pos = cur[digit] + rank;
            out_keys[pos] = key;
            out_vals[pos] = val;
        }
        __syncthreads();  // one wavefront: orders the reads above before the update below
        if (valid && rank == cnt - 1) cur[digit] += cnt;
        __syncthreads();
    }
}

}  // namespace
