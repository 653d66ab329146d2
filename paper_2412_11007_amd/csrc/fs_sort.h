// One pass of a stable least-significant-digit radix sort on 8-bit digits of int32 keys, one wavefront per
// tile of 2048 entries, shared by the translation units that sort (the CSR transposition sorts entries by
// column; the conversion orders the work list).  Every translation unit gets its own copy.
//   hist     per tile, the number of entries per digit value
//   scan     (the caller's, fs_scan.h) exclusive prefix sum over (digit value, tile), digit-major: where
//            each tile's entries with a given digit start in the output
//   scatter  each wavefront walks its tile in order, 64 entries at a time; a lane's rank among the lanes
//            of the same digit comes from eight wave-wide ballots, so equal digits keep their input order;
//            four wavefronts (four consecutive tiles) share a workgroup and write their output together
// No atomics touch global memory and the result does not depend on scheduling.
#pragma once

#include <algorithm>

#include "fs_common.h"
#include "fs_scan.h"

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

// Four wavefronts, four consecutive tiles.  In the output the entries of these tiles with a given digit are
// neighbours (the scan is digit-major, tile-minor), so the group's share of a digit is one run, four times
// as long as a tile's.  First every wavefront ranks its tile as above -- its keys are loaded up front, so the
// rounds wait for nothing but LDS -- and notes, for every output slot of the group, which entry goes there
// (a 16-bit index, 16 KB of LDS for the group); then the workgroup walks the output slots in order and
// fetches their entries again (they are still in cache), so that neighbouring lanes write neighbouring
// addresses: runs of ~128 bytes instead of scattered 4-byte pieces of ~32-byte runs.
// FIRST: the payload of entry i is i itself (its position in the source CSR order).
constexpr int kScatterWaves = 4;
constexpr int kMaxRounds = kSortTile / 64;

template <bool FIRST>
__global__ void __launch_bounds__(64 * kScatterWaves)
k_digit_scatter(const int32_t *__restrict__ keys, const int32_t *__restrict__ vals, int64_t n, int shift, int64_t ntile,
                const int *__restrict__ start, int32_t *__restrict__ out_keys, int32_t *__restrict__ out_vals,
                int tile = kSortTile)
{
    static_assert(64 * kScatterWaves == kDigits && kDigits == kScanThreads, "one thread per digit value builds the tables");
    __shared__ int cur[kScatterWaves][kDigits];  // where a tile's next entry with digit d goes in the output
    __shared__ int gbase[kDigits];               // where the group's entries with digit d start in the output ...
    __shared__ int lstart[kDigits];              // ... and among the group's own output slots
    __shared__ uint16_t source[kScatterWaves * kSortTile];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t t0 = (int64_t)blockIdx.x * kScatterWaves, t1 = std::min<int64_t>(t0 + kScatterWaves, ntile);
    {
        const int d = threadIdx.x;
        const int g0 = start[(int64_t)d * ntile + t0], g1 = start[(int64_t)d * ntile + t1];
        int tot;
        lstart[d] = block_exclusive_scan(g1 - g0, &tot);
        gbase[d] = g0;
#pragma unroll
        for (int k = 0; k < kScatterWaves; k++) cur[k][d] = t0 + k < ntile ? start[(int64_t)d * ntile + t0 + k] : 0;
    }
    __syncthreads();
    const int64_t first = t0 * tile;  // the group's first entry
    const int64_t base = (t0 + w) * tile, end = std::min<int64_t>(base + tile, n);
    const uint64_t below = ((uint64_t)1 << lane) - 1;
    int32_t key[kMaxRounds];
#pragma unroll
    for (int r = 0; r < kMaxRounds; r++) {
        const int64_t i = base + r * 64 + lane;
        key[r] = (r * 64 < tile && i < end) ? keys[i] : 0;
    }
#pragma unroll
    for (int r = 0; r < kMaxRounds; r++) {
        if (r * 64 >= tile || base + r * 64 >= end) break;  // the same for all lanes
        const int64_t i = base + r * 64 + lane;
        const bool valid = i < end;
        const int digit = ((uint32_t)key[r] >> shift) & (kDigits - 1);
        uint64_t same = __ballot(valid);
#pragma unroll
        for (int b = 0; b < kDigitBits; b++) {
            const bool bit = (digit >> b) & 1;
            const uint64_t set = __ballot(valid && bit);
            same &= bit ? set : ~set;
        }
        const int rank = __popcll(same & below), cnt = __popcll(same);
        int pos = 0;
        if (valid) {
            pos = cur[w][digit];
            source[pos + rank - gbase[digit] + lstart[digit]] = (uint16_t)(i - first);
        }
        __builtin_amdgcn_wave_barrier();  // the wavefront's reads above stay before its update below
        if (valid && rank == cnt - 1) cur[w][digit] = pos + cnt;
        __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();
    const int total = (int)(std::min<int64_t>(t1 * tile, n) - first);
#pragma unroll 4
    for (int s = threadIdx.x; s < total; s += 64 * kScatterWaves) {
        const int64_t i = first + source[s];
        const int32_t k = keys[i];
        const int32_t v = FIRST ? (int32_t)i : vals[i];
        const int digit = ((uint32_t)k >> shift) & (kDigits - 1);
        const int pos = gbase[digit] + (s - lstart[digit]);
        out_keys[pos] = k;
        out_vals[pos] = v;
    }
}

}  // namespace
