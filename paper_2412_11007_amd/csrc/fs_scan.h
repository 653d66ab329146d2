// Exclusive prefix sums over int32 arrays on the device (blocked reduce / recurse / apply), shared by
// the translation units that build index structures.  Every translation unit gets its own copy.
#pragma once

#include "fs_common.h"

namespace {

constexpr int kScanThreads = 256;
constexpr int kScanPerThread = 8;
constexpr int kScanTile = kScanThreads * kScanPerThread;

// ---------------------------------------------------------------- prefix sums
__device__ __forceinline__ int wave_inclusive_scan(int x)
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        int y = __shfl_up(x, d, 64);
        if (lane >= d) x += y;
    }
    return x;
}

// Exclusive scan of one int per thread across a 256-thread block; *total gets the block sum.
__device__ __forceinline__ int block_exclusive_scan(int x, int *total)
{
    __shared__ int wave_sum[kScanThreads / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc = wave_inclusive_scan(x);
    if (lane == 63) wave_sum[wave] = inc;
    __syncthreads();
    int ofs = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kScanThreads / 64; w++) {
        int s = wave_sum[w];
        if (w < wave) ofs += s;
        tot += s;
    }
    __syncthreads();
    *total = tot;
    return ofs + inc - x;
}

// Eight consecutive values of one thread (data is 16-byte aligned and base a multiple of eight): two 16-byte
// accesses where all eight exist, element by element at the end of the array.
__device__ __forceinline__ void scan_load8(const int *__restrict__ data, int64_t base, int64_t n, int (&v)[8])
{
    if (base + 8 <= n) {
        const int4 a = *reinterpret_cast<const int4 *>(data + base), b = *reinterpret_cast<const int4 *>(data + base + 4);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    } else {
#pragma unroll
        for (int i = 0; i < 8; i++) v[i] = base + i < n ? data[base + i] : 0;
    }
}
__device__ __forceinline__ void scan_store8(int *__restrict__ data, int64_t base, int64_t n, const int (&o)[8])
{
    if (base + 8 <= n) {
        *reinterpret_cast<int4 *>(data + base) = int4{o[0], o[1], o[2], o[3]};
        *reinterpret_cast<int4 *>(data + base + 4) = int4{o[4], o[5], o[6], o[7]};
    } else {
#pragma unroll
        for (int i = 0; i < 8; i++)
            if (base + i < n) data[base + i] = o[i];
    }
}
static_assert(kScanPerThread == 8, "scan_load8 / scan_store8 move eight values per thread");

__global__ void __launch_bounds__(kScanThreads) k_scan_reduce(const int *__restrict__ in, int64_t n, int *__restrict__ bsum)
{
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanPerThread;
    int v[kScanPerThread];
    scan_load8(in, base, n, v);
    int s = 0;
#pragma unroll
    for (int i = 0; i < kScanPerThread; i++) s += v[i];
    int tot;
    block_exclusive_scan(s, &tot);
    if (threadIdx.x == 0) bsum[blockIdx.x] = tot;
}

// In place: data[i] <- sum of data[0..i); the last block also writes data[n] <- grand total.
__global__ void __launch_bounds__(kScanThreads) k_scan_apply(int *__restrict__ data, int64_t n, const int *__restrict__ bofs,
                                                             int *__restrict__ total_out)
{
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanPerThread;
    int v[kScanPerThread], o[kScanPerThread];
    scan_load8(data, base, n, v);
    int s = 0;
#pragma unroll
    for (int i = 0; i < kScanPerThread; i++) s += v[i];
    int tot;
    int ofs = block_exclusive_scan(s, &tot) + (bofs ? bofs[blockIdx.x] : 0);
#pragma unroll
    for (int i = 0; i < kScanPerThread; i++) {
        o[i] = ofs;
        ofs += v[i];
    }
    scan_store8(data, base, n, o);
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == kScanThreads - 1) {
        data[n] = ofs;
        if (total_out) *total_out = ofs;
    }
}

// Up to 65536 values in one launch: a single workgroup of 1024 threads walks tiles of 8192 values, every
// thread eight consecutive ones per tile (a wavefront reads 2 KiB contiguously), carrying the running total.
// The next tile's values are loaded before the current tile is scanned, so that only the first load's
// latency is exposed.
constexpr int kSmallScanThreads = 1024;
constexpr int kSmallScanMax = 65536;
__global__ void __launch_bounds__(kSmallScanThreads) k_scan_small(int *__restrict__ data, int n, int *__restrict__ total_out)
{
    __shared__ int wave_sum[2][kSmallScanThreads / 64];
    constexpr int kTile = kSmallScanThreads * 8;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    auto load_tile = [&](int t0, int (&v)[8]) { scan_load8(data, t0 + threadIdx.x * 8, n, v); };
    int carry = 0, buf = 0;
    int v[8];
    load_tile(0, v);
    for (int t0 = 0; t0 < n; t0 += kTile, buf ^= 1) {
        int nv[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if (t0 + kTile < n) load_tile(t0 + kTile, nv);
        const int base = t0 + threadIdx.x * 8;
        int s = 0;
#pragma unroll
        for (int i = 0; i < 8; i++) s += v[i];
        const int inc = wave_inclusive_scan(s);
        if (lane == 63) wave_sum[buf][wave] = inc;
        __syncthreads();  // (the other buffer is rewritten only after the next tile's barrier)
        int ofs = 0, tot = 0;
#pragma unroll
        for (int w = 0; w < kSmallScanThreads / 64; w++) {
            const int x = wave_sum[buf][w];
            if (w < wave) ofs += x;
            tot += x;
        }
        int run = carry + ofs + inc - s;
        int o[8];
#pragma unroll
        for (int i = 0; i < 8; i++) {
            o[i] = run;
            run += v[i];
        }
        scan_store8(data, base, n, o);
        carry += tot;
#pragma unroll
        for (int i = 0; i < 8; i++) v[i] = nv[i];
    }
    if (threadIdx.x == 0) {
        data[n] = carry;
        if (total_out) *total_out = carry;
    }
}

size_t scan_tmp_ints(int64_t n)
{
    size_t tot = 0;
    while (n > kScanTile) {
        int64_t nb = (n + kScanTile - 1) / kScanTile;
        tot += fs_align_up((size_t)nb + 1, 64);
        n = nb;
    }
    return tot + 64;
}

// data has n+1 ints; tmp has scan_tmp_ints(n) ints.  total_out (optional) also receives the grand total.
fs_status scan_exclusive(int *data, int64_t n, int *tmp, hipStream_t st, int *total_out = nullptr)
{
    int64_t nb = n <= 0 ? 1 : (n + kScanTile - 1) / kScanTile;
    if (nb > 1 && n <= kSmallScanMax) {
        k_scan_small<<<1, kSmallScanThreads, 0, st>>>(data, (int)n, total_out);
        FS_LAUNCH_CHECK();
        return FS_OK;
    }
    if (nb == 1) {
        k_scan_apply<<<1, kScanThreads, 0, st>>>(data, n < 0 ? 0 : n, nullptr, total_out);
        FS_LAUNCH_CHECK();
        return FS_OK;
    }
    k_scan_reduce<<<(unsigned)nb, kScanThreads, 0, st>>>(data, n, tmp);
    FS_LAUNCH_CHECK();
    fs_status s = scan_exclusive(tmp, nb, tmp + fs_align_up((size_t)nb + 1, 64), st);
    if (s != FS_OK) return s;
    k_scan_apply<<<(unsigned)nb, kScanThreads, 0, st>>>(data, n, tmp, total_out);
    FS_LAUNCH_CHECK();
    return FS_OK;
}


}  // namespace
