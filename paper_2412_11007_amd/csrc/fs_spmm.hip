// SpMM on the CDNA4 matrix cores over the row-window format (paper Section 3.3).
//
// One wavefront owns one work item = a run of consecutive 32-vector blocks
// (whole small windows packed together, or a piece of a long window), and all
// N output columns of a 128-column pass.  Per block of 32 vectors it
//   * reads the 32 column indices (one per lane),
//   * gathers the 32 rows of B they name, every lane loading 16 contiguous
//     bytes so that a row is read as one contiguous run by adjacent lanes
//     (the intent of the paper's memory-efficient thread mapping, Section 3.3),
//   * stages them in LDS and reads them back transposed (ds_read_b64_tr_b16),
//     which yields the matrix-core operand layout where one lane holds eight
//     consecutive k for one column,
//   * issues one v_mfma_f32_16x16x32 per 16 output columns.
//
// Operand roles follow the paper's swap-and-transpose idea (Section 3.2,
// Equation 1): the product is computed as C^T = B^T * A^T, i.e. the gathered
// dense tile is the matrix core's left operand (16 columns x 32 vectors) and
// the sparse block its right operand (32 vectors x 16 window rows).  With
// that choice a lane's four accumulators are four consecutive columns of one
// row of C: rounded, they pass through LDS once more and leave as 16-byte pieces
// of contiguous rows.  For V = 8 the upper eight window rows of the right
// operand are zero.
//
// The last block of a window may hold fewer than 32 vectors; lanes past its
// width feed zeros and load nothing (paper Section 3.5, residue handling).
//
// A window that lies whole inside an item is rounded and stored to C when its
// last block is done.  Windows cut across items accumulate into fp32 partial
// tiles that a second kernel adds in a fixed order: no atomics, bit-reproducible
// results.
#include <cstdlib>

#include "fs_common.h"

#ifndef FS_SPMM_WPB
#define FS_SPMM_WPB 4  // wavefronts (= work items) per workgroup
#endif

namespace {

// Rotation (in 32-byte units) applied to the column position of LDS row r, chosen so that the
// eight rows one half-wave reads in a transposed load fall into distinct banks.
template <int NT>
__device__ __forceinline__ int lds_rot(int r)
{
    if constexpr (NT == 8) return (r & 3) + 4 * ((r >> 3) & 1);
    else if constexpr (NT == 4) return ((r >> 1) & 1) + 2 * ((r >> 3) & 1);
    else if constexpr (NT == 2) return (r >> 3) & 1;
    else return 0;
}

// One 32-vector block of an item (all fields are wave-uniform).
struct BlockDesc {
    int s;      // first vector
    int kb;     // vectors in the block, 0..32 (0: the block slot of an empty window)
    int w;      // window
    bool last;  // last block of its window
};

template <int DT, int V, int NT, int WPB>
__global__ void __launch_bounds__(64 * WPB) __attribute__((amdgpu_waves_per_eu(4)))
k_spmm(const int4 *__restrict__ items, int n_items, const int32_t *__restrict__ win_ptr, int W,
       const int32_t *__restrict__ vec_col, const uint16_t *__restrict__ vals,
       const uint16_t *__restrict__ B, int64_t ldb, int N,
       uint16_t *__restrict__ C, int64_t ldc, float *__restrict__ part, int64_t M, int nbx)
{
    constexpr int NC = NT * 16;   // columns per pass
    constexpr int LPR = NC / 8;   // lanes that share one gathered row (16 bytes each)
    constexpr int RPI = 64 / LPR; // rows per wave-wide load
    constexpr int NLD = 32 / RPI; // wave-wide loads per 32-vector block
    constexpr int RS = NC * 2;    // LDS row stride in bytes

    __shared__ __attribute__((aligned(16))) unsigned char lds_all[WPB][32 * RS];

    // column pass and group of WPB items of this workgroup
    const int pass = blockIdx.x / nbx;
    const int bx = blockIdx.x - pass * nbx;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int item = __builtin_amdgcn_readfirstlane(bx * WPB + wave);  // wave-uniform
    if (item >= n_items) return;  // no block-wide barrier is used below
    unsigned char *lds = lds_all[wave];

    const int4 it = items[item];
    const int nblk = it.z;
    if (nblk == 0) return;
    const int w0 = it.x;
    int slot = it.w;
    const int n0 = pass * NC;  // first column of this pass
    const int j = lane & 15, g = lane >> 4;

    // pointers of the item's windows: lane l holds win_ptr[w0 + l]
    const int wp_l = win_ptr[min(w0 + lane, W)];
    auto wp = [&](int wabs) -> int {
        const int rel = wabs - w0;
        return rel <= 63 ? __builtin_amdgcn_readlane(wp_l, rel) : win_ptr[min(wabs, W)];
    };
    // iterator over the item's blocks; it runs two blocks ahead of the multiply
    int iw = w0, ib = it.y, iws = wp(w0), iwe = wp(w0 + 1), produced = 0;
    auto next_block = [&]() -> BlockDesc {
        BlockDesc d;
        if (produced >= nblk) {
            d.s = 0; d.kb = 0; d.w = iw; d.last = false;
            return d;
        }
        produced++;
        d.s = iws + 32 * ib;
        d.kb = min(32, iwe - d.s);
        d.w = iw;
        d.last = d.s + 32 >= iwe;
        if (d.last) {
            iw++;
            ib = 0;
            iws = iwe;
            iwe = wp(iw + 1);
        } else {
            ib++;
        }
        return d;
    };

    fs_f4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; t++) acc[t] = fs_f4{0.f, 0.f, 0.f, 0.f};

    // per-lane constants of the gather and of the transposed read
    const int g_row = lane / LPR;                         // row within one wave-wide load
    const int g_col = n0 + (lane % LPR) * 8;              // first column of this lane's 16 bytes
    const uint16_t *Bcol = B + (g_col < N ? g_col : 0);   // lanes past N read (and never store) column 0
    const int e = (lane & 15) >> 2, q = lane & 3;

    // column indices (one per lane) of a block; lanes past its width load nothing
    auto load_cols = [&](const BlockDesc &d) -> int { return (lane < d.kb) ? vec_col[d.s + lane] : -1; };
    // 16 bytes of the block's values per lane.  Full block (row stride 32): lane (j, g) gets its operand
    // directly, vectors 8g..8g+7 of row j.  Narrow last block of a window (row stride kb < 32): the
    // V*kb values are contiguous, lane l takes elements 8l..8l+7; they are re-laid through LDS at use.
    auto load_vals = [&](const BlockDesc &d) -> fs_u4 {
        fs_u4 raw = fs_u4{0u, 0u, 0u, 0u};
        const uint16_t *blk = vals + (int64_t)V * d.s;
        if (d.kb == 32) {
            if (j < V) raw = *reinterpret_cast<const fs_u4 *>(blk + j * 32 + 8 * g);
        } else if (lane * 8 < V * d.kb) {
            raw = *reinterpret_cast<const fs_u4 *>(blk + 8 * lane);
        }
        return raw;
    };
    // Gather of a block's B rows into `stage`.  Vectors past the block's width re-read the block's first
    // row (row 0 for the block slot of an empty window): the sparse operand is zero there, so the
    // product ignores them and no lane has to be masked off.
    fs_u4 stage[NLD];
#define FS_GATHER(cols)                                                                      \
    {                                                                                        \
        const int first_ = max(__builtin_amdgcn_readfirstlane(cols), 0);                     \
        _Pragma("unroll") for (int l = 0; l < NLD; l++) {                                    \
            int idx_ = __shfl(cols, l * RPI + g_row, 64);                                    \
            idx_ = idx_ < 0 ? first_ : idx_;                                                 \
            stage[l] = *reinterpret_cast<const fs_u4 *>(Bcol + (int64_t)idx_ * ldb);         \
        }                                                                                    \
    }

    // software pipeline: while block i is multiplied, the gather and the values of block i+1 and the
    // indices of block i+2 are in flight
    BlockDesc d0 = next_block(), d1 = next_block();
    int col0 = load_cols(d0), col1 = load_cols(d1);
    fs_u4 raw0 = load_vals(d0);
    FS_GATHER(col0)

    for (int step = 0; step < nblk; step++) {
        const int kb = d0.kb;
        // sparse operand: rows j < V of the block, vectors 8g .. 8g+7; vectors past kb are zero
        fs_frag sp;
        sp.u = raw0;
        if (kb > 0 && kb < 32) {
            *reinterpret_cast<fs_u4 *>(lds + 16 * lane) = raw0;  // V*kb*2 <= 1 KB of contiguous values
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const uint16_t *lv = reinterpret_cast<const uint16_t *>(lds);
            const int jr = (j < V ? j : 0) * kb;
#pragma unroll
            for (int x = 0; x < 8; x++) {
                const int c = 8 * g + x;
                const uint16_t v = lv[jr + min(c, kb - 1)];
                sp.e[x] = (c < kb && j < V) ? v : (uint16_t)0;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
        if (kb > 0) {
            // the gathered rows go to LDS (this is where the wave waits for the gather)
#pragma unroll
            for (int l = 0; l < NLD; l++) {
                const int r = l * RPI + g_row;
                const int pos = (((lane % LPR) * 16) + 32 * lds_rot<NT>(r)) & (RS - 1);
                *reinterpret_cast<fs_u4 *>(lds + r * RS + pos) = stage[l];
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }

        // queue the loads of the blocks ahead before multiplying: the indices two blocks ahead first,
        // then the values and the gather of the next block (its indices arrived a step ago)
        const BlockDesc d2 = next_block();
        const int col2 = load_cols(d2);
        const fs_u4 raw1 = load_vals(d1);
        if (step + 1 < nblk) FS_GATHER(col1)

        if (kb > 0) {
            // transposed reads + matrix-core products, one per 16-column tile
#pragma unroll
            for (int t = 0; t < NT; t++) {
                fs_frag dn;
#pragma unroll
                for (int h = 0; h < 2; h++) {
                    const int r = 8 * g + 4 * h + e;
                    const int pos = (32 * t + 8 * q + 32 * lds_rot<NT>(r)) & (RS - 1);
                    dn.s[h] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (fs_s4 __attribute__((address_space(3))) *)(lds + r * RS + pos));
                }
                acc[t] = fs_mfma_16x16x32<DT>(dn, sp, acc[t]);
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }

        if (d0.last || step == nblk - 1) {
            // flush: lane (j, g) holds C[w*V + j][n0 + 16t + 4g .. +3].  A window that lies whole inside
            // the item goes to C (zeros for an empty window); a part of a window goes to an fp32
            // partial tile.
            const bool whole = d0.last && (d0.w != w0 || it.y == 0);
            if (whole && NT <= 4) {
                // Narrow passes flush often relative to their work: round, lay the V x NC tile out
                // row-major in LDS (rows rotated by 32 bytes each so the writes spread over all banks),
                // then store it with the lane-to-row mapping of the gather: adjacent lanes write one row
                // of C contiguously, 16 bytes each.
                if (j < V) {
#pragma unroll
                    for (int t = 0; t < NT; t++) {
                        uint2 o;
                        o.x = (uint32_t)fs_round_bits<DT>(acc[t][0]) | ((uint32_t)fs_round_bits<DT>(acc[t][1]) << 16);
                        o.y = (uint32_t)fs_round_bits<DT>(acc[t][2]) | ((uint32_t)fs_round_bits<DT>(acc[t][3]) << 16);
                        const int pos = (32 * t + 8 * g + 32 * j) & (RS - 1);
                        *reinterpret_cast<uint2 *>(lds + j * RS + pos) = o;
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
                for (int l = 0; l < (V + RPI - 1) / RPI; l++) {
                    const int r = l * RPI + g_row;
                    const int64_t row = (int64_t)d0.w * V + r;
                    if (r < V && row < M && g_col < N) {
                        const int pos = (((lane % LPR) * 16) + 32 * r) & (RS - 1);
                        *reinterpret_cast<fs_u4 *>(C + row * ldc + g_col) = *reinterpret_cast<const fs_u4 *>(lds + r * RS + pos);
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            } else if (whole) {
                // 128-column passes: 8-byte pieces of contiguous rows straight from the accumulators
                const int64_t row = (int64_t)d0.w * V + j;
                if (j < V && row < M) {
                    uint16_t *crow = C + row * ldc;
#pragma unroll
                    for (int t = 0; t < NT; t++) {
                        const int col = n0 + 16 * t + 4 * g;
                        if (col < N) {
                            uint2 o;
                            o.x = (uint32_t)fs_round_bits<DT>(acc[t][0]) | ((uint32_t)fs_round_bits<DT>(acc[t][1]) << 16);
                            o.y = (uint32_t)fs_round_bits<DT>(acc[t][2]) | ((uint32_t)fs_round_bits<DT>(acc[t][3]) << 16);
                            *reinterpret_cast<uint2 *>(crow + col) = o;
                        }
                    }
                }
            } else {
                const int64_t row = (int64_t)d0.w * V + j;
                if (j < V && row < M) {
                    float *prow = part + ((int64_t)slot * V + j) * N;
#pragma unroll
                    for (int t = 0; t < NT; t++) {
                        const int col = n0 + 16 * t + 4 * g;
                        if (col < N)
                            *reinterpret_cast<float4 *>(prow + col) = make_float4(acc[t][0], acc[t][1], acc[t][2], acc[t][3]);
                    }
                }
            }
            if (!whole) slot++;
#pragma unroll
            for (int t = 0; t < NT; t++) acc[t] = fs_f4{0.f, 0.f, 0.f, 0.f};
        }
        d0 = d1; d1 = d2;
        col1 = col2;
        raw0 = raw1;
    }
#undef FS_GATHER
}

// Adds the partial tiles of one cut window in slot order and stores the rounded rows of C.
template <int DT, int V>
__global__ void __launch_bounds__(256)
k_spmm_reduce(const int4 *__restrict__ split_windows, const float *__restrict__ part, int N,
              uint16_t *__restrict__ C, int64_t ldc, int64_t M)
{
    const int4 sw = split_windows[blockIdx.x];
    const int w = sw.x, p0 = sw.y, cnt = sw.z;
    const int n4 = N / 4;
    const int64_t tile = (int64_t)V * N;  // floats per partial tile
    for (int idx = threadIdx.x; idx < V * n4; idx += blockDim.x) {
        const int j = idx / n4, c4 = idx - j * n4;
        const int64_t row = (int64_t)w * V + j;
        if (row >= M) continue;
        const float *src = part + (int64_t)p0 * tile + (int64_t)j * N + 4 * c4;
        float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
        int k = 0;
        for (; k + 8 <= cnt; k += 8) {  // eight loads in flight, added in slot order
            float4 v[8];
#pragma unroll
            for (int u = 0; u < 8; u++) v[u] = *reinterpret_cast<const float4 *>(src + (int64_t)(k + u) * tile);
#pragma unroll
            for (int u = 0; u < 8; u++) { sum.x += v[u].x; sum.y += v[u].y; sum.z += v[u].z; sum.w += v[u].w; }
        }
        for (; k < cnt; k++) {
            const float4 v = *reinterpret_cast<const float4 *>(src + (int64_t)k * tile);
            sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
        }
        uint2 o;
        o.x = (uint32_t)fs_round_bits<DT>(sum.x) | ((uint32_t)fs_round_bits<DT>(sum.y) << 16);
        o.y = (uint32_t)fs_round_bits<DT>(sum.z) | ((uint32_t)fs_round_bits<DT>(sum.w) << 16);
        *reinterpret_cast<uint2 *>(C + row * ldc + 4 * c4) = o;
    }
}

// Columns per pass for N > 64.  Measured on MI355X: 64-column passes (more, lighter wavefronts per CU)
// win on large matrices, 128-column passes (one pass for N = 128) on small ones.  FS_SPMM_PASS=64|128
// overrides the choice.
int fs_spmm_pass_override() { static int v = getenv("FS_SPMM_PASS") ? atoi(getenv("FS_SPMM_PASS")) : 0; return v; }

template <int DT, int V>
fs_status launch(const fs_format *f, const uint16_t *vals, const uint16_t *B, int64_t N, int64_t ldb, uint16_t *C,
                 int64_t ldc, float *part, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1)
{
    if (f->n_items == 0) return FS_OK;
    const int4 *items = (const int4 *)f->items;
    const int n_items = (int)f->n_items;
    constexpr int WPB = FS_SPMM_WPB;
    const int nbx = (n_items + WPB - 1) / WPB;
    int nc = N <= 32 ? 32 : N <= 64 ? 64 : (N <= 128 && n_items >= 16384) ? 64 : 128;  // columns per pass
    if (N > 64 && (fs_spmm_pass_override() == 64 || fs_spmm_pass_override() == 128)) nc = fs_spmm_pass_override();
    const int passes = (int)((N + nc - 1) / nc);
    const int64_t nblocks = (int64_t)nbx * passes;
    if (nblocks >= ((int64_t)1 << 31)) return FS_ERR_TOO_LARGE;
    dim3 grid((unsigned)nblocks, 1, 1), block(64 * WPB, 1, 1);
    if (ev0) FS_HIP(hipEventRecord(ev0, st));
#define FS_SPMM_ARGS items, n_items, f->win_ptr, (int)f->W, f->vec_col, vals, B, ldb, (int)N, C, ldc, part, f->M, nbx
    if (nc == 32)
        k_spmm<DT, V, 2, WPB><<<grid, block, 0, st>>>(FS_SPMM_ARGS);
    else if (nc == 64)
        k_spmm<DT, V, 4, WPB><<<grid, block, 0, st>>>(FS_SPMM_ARGS);
    else
        k_spmm<DT, V, 8, WPB><<<grid, block, 0, st>>>(FS_SPMM_ARGS);
#undef FS_SPMM_ARGS
    FS_LAUNCH_CHECK();
    if (ev1) FS_HIP(hipEventRecord(ev1, st));
    if (f->n_split_windows > 0) {
        k_spmm_reduce<DT, V><<<(unsigned)f->n_split_windows, 256, 0, st>>>((const int4 *)f->split_windows, part, (int)N, C,
                                                                            ldc, f->M);
        FS_LAUNCH_CHECK();
    }
    return FS_OK;
}

}  // namespace

fs_status fs_spmm_launch(const fs_format *f, const void *d_vals, const void *d_B, int64_t N, int64_t ldb, void *d_C,
                         int64_t ldc, void *d_work, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1)
{
    const uint16_t *vals = (const uint16_t *)(d_vals ? d_vals : f->vals_blk);
    const uint16_t *B = (const uint16_t *)d_B;
    uint16_t *C = (uint16_t *)d_C;
    float *part = (float *)d_work;
    if (f->dtype == FS_F16) {
        if (f->V == 8) return launch<FS_F16, 8>(f, vals, B, N, ldb, C, ldc, part, st, ev0, ev1);
        if (f->V == 16) return launch<FS_F16, 16>(f, vals, B, N, ldb, C, ldc, part, st, ev0, ev1);
    } else if (f->dtype == FS_BF16) {
        if (f->V == 8) return launch<FS_BF16, 8>(f, vals, B, N, ldb, C, ldc, part, st, ev0, ev1);
        if (f->V == 16) return launch<FS_BF16, 16>(f, vals, B, N, ldb, C, ldc, part, st, ev0, ev1);
    }
    return FS_ERR_UNSUPPORTED;
}
