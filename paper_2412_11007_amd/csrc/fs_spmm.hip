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
// The last block of a window may hold fewer than 32 vectors; the positions past
// its width feed zeros to the matrix core, and the lanes that would gather rows
// for them re-read the block's last valid row instead of the next window's
// (paper Section 3.5, residue handling).
//
// A window that lies whole inside an item is rounded and stored to C when its
// last block is done.  Windows cut across items accumulate into fp32 partial
// tiles that a second kernel adds in a fixed order: no atomics, bit-reproducible
// results.
#include <algorithm>
#include <cstdlib>
#include <utility>

#include "fs_common.h"
#include "fs_tile.h"

namespace {

// 16 bytes at a 2-byte-aligned address, read with one load instruction
typedef fs_u4 fs_u4_unaligned __attribute__((aligned(2)));

// Packed values -> sparse operand.  `raw` holds the lane's stored values back to back (halfword 0 first),
// bit x of m8 says whether vector x of the lane's eight is stored: stored positions take the next
// halfword, the others +0.0.
__device__ __forceinline__ fs_u4 fs_expand8(fs_u4 raw, uint32_t m8)
{
    uint64_t lo = raw.x | ((uint64_t)raw.y << 32), hi = raw.z | ((uint64_t)raw.w << 32);
    uint32_t out[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int x = 0; x < 8; x++) {
        const bool bit = (m8 >> x) & 1u;
        const uint32_t h = (uint32_t)lo & 0xFFFFu;
        out[x >> 1] |= bit ? (h << (16 * (x & 1))) : 0u;
        const uint64_t lo_next = (lo >> 16) | (hi << 48);
        lo = bit ? lo_next : lo;
        hi = bit ? (hi >> 16) : hi;
    }
    return fs_u4{out[0], out[1], out[2], out[3]};
}

// BIG: B spans 4 GiB or more, 64-bit gather offsets.  PK: `vals` holds only the stored values, block
// after block and row-major inside a block, blk_ofs[b] is the first value of block slot b, and the
// sparse operand is rebuilt from the per-vector occupancy masks (no zero is read from memory).
template <int DT, int V, int NT, int WPB, bool BIG, bool PK = false>
__global__ void __launch_bounds__(64 * WPB) __attribute__((amdgpu_waves_per_eu(PK ? 3 : 4)))
k_spmm(const int4 *__restrict__ items, int n_items, const int4 *__restrict__ blk_desc, int nvec,
       const int32_t *__restrict__ vec_col, const uint16_t *__restrict__ vals,
       const uint16_t *__restrict__ B, int64_t ldb, int N,
       uint16_t *__restrict__ C, int64_t ldc, float *__restrict__ part, int64_t M, int nbx, int slice, int n_swz,
       const int32_t *__restrict__ blk_ofs = nullptr, const void *__restrict__ masks = nullptr)
{
    constexpr int NC = NT * 16;   // columns per pass
    constexpr int LPR = NC / 8;   // lanes that share one gathered row (16 bytes each)
    constexpr int RPI = 64 / LPR; // rows per wave-wide load
    constexpr int NLD = 32 / RPI; // wave-wide loads per 32-vector block
    constexpr int RS = NC * 2;    // LDS row stride in bytes
    // With at least 16 lanes per gathered row, every group of 16 lanes wants the same column index for a
    // given wave-wide load: lane i of a group then holds the index for load i, and a DPP broadcast hands
    // it out.  Narrower passes keep the indices one per vector and use cross-lane reads.
    constexpr bool DPPR = LPR >= 16;

    constexpr int LDS_BYTES = lds_row<RS>(31) + RS;  // bytes of one wavefront's tile

    __shared__ __attribute__((aligned(16))) unsigned char lds_all[WPB][(LDS_BYTES + 15) / 16 * 16];

    // column pass and group of WPB items of this workgroup
    const int pass = blockIdx.x / nbx;
    const int bx = blockIdx.x - pass * nbx;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int u = fs_launch_turn<WPB>(bx, slice, n_swz);  // the workgroup's first position in the launch order
    const int turn = __builtin_amdgcn_readfirstlane(u + wave);  // wave-uniform
    if (turn >= n_items) return;  // no block-wide barrier is used below
    unsigned char *lds = lds_all[wave];

    const int4 it = items[turn];  // the work list in launch order, costliest items first  // {first block slot, blocks, first partial slot, first vector}
    const int nblk = it.y;
    if (nblk == 0) return;
    int slot = it.z;
    const int n0 = pass * NC;  // first column of this pass
    const int j = lane & 15, g = lane >> 4;

    // descriptors of the item's blocks (at most 64), one per lane, and the column indices of its first
    // 64 vectors (an item's vectors are consecutive): both only need the item record
    const int4 my_desc = blk_desc[it.x + min(lane, nblk - 1)];
    const int cols64 = vec_col[max(min(it.w + (DPPR ? (lane & 15) * RPI + lane / LPR : lane), nvec - 1), 0)];
    auto block = [&](int i) -> BlockDesc { return fs_item_block(my_desc, i, nblk); };

    fs_f4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; t++) acc[t] = fs_f4{0.f, 0.f, 0.f, 0.f};

    // per-lane constants of the gather and of the transposed read
    const int g_row = lane / LPR;                         // row within one wave-wide load
    const int g_col = n0 + (lane % LPR) * 8;              // first column of this lane's 16 bytes
    const uint32_t g_colb = (g_col < N ? g_col : 0) * 2;  // its byte offset; lanes past N read (never store) column 0
    const unsigned char *Bb = reinterpret_cast<const unsigned char *>(B);
    const uint32_t ldb2 = (uint32_t)ldb * 2;              // bytes between rows of B
    const bool full_pass = n0 + NC <= N;                  // no column of this pass lies past N
    const int e = (lane & 15) >> 2, q = lane & 3;
    // fp32 partial tiles are stored 16-column tile after 16-column tile, each as (4-column group g, row j,
    // 4 columns): the V*4 lanes that hold a column tile write V*64 contiguous bytes per store
    const uint32_t p_lane = (uint32_t)((n0 / 16) * (V * 16) + (g * V + j) * 4) * 4;
    unsigned char *lds_wr = lds + lds_row<RS>(g_row) + (lane % LPR) * 16;    // + lds_row(l*RPI) per load
    const unsigned char *lds_rd = lds + lds_row<RS>(8 * g + e) + 8 * q;      // + lds_row(4h) + 32t per read

    // Column indices of a block, one per lane.  Lanes past its width repeat its last vector: the sparse
    // operand is zero there, so the rows they make the gather re-read are ignored by the product and no
    // lane has to be masked off.  (The block slot of an empty window reads some valid index.)
    auto load_cols = [&](const BlockDesc &d) -> int {
        const int v = DPPR ? (lane & 15) * RPI + lane / LPR : lane;  // the vector whose index this lane holds
        return vec_col[max(min(d.s + min(v, d.kb - 1), nvec - 1), 0)];
    };
    // 16 bytes of the block's values per lane.  Full block (row stride 32): lane (j, g) gets its operand
    // directly, vectors 8g..8g+7 of row j.  Narrow last block of a window (row stride kb < 32): the
    // V*kb values are contiguous, lane l takes elements 8l..8l+7; they are re-laid through LDS at use.
    auto load_vals = [&](const BlockDesc &d) -> fs_u4 {
        fs_u4 raw = fs_u4{0u, 0u, 0u, 0u};
        const uint16_t *blk = vals + (int64_t)V * d.s;
        if constexpr (V % 8 == 0) {
            // V * kb is a multiple of eight: every lane loads (lanes with nothing to fetch re-read a valid
            // piece and drop it), so that the step issues the same number of loads on every path and the
            // compiler can count what is still in flight instead of waiting for all of it
            const bool full = d.kb == 32;
            const int pieces = V * d.kb / 8;  // 16-byte pieces of a narrow block
            const bool mine = full ? j < V : lane < pieces;
            const int at = full ? (j & (V - 1)) * 32 + 8 * g : 8 * min(lane, max(pieces - 1, 0));
            // (a block without vectors may sit at the very end of a caller's value array: read the index
            // array's first bytes instead, which always exist)
            const uint16_t *src = d.kb > 0 ? blk + at : reinterpret_cast<const uint16_t *>(vec_col);
            const fs_u4 got = *reinterpret_cast<const fs_u4 *>(src);
            raw = (mine && d.kb > 0) ? got : raw;
        } else if (d.kb == 32) {
            if (j < V) raw = *reinterpret_cast<const fs_u4 *>(blk + j * 32 + 8 * g);
        } else if (lane * 8 + 8 <= V * d.kb) {
            raw = *reinterpret_cast<const fs_u4 *>(blk + 8 * lane);
        } else if (V == 4 && lane * 8 < V * d.kb) {  // V = 4, odd width: the last piece holds four values
            const uint2 half = *reinterpret_cast<const uint2 *>(blk + 8 * lane);
            raw.x = half.x;
            raw.y = half.y;
        }
        return raw;
    };
    // Packed values: the masks of a block (one per lane, zero past its width), and from them the lane's
    // eight occupancy bits and the address of its first stored value: the block's first value, plus the
    // stored entries of the rows above j, plus those of row j in the vectors before 8g.
    int my_ofs = 0;
    if constexpr (PK) my_ofs = blk_ofs[it.x + min(lane, nblk - 1)];
    auto load_mask = [&](const BlockDesc &d) -> uint32_t {
        const int v = max(min(d.s + min(lane, d.kb - 1), nvec - 1), 0);
        const uint32_t m = V <= 8 ? (uint32_t) reinterpret_cast<const uint8_t *>(masks)[v]
                                  : (uint32_t) reinterpret_cast<const uint16_t *>(masks)[v];
        return lane < d.kb ? m : 0u;
    };
    auto locate = [&](uint32_t msk, int i, uint32_t &m8) -> const uint16_t * {
        uint32_t mine = 0;
        int above = 0;
#pragma unroll
        for (int r = 0; r < V; r++) {
            const uint32_t has = (uint32_t)__ballot((msk >> r) & 1u);
            mine = (j == r) ? has : mine;
            above += (j > r) ? __popc(has) : 0;
        }
        m8 = (mine >> (8 * g)) & 0xFFu;
        const int before = __popc(mine & ((1u << (8 * g)) - 1u));
        return vals + __builtin_amdgcn_readlane(my_ofs, min(i, nblk - 1)) + above + before;
    };
    // Rows of B this lane gathers for a block, one per wave-wide load, from the block's column indices.
    // Kept as 32-bit byte offsets from B (row * ldb2 + column bytes, a 24-bit multiply) unless B is huge.
    uint32_t grow[NLD];
#define FS_ROWS(cols)                                                                            \
    {                                                                                            \
        if constexpr (DPPR) {                                                                    \
            fs_for_each_index([&](auto l_) {                                                     \
                constexpr int l = decltype(l_)::value;                                           \
                const int idx_ = fs_row_bcast<l>(cols);                                          \
                grow[l] = BIG ? (uint32_t)idx_ : __umul24((uint32_t)idx_, ldb2) + g_colb;        \
            }, std::make_integer_sequence<int, NLD>{});                                          \
        } else {                                                                                 \
            _Pragma("unroll") for (int l = 0; l < NLD; l++) {                                    \
                const int idx_ = __shfl(cols, l * RPI + g_row, 64);                              \
                grow[l] = BIG ? (uint32_t)idx_ : __umul24((uint32_t)idx_, ldb2) + g_colb;        \
            }                                                                                    \
        }                                                                                        \
    }
    fs_u4 stage[NLD];
#define FS_GATHER()                                                                              \
    _Pragma("unroll") for (int l = 0; l < NLD; l++)                                              \
        stage[l] = *reinterpret_cast<const fs_u4 *>(                                             \
            Bb + (BIG ? (uint64_t)grow[l] * ldb2 + g_colb : (uint64_t)grow[l]));

    // Software pipeline.  While block i is multiplied, the gather and the values of block i+1 are in
    // flight; their row numbers were worked out a step earlier (from indices loaded two steps earlier),
    // so the gather is issued the moment block i's rows have left the staging registers.
    BlockDesc d0 = block(0), d1 = block(1), d2 = block(2);
    // Block 0 starts at the item's first vector, so its indices only need the item record; lanes past its
    // width take the index of its last vector, like load_cols.
    int col0, col1;
    if constexpr (DPPR) {
        const int last = max(d0.kb - 1, 0);
        const int at_last = __shfl(cols64, (last % RPI) * LPR + last / RPI, 64);
        col0 = ((lane & 15) * RPI + lane / LPR < d0.kb) ? cols64 : at_last;
        col1 = load_cols(d1);
    } else {
        col0 = __shfl(cols64, min(lane, max(d0.kb - 1, 0)), 64);
        col1 = __shfl(cols64, d0.kb + min(lane, max(d1.kb - 1, 0)), 64);  // block 1 starts right after block 0
    }
    int col2 = load_cols(d2);
    fs_u4 raw0;
    uint32_t m8_0 = 0, msk1 = 0;
    if constexpr (PK) {
        const uint32_t msk0 = load_mask(d0);
        msk1 = load_mask(d1);
        raw0 = *reinterpret_cast<const fs_u4_unaligned *>(locate(msk0, 0, m8_0));
    } else {
        raw0 = load_vals(d0);
    }
    bool from_first = d0.first;  // the current window's first block lies inside this item
    FS_ROWS(col0)
    FS_GATHER()
    FS_ROWS(col1)

    // One block step.  MORE: another block of the item follows (its gather is issued here).  The last step
    // is a second instance of the same code, so that inside the loop every path issues the same loads and
    // the compiler can wait for exactly the ones it needs: loads return in the order they were issued, and a
    // wait that cannot tell would also wait for the stores of a window just flushed.
    int step = 0;
    auto block_step = [&](auto more_) {
        constexpr bool MORE = decltype(more_)::value;
        const int kb = d0.kb;
        // sparse operand: rows j < V of the block, vectors 8g .. 8g+7; vectors past kb are zero
        fs_frag sp;
        sp.u = PK ? fs_expand8(raw0, m8_0) : raw0;
        if (!PK && kb > 0 && kb < 32) {
            *reinterpret_cast<fs_u4 *>(lds + 16 * lane) = raw0;  // V*kb*2 <= 1 KB of contiguous values
            FS_WAVE_SYNC();
            // element (j, 8g + x) sits at j*kb + 8g + x; reads past the row's end stay inside the staged
            // values (or the 16 bytes after them) and are cleared by the mask of valid positions
            const uint16_t *lv = reinterpret_cast<const uint16_t *>(lds) + (j < V ? j : 0) * kb + 8 * g;
            const int nv = j < V ? min(max(kb - 8 * g, 0), 8) : 0;  // valid elements of this lane
            sp.u = *reinterpret_cast<const fs_u4_unaligned *>(lv);  // one ds_read_b128 at a 2-byte-aligned address
            const uint64_t lo = nv >= 4 ? ~0ull : ((1ull << (16 * nv)) - 1);
            const uint64_t hi = nv >= 8 ? ~0ull : (nv <= 4 ? 0ull : ((1ull << (16 * (nv - 4))) - 1));
            sp.u.x &= (uint32_t)lo; sp.u.y &= (uint32_t)(lo >> 32);
            sp.u.z &= (uint32_t)hi; sp.u.w &= (uint32_t)(hi >> 32);
            FS_WAVE_SYNC();
        }
        // Queue the small loads ahead first -- the indices three blocks ahead and the next block's values.
        // They are copied to their places when the step ends; issued after the gather, that copy would wait
        // for the whole gather (and for whatever was stored since).
        const BlockDesc d3 = block(step + 3);
        const int col3 = load_cols(d3);
        fs_u4 raw1;
        uint32_t m8_1 = 0, msk2 = 0;
        if constexpr (PK) {
            raw1 = *reinterpret_cast<const fs_u4_unaligned *>(locate(msk1, step + 1, m8_1));
            msk2 = load_mask(d2);
        } else {
            raw1 = load_vals(d1);
        }
        if (kb > 0) {
            // the gathered rows go to LDS (this is where the wave waits for the gather)
#pragma unroll
            for (int l = 0; l < NLD; l++)
                *reinterpret_cast<fs_u4 *>(lds_wr + lds_row<RS>(l * RPI)) = stage[l];
        }
        // the gather of the next block, the moment this block's rows have left the staging registers
        if constexpr (MORE) FS_GATHER()
        FS_WAVE_SYNC();

        if (kb > 0) {
            // transposed reads + matrix-core products, one per 16-column tile
#pragma unroll
            for (int t = 0; t < NT; t++) {
                fs_frag dn;
#pragma unroll
                for (int h = 0; h < 2; h++)
                    dn.s[h] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (fs_s4 __attribute__((address_space(3))) *)(lds_rd + lds_row<RS>(4 * h) + 32 * t));
                acc[t] = fs_mfma_16x16x32<DT>(dn, sp, acc[t]);
            }
            FS_WAVE_SYNC();
        }
        // row numbers of the gather after next (its indices arrived during the previous step)
        FS_ROWS(col2)

        if (d0.last || !MORE) {
            // flush: lane (j, g) holds C[w*V + j][n0 + 16t + 4g .. +3].  A window that lies whole inside
            // the item goes to C (zeros for an empty window); a part of a window goes to an fp32
            // partial tile.  Addresses are a wave-uniform base plus a per-lane 32-bit offset that was
            // worked out once, plus an immediate per tile.
            const bool whole = d0.last && from_first;
            if (whole) {
                fs_round_tile_to_lds<DT, V, NT, RS>(lds, acc, j, g, 1.f);
                FS_WAVE_SYNC();
                fs_store_tile_rows<V, RPI, RS>(lds_wr, C, ldc, d0.w, M, N, g_row, g_col);
                FS_WAVE_SYNC();
            } else {
                fs_store_partial_tile<V, NT>(part, slot, N, p_lane, acc, j < V && (int64_t)d0.w * V + j < M, full_pass, n0, g);
            }
            if (!whole) slot++;
#pragma unroll
            for (int t = 0; t < NT; t++) acc[t] = fs_f4{0.f, 0.f, 0.f, 0.f};
        }
        if (d0.last) from_first = true;  // the next block opens a window
        d0 = d1; d1 = d2; d2 = d3;
        col2 = col3;
        raw0 = raw1;
        m8_0 = m8_1;
        msk1 = msk2;
    };
    for (; step + 1 < nblk; step++) block_step(std::true_type{});
    block_step(std::false_type{});
#undef FS_GATHER
#undef FS_ROWS
}

// Adds the partial tiles of one cut window in slot order and stores the rounded rows of C.  A tile is
// read in its storage order (16-column tile, 4-column group, row), so the loads are contiguous; the
// rounded values pass through LDS so that the stores are contiguous 16-byte pieces of rows of C.
template <int DT, int V>
__global__ void __launch_bounds__(64)
k_spmm_reduce(const int4 *__restrict__ split_windows, const float *__restrict__ part, int N,
              uint16_t *__restrict__ C, int64_t ldc, int64_t M)
{
    constexpr int CH = 32;  // columns per workgroup: many small workgroups, so that a hub
                            // window with dozens of parts is not one long-running workgroup
    __shared__ __attribute__((aligned(16))) uint16_t out_t[V][CH + 8];
    const int n_chunks = (N + CH - 1) / CH;
    const int4 sw = split_windows[blockIdx.x / n_chunks];
    const int w = sw.x, p0 = sw.y, cnt = sw.z;
    const int64_t tile4 = (int64_t)V * N / 4;  // float4 per partial tile
    const fs_f4 *base = reinterpret_cast<const fs_f4 *>(part) + (int64_t)p0 * tile4;
    {
        const int c0 = (blockIdx.x % n_chunks) * CH;
        const int nc = min(CH, N - c0);  // columns of this workgroup, a multiple of 8
        const fs_f4 *src0 = base + (c0 / 4) * V;
        for (int idx = threadIdx.x; idx < (nc / 4) * V; idx += 64) {
            const fs_f4 *src = src0 + idx;
            fs_f4 sum = fs_f4{0.f, 0.f, 0.f, 0.f};
            int k = 0;
            for (; k + 32 <= cnt; k += 32) {  // thirty-two loads in flight, added in slot order
                fs_f4 v[32];
#pragma unroll
                for (int u = 0; u < 32; u++) v[u] = src[(int64_t)(k + u) * tile4];
#pragma unroll
                for (int u = 0; u < 32; u++) sum += v[u];
            }
            if (k + 16 <= cnt) {
                fs_f4 v[16];
#pragma unroll
                for (int u = 0; u < 16; u++) v[u] = src[(int64_t)(k + u) * tile4];
#pragma unroll
                for (int u = 0; u < 16; u++) sum += v[u];
                k += 16;
            }
            if (k + 8 <= cnt) {
                fs_f4 v[8];
#pragma unroll
                for (int u = 0; u < 8; u++) v[u] = src[(int64_t)(k + u) * tile4];
#pragma unroll
                for (int u = 0; u < 8; u++) sum += v[u];
                k += 8;
            }
            if (k < cnt) {  // up to seven left: loads together, added in slot order
                fs_f4 v[7];
#pragma unroll
                for (int u = 0; u < 7; u++) v[u] = src[(int64_t)min(k + u, cnt - 1) * tile4];
#pragma unroll
                for (int u = 0; u < 7; u++)
                    if (k + u < cnt) sum += v[u];
            }
            const int ct = idx / (4 * V), rem = idx - ct * 4 * V, g = rem / V, j = rem - g * V;
            uint2 o;
            o.x = fs_pack2<DT>(sum[0], sum[1]);
            o.y = fs_pack2<DT>(sum[2], sum[3]);
            *reinterpret_cast<uint2 *>(&out_t[j][16 * ct + 4 * g]) = o;
        }
        __syncthreads();
        const int c8n = nc / 8;
        for (int t = threadIdx.x; t < V * c8n; t += 64) {
            const int j = t / c8n, c8 = t - j * c8n;
            const int64_t row = (int64_t)w * V + j;
            if (row < M)
                __builtin_nontemporal_store(*reinterpret_cast<const fs_u4 *>(&out_t[j][8 * c8]),
                                            reinterpret_cast<fs_u4 *>(C + row * ldc + c0 + 8 * c8));
        }
    }
}

// Columns per pass for N > 64: 128.  (With the work list in its own order, 64-column passes -- more, lighter
// wavefronts per CU -- measured 11 % faster on large matrices; with parts of hub windows launched by column
// the order reverses, cfg 4 at eight rows: 733 us against 779 us.)  A tuning build (-DFS_TUNING_ENV) lets
// FS_SPMM_PASS=64|128 override the choice; the shipped library reads no environment.
int fs_spmm_pass_override()
{
#ifdef FS_TUNING_ENV
    const char *e = getenv("FS_SPMM_PASS");
    return e ? atoi(e) : 0;
#else
    return 0;
#endif
}

template <int DT, int V>
fs_status launch(const fs_format *f, const uint16_t *vals, const uint16_t *B, int64_t N, int64_t ldb, uint16_t *C,
                 int64_t ldc, float *part, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1, const int32_t *blk_ofs = nullptr,
                 const void *masks = nullptr)
{
    if (f->n_items == 0) return FS_OK;
    const int4 *items = (const int4 *)f->items_by_cost;
    const int n_items = (int)f->n_items;
    int nc = N <= 32 ? 32 : N <= 64 ? 64 : 128;  // columns per pass
    if (blk_ofs && nc == 32) nc = 64;  // the packed-value kernels exist for 64- and 128-column passes
    if (N > 64 && (fs_spmm_pass_override() == 64 || fs_spmm_pass_override() == 128)) nc = fs_spmm_pass_override();
    // Wavefronts (= work items) per workgroup.  A workgroup keeps its slots until its slowest wavefront is
    // done, so small launches, whose tail is a large part of the run, do best with one item per workgroup
    // (cfg 2: 25.1 -> 23.7 us); 64-column passes measured best with two, wide passes on large matrices with four.
    const int wpb = nc == 32 ? 4 : nc == 64 ? 2 : (n_items < 16384 ? 1 : 4);
    int slice_len = 4096;  // launch positions per slice
#ifdef FS_TUNING_ENV
    if (const char *e = getenv("FS_SPMM_SLICE")) slice_len = atoi(e);
#endif
    const fs_launch_geometry geo = fs_launch_geometry_for(f, wpb, slice_len);
    const int nbx = geo.nbx, slice = geo.slice, n_swz = geo.n_swz;
    const int passes = (int)((N + nc - 1) / nc);
    const int64_t nblocks = (int64_t)nbx * passes;
    if (nblocks >= ((int64_t)1 << 31)) return FS_ERR_TOO_LARGE;
    dim3 grid((unsigned)nblocks, 1, 1), block(64 * wpb, 1, 1);
    if (ev0) FS_HIP(hipEventRecord(ev0, st));
    // 32-bit gather offsets need B to span less than 4 GiB and row number and row pitch to fit 24 bits
    const bool big = f->K >= ((int64_t)1 << 24) || ldb * 2 >= ((int64_t)1 << 24) ||
                     f->K * ldb * 2 >= ((int64_t)1 << 32);
#define FS_SPMM_ARGS items, n_items, (const int4 *)f->blk_desc, (int)f->nvec, f->vec_col, vals, B, ldb, (int)N, C, ldc, part, f->M, nbx, slice, n_swz
#define FS_SPMM_GO(NT_, WPB_)                                                              \
    if (big) k_spmm<DT, V, NT_, WPB_, true><<<grid, block, 0, st>>>(FS_SPMM_ARGS);        \
    else k_spmm<DT, V, NT_, WPB_, false><<<grid, block, 0, st>>>(FS_SPMM_ARGS)
    if (blk_ofs) {
        if (big) return FS_ERR_UNSUPPORTED;
        if (nc == 64) k_spmm<DT, V, 4, 2, false, true><<<grid, block, 0, st>>>(FS_SPMM_ARGS, blk_ofs, masks);
        else if (wpb == 1) k_spmm<DT, V, 8, 1, false, true><<<grid, block, 0, st>>>(FS_SPMM_ARGS, blk_ofs, masks);
        else k_spmm<DT, V, 8, 4, false, true><<<grid, block, 0, st>>>(FS_SPMM_ARGS, blk_ofs, masks);
    }
    else if (nc == 32) { FS_SPMM_GO(2, 4); }
    else if (nc == 64) { FS_SPMM_GO(4, 2); }
    else if (wpb == 1) { FS_SPMM_GO(8, 1); }
    else { FS_SPMM_GO(8, 4); }
#undef FS_SPMM_GO
#undef FS_SPMM_ARGS
    FS_LAUNCH_CHECK();
    if (ev1) FS_HIP(hipEventRecord(ev1, st));
    if (f->n_split_windows > 0) {
        const int64_t rblocks = f->n_split_windows * ((N + 31) / 32);  // one workgroup per window and 32 columns
        if (rblocks >= ((int64_t)1 << 31)) return FS_ERR_TOO_LARGE;
        k_spmm_reduce<DT, V><<<(unsigned)rblocks, 64, 0, st>>>((const int4 *)f->split_windows, part, (int)N, C, ldc, f->M);
        FS_LAUNCH_CHECK();
    }
    return FS_OK;
}

}  // namespace

fs_status fs_spmm_packed_launch(const fs_format *f, const void *d_packed, const void *d_B, int64_t N, int64_t ldb,
                                void *d_C, int64_t ldc, void *d_work, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1)
{
    const fs_packed_plan_t pl = fs_packed_plan(f);
    const unsigned char *buf = (const unsigned char *)d_packed;
    const int32_t *blk_ofs = (const int32_t *)(buf + pl.ofs);
    const uint16_t *vals = (const uint16_t *)(buf + pl.vals);
    const void *masks = buf + pl.masks;
    const uint16_t *B = (const uint16_t *)d_B;
    uint16_t *C = (uint16_t *)d_C;
    float *part = (float *)d_work;
    if (f->dtype == FS_F16) {
        if (f->V == 4) return launch<FS_F16, 4>(f, vals, B, N, ldb, C, ldc, part, st, ev0, ev1, blk_ofs, masks);
        if (f->V == 8) return launch<FS_F16, 8>(f, vals, B, N, ldb, C, ldc, part, st, ev0, ev1, blk_ofs, masks);
        if (f->V == 16) return launch<FS_F16, 16>(f, vals, B, N, ldb, C, ldc, part, st, ev0, ev1, blk_ofs, masks);
    } else if (f->dtype == FS_BF16) {
        if (f->V == 4) return launch<FS_BF16, 4>(f, vals, B, N, ldb, C, ldc, part, st, ev0, ev1, blk_ofs, masks);
        if (f->V == 8) return launch<FS_BF16, 8>(f, vals, B, N, ldb, C, ldc, part, st, ev0, ev1, blk_ofs, masks);
        if (f->V == 16) return launch<FS_BF16, 16>(f, vals, B, N, ldb, C, ldc, part, st, ev0, ev1, blk_ofs, masks);
    }
    return FS_ERR_UNSUPPORTED;
}

fs_status fs_spmm_launch(const fs_format *f, const void *d_vals, const void *d_B, int64_t N, int64_t ldb, void *d_C,
                         int64_t ldc, void *d_work, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1)
{
    // the format's own values, packed by the conversion: the lighter stream (same operands, same result)
    if (!d_vals && f->packed && f->K < ((int64_t)1 << 24) && ldb * 2 < ((int64_t)1 << 24) && f->K * ldb * 2 < ((int64_t)1 << 32))
        return fs_spmm_packed_launch(f, f->packed, d_B, N, ldb, d_C, ldc, d_work, st, ev0, ev1);
    const uint16_t *vals = (const uint16_t *)(d_vals ? d_vals : f->vals_blk);
    const uint16_t *B = (const uint16_t *)d_B;
    uint16_t *C = (uint16_t *)d_C;
    float *part = (float *)d_work;
    if (f->dtype == FS_F16) {
        if (f->V == 4) return launch<FS_F16, 4>(f, vals, B, N, ldb, C, ldc, part, st, ev0, ev1);
        if (f->V == 8) return launch<FS_F16, 8>(f, vals, B, N, ldb, C, ldc, part, st, ev0, ev1);
        if (f->V == 16) return launch<FS_F16, 16>(f, vals, B, N, ldb, C, ldc, part, st, ev0, ev1);
    } else if (f->dtype == FS_BF16) {
        if (f->V == 4) return launch<FS_BF16, 4>(f, vals, B, N, ldb, C, ldc, part, st, ev0, ev1);
        if (f->V == 8) return launch<FS_BF16, 8>(f, vals, B, N, ldb, C, ldc, part, st, ev0, ev1);
        if (f->V == 16) return launch<FS_BF16, 16>(f, vals, B, N, ldb, C, ldc, part, st, ev0, ev1);
    }
    return FS_ERR_UNSUPPORTED;
}
