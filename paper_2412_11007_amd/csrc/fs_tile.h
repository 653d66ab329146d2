// Device pieces shared by the kernels that walk work items block by block and gather rows of a dense
// operand through LDS onto the matrix cores (SpMM, the fused attention kernel): the layout of the staged
// tile, block descriptors, the index hand-out, the launch-order turn of a wavefront and the flush of an
// accumulator tile.  Every translation unit gets its own copy.
#pragma once

#include <algorithm>
#include <utility>

#include "fs_common.h"

namespace {

// Byte offset of row r of the staged tile in LDS.  Rows are RS + 32 bytes apart and every group of eight
// rows is pushed another 128 bytes, so that the eight rows one half-wave touches in a transposed read
// (r, r+1, r+2, r+3 and the same four plus 8) start in eight different groups of eight banks; the offset
// of a tile or of a wave-wide load inside a row is then a plain immediate.
template <int RS>
__device__ __forceinline__ constexpr int lds_row(int r)
{
    return r * (RS + 32) + (r >> 3) * 128;
}

// Orders a wavefront's LDS writes before its following LDS reads (and the other way round): no block-wide
// barrier, the tile belongs to one wavefront.
#define FS_WAVE_SYNC()                                              \
    do {                                                            \
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");      \
        __builtin_amdgcn_wave_barrier();                            \
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");      \
    } while (0)

// One 32-vector block of an item (all fields are wave-uniform).
struct BlockDesc {
    int s;       // first vector
    int kb;      // vectors in the block, 0..32 (0: the block slot of an empty window)
    int w;       // window
    bool last;   // last block of its window
    bool first;  // first block of its window
};

// The i-th block of an item whose descriptors (at most 64) sit one per lane in my_desc; blocks past the
// item's end are empty.
__device__ __forceinline__ BlockDesc fs_item_block(const int4 &my_desc, int i, int nblk)
{
    BlockDesc d;
    const int ic = min(i, nblk - 1);
    const int kf = __builtin_amdgcn_readlane(my_desc.y, ic);
    d.s = __builtin_amdgcn_readlane(my_desc.x, ic);
    d.w = __builtin_amdgcn_readlane(my_desc.z, ic);
    d.kb = i < nblk ? (kf & 255) : 0;
    d.last = i < nblk && (kf & 256);
    d.first = (kf & 512) != 0;
    return d;
}

// Lane L of every group of 16 lanes, broadcast to the whole group (a DPP move: no LDS-pipeline traffic).
template <int L>
__device__ __forceinline__ int fs_row_bcast(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, 0x150 + L, 0xF, 0xF, false);  // row_newbcast:L
}
template <typename F, int... Ls>
__device__ __forceinline__ void fs_for_each_index(F &&f, std::integer_sequence<int, Ls...>)
{
    (f(std::integral_constant<int, Ls>{}), ...);
}

// Which position of the launch order the first wavefront of workgroup bx takes.  The first n_swz positions
// hold the parts of cut windows, ordered by column.  Workgroups go to the eight XCDs (each with an L2 of
// its own) round robin, so inside every slice of `slice` such positions -- about what the chip holds at
// once -- XCD x takes the x-th eighth, a contiguous run: parts of different hub windows that sweep the same
// columns meet in one L2.  n_swz and slice are multiples of 8 * WPB, the workgroups per pass of 8.
template <int WPB>
__device__ __forceinline__ int fs_launch_turn(int bx, int slice, int n_swz)
{
    int u = bx * WPB;
    if (u < n_swz) {
        const int s0 = u / slice * slice;               // first position of the slice
        const int q = min(slice, n_swz - s0) / WPB / 8;  // workgroups per XCD in this slice
        const int g = (u - s0) / WPB;
        u = s0 + ((g & 7) * q + (g >> 3)) * WPB;
    }
    return u;
}

// Host side of the same: workgroups per pass, slice length and swizzled prefix for wpb items per workgroup.
struct fs_launch_geometry {
    int nbx, slice, n_swz;
};
inline fs_launch_geometry fs_launch_geometry_for(const fs_format *f, int wpb, int slice = 4096)
{
    fs_launch_geometry g;
    g.nbx = (int)((((int64_t)f->n_items + wpb - 1) / wpb + 7) / 8 * 8);
    g.slice = slice / 32 * 32;  // a multiple of 8 * wpb for wpb = 1, 2, 4
    g.n_swz = g.slice > 0 ? (int)(std::min<int64_t>(f->n_cut_items, f->n_items) / (8 * wpb) * (8 * wpb)) : 0;
    return g;
}

// Accumulators -> rounded V x NC tile, row-major in the wavefront's LDS tile (the gathered rows in it have
// been consumed).  Lane (j, g) holds C[w*V + j][n0 + 16t + 4g .. +3] in acc[t]; `scale` multiplies on the way.
template <int DT, int V, int NT, int RS>
__device__ __forceinline__ void fs_round_tile_to_lds(unsigned char *lds, const fs_f4 (&acc)[NT], int j, int g, float scale)
{
    if (j < V) {
#pragma unroll
        for (int t = 0; t < NT; t++) {
            uint2 o;
            o.x = fs_pack2<DT>(acc[t][0] * scale, acc[t][1] * scale);
            o.y = fs_pack2<DT>(acc[t][2] * scale, acc[t][3] * scale);
            *reinterpret_cast<uint2 *>(lds + lds_row<RS>(j) + 32 * t + 8 * g) = o;
        }
    }
}

// The rounded tile in LDS -> rows of C, with the lane-to-row mapping of the gather: adjacent lanes write
// one row contiguously, 16 bytes each, non-temporal (C is never read back; without the hint its lines push
// rows of the dense operand out of L2).  Storing the accumulators straight from the matrix-core layout
// (8-byte pieces scattered over V rows) measured far slower.
template <int V, int RPI, int RS>
__device__ __forceinline__ void fs_store_tile_rows(const unsigned char *lds_wr, uint16_t *C, int64_t ldc, int w, int64_t M, int N,
                                                   int g_row, int g_col)
{
    const bool rows_ok = (int64_t)(w + 1) * V <= M;  // false only for a window cut by the matrix edge
    unsigned char *Cw = reinterpret_cast<unsigned char *>(C) + (int64_t)w * V * ldc * 2;
#pragma unroll
    for (int l = 0; l < (V + RPI - 1) / RPI; l++) {
        const int r = l * RPI + g_row;
        if (r < V && (rows_ok || (int64_t)w * V + r < M) && g_col < N)
            __builtin_nontemporal_store(*reinterpret_cast<const fs_u4 *>(lds_wr + lds_row<RS>(l * RPI)),
                                        reinterpret_cast<fs_u4 *>(Cw + (uint32_t)(r * (uint32_t)ldc + g_col) * 2));
    }
}

// A part of a cut window: the fp32 accumulators go to partial tile `slot` of the workspace, in register
// order (16-column tile, 4-column group, row): the V*4 lanes that hold a column tile write V*64 contiguous
// bytes per store.  p_lane = ((n0 / 16) * (V * 16) + (g * V + j) * 4) * 4 is the lane's byte offset.
template <int V, int NT>
__device__ __forceinline__ void fs_store_partial_tile(float *part, int slot, int N, uint32_t p_lane, const fs_f4 (&acc)[NT],
                                                      bool rows_live, bool full_pass, int n0, int g)
{
    unsigned char *Pw = reinterpret_cast<unsigned char *>(part) + (int64_t)slot * V * N * 4 + p_lane;
    if (rows_live) {
        if (full_pass) {
#pragma unroll
            for (int t = 0; t < NT; t++) *reinterpret_cast<fs_f4 *>(Pw + V * 64 * t) = acc[t];
        } else {
#pragma unroll
            for (int t = 0; t < NT; t++) {
                if (n0 + 16 * t + 4 * g < N) *reinterpret_cast<fs_f4 *>(Pw + V * 64 * t) = acc[t];
            }
        }
    }
}

}  // namespace
