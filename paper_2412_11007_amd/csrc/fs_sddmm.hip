// SDDMM on the CDNA4 matrix cores over the row-window format (paper Section 3.4).
//
// For every block of up to 32 nonzero vectors of a window the kernel computes
// the V x 32 tile  X[window rows, :] * Y[vector columns, :]^T  and writes it,
// masked by the sparsity pattern, straight into the value layout fs_spmm reads
// (the role the paper gives its Algorithm 1).
//
// The contraction runs over the feature dimension d, which is contiguous in
// the rows of both X and Y (the alignment the paper points out at the end of
// Section 3.4), so every lane loads 16 contiguous bytes directly in matrix-core
// operand layout: the operands need no LDS staging.  As in SpMM the operands are swapped
// (Section 3.2): gathered Y rows are the left operand (16 vectors x 32 features),
// the window's X rows the right operand (32 features x 16 rows, rows >= V zero).
// Vector c of a block is placed on row 8*(i/4)+4t+(i%4) -> i of tile t, so that
// after both tiles a lane holds the eight consecutive vectors 8g..8g+7 of one
// window row: exactly 16 contiguous bytes of the row-major value tile.
#include "fs_common.h"

#ifndef FS_SDDMM_WPB
#define FS_SDDMM_WPB 4  // wavefronts (= work items) per workgroup
#endif

namespace {

template <int DT, int V, int KS, int WPB>  // KS = number of 32-feature steps kept in registers for X
__global__ void __launch_bounds__(64 * WPB)
k_sddmm(const int4 *__restrict__ items, int n_items, const int32_t *__restrict__ win_ptr, int W,
        const int32_t *__restrict__ vec_col, const uint32_t *__restrict__ vec_mask,
        const uint16_t *__restrict__ X, int64_t ldx, const uint16_t *__restrict__ Y, int64_t ldy, int d,
        uint16_t *__restrict__ out, int64_t M)
{
    // 1 KB per wave: re-lays the scores of a narrow block before they are stored
    __shared__ __attribute__((aligned(16))) uint16_t lds_all[WPB][512];

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int item = __builtin_amdgcn_readfirstlane(blockIdx.x * WPB + wave);  // wave-uniform
    if (item >= n_items) return;
    const int4 it = items[item];
    const int nblk = it.z;
    if (nblk == 0) return;
    uint16_t *lds = lds_all[wave];
    int w = it.x, b = it.y;
    const int j = lane & 15, g = lane >> 4;
    const int nsteps = (d + 31) / 32;

    int wbase = w;
    int wp_l = win_ptr[min(wbase + lane, W)];
    int ws = __builtin_amdgcn_readlane(wp_l, 0), we = __builtin_amdgcn_readlane(wp_l, 1);

    // X operand of window w: lane (j, g) holds X[w*V + j][32*ks + 8g .. +7]
    fs_frag xf[KS];
    int64_t xrow;
    bool x_ok;
    auto load_x = [&]() {
        xrow = (int64_t)w * V + j;
        x_ok = j < V && xrow < M;
#pragma unroll
        for (int ks = 0; ks < KS; ks++) {
            xf[ks].u = fs_u4{0u, 0u, 0u, 0u};
            const int f0 = 32 * ks + 8 * g;
            if (x_ok && f0 < d) xf[ks].u = *reinterpret_cast<const fs_u4 *>(X + xrow * ldx + f0);
        }
    };
    load_x();

    for (int step = 0; step < nblk; step++) {
        const int s = ws + 32 * b;
        const int kb = min(32, we - s);  // 0 for an empty window
        if (kb > 0) {
            // column and row-occupancy mask of vector s + lane
            const int my_col = (lane < kb) ? vec_col[s + lane] : -1;
            const uint32_t my_mask = (lane < kb) ? vec_mask[s + lane] : 0u;
            fs_f4 acc[2];
#pragma unroll
            for (int t = 0; t < 2; t++) {
                acc[t] = fs_f4{0.f, 0.f, 0.f, 0.f};
                const int c = 8 * (j >> 2) + 4 * t + (j & 3);  // vector of the block on matrix row j of tile t
                const int64_t yrow = __shfl(my_col, c, 64);
                for (int k0 = 0; k0 < nsteps; k0 += KS) {
#pragma unroll
                    for (int ks = 0; ks < KS; ks++) {
                        const int f0 = 32 * (k0 + ks) + 8 * g;
                        fs_frag yf, xx;
                        yf.u = fs_u4{0u, 0u, 0u, 0u};
                        if (yrow >= 0 && f0 < d) yf.u = *reinterpret_cast<const fs_u4 *>(Y + yrow * ldy + f0);
                        if (nsteps <= KS) {
                            xx = xf[ks];
                        } else {
                            xx.u = fs_u4{0u, 0u, 0u, 0u};
                            if (x_ok && f0 < d) xx.u = *reinterpret_cast<const fs_u4 *>(X + xrow * ldx + f0);
                        }
                        acc[t] = fs_mfma_16x16x32<DT>(yf, xx, acc[t]);
                    }
                }
            }
            // lane (j, g): acc[t][e] is the score of window row j and vector 8g + 4t + e
            fs_frag o;
#pragma unroll
            for (int x = 0; x < 8; x++) {
                const uint32_t m = (uint32_t)__shfl((int)my_mask, 8 * g + x, 64);
                o.e[x] = ((m >> j) & 1u) ? fs_round_bits<DT>(acc[x >> 2][x & 3]) : (uint16_t)0;
            }
            uint16_t *blk = out + (int64_t)V * s;
            if (kb == 32) {
                if (j < V) *reinterpret_cast<fs_u4 *>(blk + j * 32 + 8 * g) = o.u;
            } else {
                // narrow last block of the window (row stride kb): gather the V x kb tile in LDS,
                // then store its V*kb contiguous values 16 bytes per lane
                if (j < V) {
#pragma unroll
                    for (int x = 0; x < 8; x++) {
                        const int c = 8 * g + x;
                        if (c < kb) lds[j * kb + c] = o.e[x];
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                if (lane * 8 < V * kb)
                    *reinterpret_cast<fs_u4 *>(blk + 8 * lane) = *reinterpret_cast<const fs_u4 *>(lds + 8 * lane);
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
        }
        if (s + 32 >= we) {  // last block of the window: move on to the next one
            w++;
            b = 0;
            int rel = w - wbase;
            if (rel >= 63) {
                wbase = w;
                wp_l = win_ptr[min(wbase + lane, W)];
                rel = 0;
            }
            ws = __builtin_amdgcn_readlane(wp_l, rel);
            we = __builtin_amdgcn_readlane(wp_l, rel + 1);
            if (step + 1 < nblk) load_x();
        } else {
            b++;
        }
    }
}

template <int DT, int V>
fs_status launch(const fs_format *f, const uint16_t *X, int64_t ldx, const uint16_t *Y, int64_t ldy, int64_t d,
                 uint16_t *out, hipStream_t st)
{
    if (f->n_items == 0) return FS_OK;
    const int4 *items = (const int4 *)f->items;
    const int n_items = (int)f->n_items;
    constexpr int WPB = FS_SDDMM_WPB;
    dim3 grid((unsigned)((n_items + WPB - 1) / WPB)), block(64 * WPB);
    const int W = (int)f->W;
    if (d <= 32)
        k_sddmm<DT, V, 1, WPB><<<grid, block, 0, st>>>(items, n_items, f->win_ptr, W, f->vec_col, f->vec_mask, X, ldx, Y, ldy, (int)d, out, f->M);
    else if (d <= 64)
        k_sddmm<DT, V, 2, WPB><<<grid, block, 0, st>>>(items, n_items, f->win_ptr, W, f->vec_col, f->vec_mask, X, ldx, Y, ldy, (int)d, out, f->M);
    else
        k_sddmm<DT, V, 4, WPB><<<grid, block, 0, st>>>(items, n_items, f->win_ptr, W, f->vec_col, f->vec_mask, X, ldx, Y, ldy, (int)d, out, f->M);
    FS_LAUNCH_CHECK();
    return FS_OK;
}

}  // namespace

fs_status fs_sddmm_launch(const fs_format *f, const void *d_X, int64_t ldx, const void *d_Y, int64_t ldy, int64_t d,
                          void *d_out_blk, hipStream_t st)
{
    const uint16_t *X = (const uint16_t *)d_X, *Y = (const uint16_t *)d_Y;
    uint16_t *out = (uint16_t *)d_out_blk;
    if (f->dtype == FS_F16) {
        if (f->V == 8) return launch<FS_F16, 8>(f, X, ldx, Y, ldy, d, out, st);
        if (f->V == 16) return launch<FS_F16, 16>(f, X, ldx, Y, ldy, d, out, st);
    } else if (f->dtype == FS_BF16) {
        if (f->V == 8) return launch<FS_BF16, 8>(f, X, ldx, Y, ldy, d, out, st);
        if (f->V == 16) return launch<FS_BF16, 16>(f, X, ldx, Y, ldy, d, out, st);
    }
    return FS_ERR_UNSUPPORTED;
}
