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
// operand layout: no LDS, no shuffles.  As in SpMM the operands are swapped
// (Section 3.2): gathered Y rows are the left operand (16 vectors x 32 features),
// the window's X rows the right operand (32 features x 16 rows, rows >= V zero).
// Vector c of a block is placed on row 8*(i/4)+4t+(i%4) -> i of tile t, so that
// after both tiles a lane holds the eight consecutive vectors 8g..8g+7 of one
// window row: exactly 16 contiguous bytes of the row-major value tile.
#include "fs_common.h"

namespace {

template <int DT, int V, int KS>  // KS = number of 32-feature steps kept in registers for X
__global__ void __launch_bounds__(256)
k_sddmm(const int4 *__restrict__ items, int n_items, const int32_t *__restrict__ vec_col,
        const uint32_t *__restrict__ vec_mask, const uint16_t *__restrict__ X, int64_t ldx,
        const uint16_t *__restrict__ Y, int64_t ldy, int d, uint16_t *__restrict__ out, int64_t M)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int item = blockIdx.x * 4 + wave;
    if (item >= n_items) return;
    const int4 it = items[item];
    const int w = it.x, s_begin = it.y, s_end = it.y + it.z;
    const int j = lane & 15, g = lane >> 4;
    const int nsteps = (d + 31) / 32;

    // X operand of the window: lane (j, g) holds X[w*V + j][32*ks + 8g .. +7]
    const int64_t xrow = (int64_t)w * V + j;
    const bool x_ok = j < V && xrow < M;
    fs_frag xf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
        xf[ks].u = make_uint4(0, 0, 0, 0);
        const int f0 = 32 * ks + 8 * g;
        if (x_ok && f0 < d) xf[ks].u = *reinterpret_cast<const uint4 *>(X + xrow * ldx + f0);
    }

    for (int s = s_begin; s < s_end; s += 32) {
        const int kb = min(32, s_end - s);
        fs_f4 acc[2];
#pragma unroll
        for (int t = 0; t < 2; t++) {
            acc[t] = fs_f4{0.f, 0.f, 0.f, 0.f};
            const int c = 8 * (j >> 2) + 4 * t + (j & 3);  // vector of the block on matrix row j of tile t
            const int64_t yrow = (c < kb) ? vec_col[s + c] : -1;
            for (int k0 = 0; k0 < nsteps; k0 += KS) {
#pragma unroll
                for (int ks = 0; ks < KS; ks++) {
                    const int f0 = 32 * (k0 + ks) + 8 * g;
                    fs_frag yf, xx;
                    yf.u = make_uint4(0, 0, 0, 0);
                    if (yrow >= 0 && f0 < d) yf.u = *reinterpret_cast<const uint4 *>(Y + yrow * ldy + f0);
                    if (nsteps <= KS) {
                        xx = xf[ks];
                    } else {
                        xx.u = make_uint4(0, 0, 0, 0);
                        if (x_ok && f0 < d) xx.u = *reinterpret_cast<const uint4 *>(X + xrow * ldx + f0);
                    }
                    acc[t] = fs_mfma_16x16x32<DT>(yf, xx, acc[t]);
                }
            }
        }
        // lane (j, g): acc[t][e] is the score of window row j and vector 8g + 4t + e
        if (j < V) {
            fs_frag o;
#pragma unroll
            for (int x = 0; x < 8; x++) {
                const int c = 8 * g + x;
                uint16_t bits = 0;
                if (c < kb && ((vec_mask[s + c] >> j) & 1u)) bits = fs_round_bits<DT>(acc[x >> 2][x & 3]);
                o.e[x] = bits;
            }
            uint16_t *blk = out + (int64_t)V * s;
            if (kb == 32) {
                *reinterpret_cast<uint4 *>(blk + j * 32 + 8 * g) = o.u;
            } else {
#pragma unroll
                for (int x = 0; x < 8; x++) {
                    const int c = 8 * g + x;
                    if (c < kb) blk[j * kb + c] = o.e[x];
                }
            }
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
    dim3 grid((unsigned)((n_items + 3) / 4)), block(256);
    if (d <= 32)
        k_sddmm<DT, V, 1><<<grid, block, 0, st>>>(items, n_items, f->vec_col, f->vec_mask, X, ldx, Y, ldy, (int)d, out, f->M);
    else if (d <= 64)
        k_sddmm<DT, V, 2><<<grid, block, 0, st>>>(items, n_items, f->vec_col, f->vec_mask, X, ldx, Y, ldy, (int)d, out, f->M);
    else
        k_sddmm<DT, V, 4><<<grid, block, 0, st>>>(items, n_items, f->vec_col, f->vec_mask, X, ldx, Y, ldy, (int)d, out, f->M);
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
