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
#include <algorithm>
#include <cstdlib>

#include "fs_common.h"

// Wavefronts per workgroup.  The wavefronts of a workgroup share nothing, and a workgroup keeps its slots
// until its slowest wavefront is done: one per workgroup measured best (cfg 5: 122 us against 128 us with
// four, cfg 1 and cfg 2 unchanged).
#ifndef FS_SDDMM_WPB
#define FS_SDDMM_WPB 1
#endif

namespace {

// One 32-vector block (all fields are wave-uniform).
struct BlockDesc {
    int s;   // first vector
    int kb;  // vectors in the block, 0..32 (0: block slot of an empty window, or past the end)
    int w;   // window
};

// KS = 32-feature steps of the contraction (d <= 32*KS), BB = blocks handled per round.  A block of
// scores depends on nothing but its own descriptor, so the work is cut into units of G consecutive
// block slots straight from the block table (G <= 64), whatever windows they belong to.
// CSR: also (or only) write the scores in CSR order; kept out of the plain instantiation, whose registers it
// would cost (d <= 32: 88 -> 101, one wavefront per SIMD fewer, 13.8 -> 15 us on cfg 2).
template <int DT, int V, int KS, int BB, int WPB, bool BIG, bool CSR>  // BIG: X or Y spans 4 GiB or more
__global__ void __launch_bounds__(64 * WPB)
k_sddmm(int n_blocks, int G, const int4 *__restrict__ blk_desc,
        const int32_t *__restrict__ vec_col, const uint32_t *__restrict__ vec_mask,
        const uint16_t *__restrict__ X, int64_t ldx, const uint16_t *__restrict__ Y, int64_t ldy, int d,
        uint16_t *__restrict__ out, int64_t M, uint16_t *__restrict__ out_csr, const int32_t *__restrict__ row_base)
{
    // 1 KB per wave: re-lays the scores of a narrow block before they are stored
    __shared__ __attribute__((aligned(16))) uint16_t lds_all[WPB][512];

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int unit = __builtin_amdgcn_readfirstlane(blockIdx.x * WPB + wave);  // wave-uniform
    const int first = unit * G;  // first block slot of this wavefront
    if (first >= n_blocks) return;
    const int nblk = min(G, n_blocks - first);
    const int b_lo = 0, b_hi = nblk;
    uint16_t *lds = lds_all[wave];
    const int j = lane & 15, g = lane >> 4;
    const unsigned char *Xb = reinterpret_cast<const unsigned char *>(X);
    const unsigned char *Yb = reinterpret_cast<const unsigned char *>(Y);
    const uint32_t ldx2 = (uint32_t)ldx * 2, ldy2 = (uint32_t)ldy * 2;  // bytes between rows

    // descriptors of the unit's blocks (at most 64), one per lane
    const int4 my_desc = blk_desc[first + min(lane, nblk - 1)];
    auto block = [&](int i) -> BlockDesc {  // i-th block of the unit; blocks past its end are empty
        BlockDesc dsc;
        const int ic = min(i, nblk - 1);
        dsc.s = __builtin_amdgcn_readlane(my_desc.x, ic);
        dsc.kb = i < b_hi ? (__builtin_amdgcn_readlane(my_desc.y, ic) & 255) : 0;
        dsc.w = __builtin_amdgcn_readlane(my_desc.z, ic);
        return dsc;
    };

    for (int b0 = b_lo; b0 < b_hi; b0 += BB) {
        // round of up to BB blocks: first every block's indices, masks and X rows, then every Y row,
        // so that a round costs two memory round trips however many blocks it holds
        BlockDesc dsc[BB];
        int col[BB];
        uint32_t msk[BB];
        int rbase[BB];  // CSR position of window row j's first entry in the block (CSR-order output only)
        fs_frag xf[BB][KS];
#pragma unroll
        for (int u = 0; u < BB; u++) {
            dsc[u] = block(b0 + u);
            col[u] = (lane < dsc[u].kb) ? vec_col[dsc[u].s + lane] : -1;
            msk[u] = (lane < dsc[u].kb) ? vec_mask[dsc[u].s + lane] : 0u;
            rbase[u] = 0;
            if constexpr (CSR) rbase[u] = (j < V && b0 + u < b_hi) ? row_base[(int64_t)(first + b0 + u) * V + j] : 0;
            // X operand: lane (j, g) holds X[w*V + j][32*ks + 8g .. +7]; rows past V or M are zero
            const int64_t xrow = (int64_t)dsc[u].w * V + j;
            const bool x_ok = dsc[u].kb > 0 && j < V && xrow < M;
            const uint64_t xoff = BIG ? (uint64_t)xrow * ldx2 : (uint64_t)__umul24((uint32_t)xrow, ldx2);
#pragma unroll
            for (int ks = 0; ks < KS; ks++) {
                const int f0 = 32 * ks + 8 * g;
                xf[u][ks].u = fs_u4{0u, 0u, 0u, 0u};
                if (x_ok && f0 < d) xf[u][ks].u = *reinterpret_cast<const fs_u4 *>(Xb + xoff + 2 * f0);
            }
        }
        // Y operand: matrix row j of tile t is vector 8*(j/4) + 4t + (j%4) of the block; vectors past the
        // block's width re-read its first row and are masked out below
        fs_frag yf[BB][2][KS];
#pragma unroll
        for (int u = 0; u < BB; u++) {
            const int first = max(__builtin_amdgcn_readfirstlane(col[u]), 0);
#pragma unroll
            for (int t = 0; t < 2; t++) {
                int yrow = __shfl(col[u], 8 * (j >> 2) + 4 * t + (j & 3), 64);
                yrow = yrow < 0 ? first : yrow;
                const uint64_t yoff = BIG ? (uint64_t)yrow * ldy2 : (uint64_t)__umul24((uint32_t)yrow, ldy2);
#pragma unroll
                for (int ks = 0; ks < KS; ks++) {
                    const int f0 = 32 * ks + 8 * g;
                    yf[u][t][ks].u = *reinterpret_cast<const fs_u4 *>(Yb + yoff + 2 * (f0 < d ? f0 : 0));
                    if (f0 >= d) yf[u][t][ks].u = fs_u4{0u, 0u, 0u, 0u};
                }
            }
        }
#pragma unroll
        for (int u = 0; u < BB; u++) {
            const int kb = dsc[u].kb;
            if (kb <= 0) continue;
            fs_f4 acc[2];
#pragma unroll
            for (int t = 0; t < 2; t++) {
                acc[t] = fs_f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ks++) acc[t] = fs_mfma_16x16x32<DT>(yf[u][t][ks], xf[u][ks], acc[t]);
            }
            // lane (j, g): acc[t][e] is the score of window row j and vector 8g + 4t + e
            fs_frag o;
            o.u.x = fs_pack2<DT>(acc[0][0], acc[0][1]);
            o.u.y = fs_pack2<DT>(acc[0][2], acc[0][3]);
            o.u.z = fs_pack2<DT>(acc[1][0], acc[1][1]);
            o.u.w = fs_pack2<DT>(acc[1][2], acc[1][3]);
            // bit c of `bits`: vector c of the block stores window row j.  Wave-wide ballots over the
            // per-vector occupancy masks, one per window row, instead of eight cross-lane reads.
            uint32_t bits = 0;
#pragma unroll
            for (int r = 0; r < V; r++) {
                const uint32_t has = (uint32_t)__ballot((msk[u] >> r) & 1u);
                bits = (j == r) ? has : bits;
            }
            const uint32_t mine = bits >> (8 * g);  // bit x: vector 8g + x
            uint32_t keep[4];  // 0xFFFF per stored position, else 0
#pragma unroll
            for (int p = 0; p < 4; p++)
                keep[p] = (((mine >> (2 * p)) & 1u) ? 0xFFFFu : 0u) | (((mine >> (2 * p + 1)) & 1u) ? 0xFFFF0000u : 0u);
            o.u.x &= keep[0]; o.u.y &= keep[1]; o.u.z &= keep[2]; o.u.w &= keep[3];
            if constexpr (CSR) {
                if (j < V) {
                    // CSR order: the entries of row j inside this block are consecutive positions, in vector order
                    int pos = rbase[u] + __popc(bits & ((1u << (8 * g)) - 1u));
#pragma unroll
                    for (int x = 0; x < 8; x++) {
                        if ((mine >> x) & 1u) out_csr[pos++] = o.e[x];
                    }
                }
                if (!out) continue;
            }
            uint16_t *blk = out + (int64_t)V * dsc[u].s;
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
                if (lane * 8 + 8 <= V * kb)
                    *reinterpret_cast<fs_u4 *>(blk + 8 * lane) = *reinterpret_cast<const fs_u4 *>(lds + 8 * lane);
                else if (V == 4 && lane * 8 < V * kb)  // V = 4, odd width: the last piece holds four values
                    *reinterpret_cast<uint2 *>(blk + 8 * lane) = *reinterpret_cast<const uint2 *>(lds + 8 * lane);
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
        }
    }
}

// Generic fallback for long feature dimensions (d > 128): one block at a time, the contraction in
// 32-feature steps with both operands loaded per step.
template <int DT, int V, int WPB>
__global__ void __launch_bounds__(64 * WPB)
k_sddmm_long(int n_blocks, int G, const int4 *__restrict__ blk_desc,
             const int32_t *__restrict__ vec_col, const uint32_t *__restrict__ vec_mask,
             const uint16_t *__restrict__ X, int64_t ldx, const uint16_t *__restrict__ Y, int64_t ldy, int d,
             uint16_t *__restrict__ out, int64_t M, uint16_t *__restrict__ out_csr, const int32_t *__restrict__ row_base)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int unit = __builtin_amdgcn_readfirstlane(blockIdx.x * WPB + wave);
    const int first = unit * G;
    if (first >= n_blocks) return;
    const int nblk = min(G, n_blocks - first);
    const int j = lane & 15, g = lane >> 4;
    const int nsteps = (d + 31) / 32;
    for (int step = 0; step < nblk; step++) {
        const int4 dsc = blk_desc[first + step];
        const int s = dsc.x, kb = dsc.y & 255, w = dsc.z;
        if (kb > 0) {
            const int my_col = (lane < kb) ? vec_col[s + lane] : -1;
            const uint32_t my_mask = (lane < kb) ? vec_mask[s + lane] : 0u;
            const int64_t xrow = (int64_t)w * V + j;
            const bool x_ok = j < V && xrow < M;
            fs_f4 acc[2];
#pragma unroll
            for (int t = 0; t < 2; t++) {
                acc[t] = fs_f4{0.f, 0.f, 0.f, 0.f};
                const int64_t yrow = __shfl(my_col, 8 * (j >> 2) + 4 * t + (j & 3), 64);
                for (int ks = 0; ks < nsteps; ks++) {
                    const int f0 = 32 * ks + 8 * g;
                    fs_frag yf, xx;
                    yf.u = fs_u4{0u, 0u, 0u, 0u};
                    xx.u = fs_u4{0u, 0u, 0u, 0u};
                    if (yrow >= 0 && f0 < d) yf.u = *reinterpret_cast<const fs_u4 *>(Y + yrow * ldy + f0);
                    if (x_ok && f0 < d) xx.u = *reinterpret_cast<const fs_u4 *>(X + xrow * ldx + f0);
                    acc[t] = fs_mfma_16x16x32<DT>(yf, xx, acc[t]);
                }
            }
            (void)my_mask;
            if (j < V) {
                uint16_t *blk = out ? out + (int64_t)V * s : nullptr;
                int pos = out_csr ? row_base[(int64_t)(first + step) * V + j] : 0;
                for (int c = 0; c < 8 * g && out_csr; c++) pos += (c < kb && ((vec_mask[s + c] >> j) & 1u)) ? 1 : 0;
#pragma unroll
                for (int x = 0; x < 8; x++) {
                    const int c = 8 * g + x;
                    if (c < kb) {
                        const uint32_t m = vec_mask[s + c];
                        const bool stored = (m >> j) & 1u;
                        const uint16_t v = stored ? fs_round_bits<DT>(acc[x >> 2][x & 3]) : (uint16_t)0;
                        if (blk) blk[j * kb + c] = v;
                        if (out_csr && stored) out_csr[pos++] = v;
                    }
                }
            }
        }
    }
}

template <int DT, int V>
fs_status launch(const fs_format *f, const uint16_t *X, int64_t ldx, const uint16_t *Y, int64_t ldy, int64_t d,
                 uint16_t *out, uint16_t *out_csr, hipStream_t st)
{
    if (f->n_blocks == 0) return FS_OK;
    const int n_blocks = (int)f->n_blocks;
    constexpr int WPB = FS_SDDMM_WPB;
    // blocks per wavefront: whole rounds, 4 to 16 blocks, about 16384 wavefronts on large matrices
    // (measured: 4 to 8 blocks are best from 30 thousand to 180 thousand blocks, 16 and more lose 5-15 %)
    int G = (int)std::min<int64_t>(std::max<int64_t>(((n_blocks + 16383) / 16384 + 3) / 4 * 4, 4), 16);
#ifdef FS_TUNING_ENV  // tuning builds only (-DFS_TUNING_ENV): the shipped library reads no environment
    if (const char *e = getenv("FS_SDDMM_G")) G = std::min(std::max(atoi(e), 1), 64);
#endif
    // 32-bit row offsets need X and Y to span less than 4 GiB and row number and pitch to fit 24 bits
    const bool big = f->K >= ((int64_t)1 << 24) || f->M >= ((int64_t)1 << 24) || ldx * 2 >= ((int64_t)1 << 24) ||
                     ldy * 2 >= ((int64_t)1 << 24) || f->K * ldy * 2 >= ((int64_t)1 << 32) ||
                     (f->M + 32) * ldx * 2 >= ((int64_t)1 << 32);
    const int64_t units = ((int64_t)n_blocks + G - 1) / G;
    const dim3 grid((unsigned)((units + WPB - 1) / WPB)), block(64 * WPB);
#define FS_SDDMM_ARGS n_blocks, G, (const int4 *)f->blk_desc, f->vec_col, f->vec_mask, X, ldx, Y, ldy, (int)d, out, f->M, out_csr, f->blk_row_base
#define FS_SDDMM_LAUNCH(KS, BB)                                                                           \
    {                                                                                                     \
        if (out_csr) {                                                                                    \
            if (big) k_sddmm<DT, V, KS, BB, WPB, true, true><<<grid, block, 0, st>>>(FS_SDDMM_ARGS);      \
            else k_sddmm<DT, V, KS, BB, WPB, false, true><<<grid, block, 0, st>>>(FS_SDDMM_ARGS);         \
        } else {                                                                                          \
            if (big) k_sddmm<DT, V, KS, BB, WPB, true, false><<<grid, block, 0, st>>>(FS_SDDMM_ARGS);     \
            else k_sddmm<DT, V, KS, BB, WPB, false, false><<<grid, block, 0, st>>>(FS_SDDMM_ARGS);        \
        }                                                                                                 \
    }
    if (d <= 32) FS_SDDMM_LAUNCH(1, 4)
    else if (d <= 64) FS_SDDMM_LAUNCH(2, 2)
    else if (d <= 128) FS_SDDMM_LAUNCH(4, 1)
    else k_sddmm_long<DT, V, WPB><<<grid, block, 0, st>>>(FS_SDDMM_ARGS);
#undef FS_SDDMM_LAUNCH
#undef FS_SDDMM_ARGS
    FS_LAUNCH_CHECK();
    return FS_OK;
}

}  // namespace

fs_status fs_sddmm_launch(const fs_format *f, const void *d_X, int64_t ldx, const void *d_Y, int64_t ldy, int64_t d,
                          void *d_out_blk, void *d_out_csr, hipStream_t st)
{
    const uint16_t *X = (const uint16_t *)d_X, *Y = (const uint16_t *)d_Y;
    uint16_t *out = (uint16_t *)d_out_blk, *out_csr = (uint16_t *)d_out_csr;
    if (f->dtype == FS_F16) {
        if (f->V == 4) return launch<FS_F16, 4>(f, X, ldx, Y, ldy, d, out, out_csr, st);
        if (f->V == 8) return launch<FS_F16, 8>(f, X, ldx, Y, ldy, d, out, out_csr, st);
        if (f->V == 16) return launch<FS_F16, 16>(f, X, ldx, Y, ldy, d, out, out_csr, st);
    } else if (f->dtype == FS_BF16) {
        if (f->V == 4) return launch<FS_BF16, 4>(f, X, ldx, Y, ldy, d, out, out_csr, st);
        if (f->V == 8) return launch<FS_BF16, 8>(f, X, ldx, Y, ldy, d, out, out_csr, st);
        if (f->V == 16) return launch<FS_BF16, 16>(f, X, ldx, Y, ldy, d, out, out_csr, st);
    }
    return FS_ERR_UNSUPPORTED;
}
