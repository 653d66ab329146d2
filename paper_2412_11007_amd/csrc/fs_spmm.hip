// SpMM on the CDNA4 matrix cores over the row-window format (paper Section 3.3).
//
// One wavefront owns one work item = up to `chunk` consecutive nonzero vectors
// of one window, and all N output columns of a 128-column pass.  Per block of
// 32 vectors it
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
// row of C, so results go to memory as 8-byte pieces of contiguous rows.  For
// V = 8 the upper eight window rows of the right operand are zero.
//
// The last block of a window may hold fewer than 32 vectors; lanes past its
// width feed zeros and load nothing (paper Section 3.5, residue handling).
//
// Windows cut into several items (more than `chunk` vectors) accumulate into
// fp32 partial tiles that a second kernel adds in a fixed order: no atomics,
// bit-reproducible results.
#include "fs_common.h"

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

template <int DT, int V, int NT>
__global__ void __launch_bounds__(256)
k_spmm(const int4 *__restrict__ items, int n_items, const int32_t *__restrict__ vec_col,
       const uint16_t *__restrict__ vals, const uint16_t *__restrict__ B, int64_t ldb, int N,
       uint16_t *__restrict__ C, int64_t ldc, float *__restrict__ part, int64_t M)
{
    constexpr int NC = NT * 16;   // columns per pass
    constexpr int LPR = NC / 8;   // lanes that share one gathered row (16 bytes each)
    constexpr int RPI = 64 / LPR; // rows per wave-wide load
    constexpr int NLD = 32 / RPI; // wave-wide loads per 32-vector block
    constexpr int RS = NC * 2;    // LDS row stride in bytes

    __shared__ __attribute__((aligned(16))) unsigned char lds_all[4][32 * RS];

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int item = blockIdx.x * 4 + wave;
    if (item >= n_items) return;  // no block-wide barrier is used below
    unsigned char *lds = lds_all[wave];

    const int4 it = items[item];
    const int w = it.x, s_begin = it.y, s_end = it.y + it.z, pslot = it.w;
    const int n0 = blockIdx.y * 128;  // first column of this pass
    const int j = lane & 15, g = lane >> 4;

    fs_f4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; t++) acc[t] = fs_f4{0.f, 0.f, 0.f, 0.f};

    // per-lane constants of the gather and of the transposed read
    const int g_row = lane / LPR;          // row within one wave-wide load
    const int g_col = n0 + (lane % LPR) * 8;  // first column of this lane's 16 bytes
    const bool g_col_ok = g_col < N;
    const int e = (lane & 15) >> 2, q = lane & 3;

    for (int s = s_begin; s < s_end; s += 32) {
        const int kb = min(32, s_end - s);

        // sparse operand: rows j < V of the block, vectors 8g .. 8g+7
        fs_frag sp;
        sp.u = make_uint4(0, 0, 0, 0);
        if (j < V) {
            const uint16_t *blk = vals + (int64_t)V * s;
            if (kb == 32) {
                sp.u = *reinterpret_cast<const uint4 *>(blk + j * 32 + 8 * g);
            } else {
#pragma unroll
                for (int x = 0; x < 8; x++) {
                    const int c = 8 * g + x;
                    if (c < kb) sp.e[x] = blk[j * kb + c];
                }
            }
        }

        // column indices, one per lane
        const int my_col = (lane < kb) ? vec_col[s + lane] : -1;

        // gather: NLD wave-wide loads of RPI rows each
        uint4 stage[NLD];
#pragma unroll
        for (int l = 0; l < NLD; l++) {
            const int r = l * RPI + g_row;
            const int idx = __shfl(my_col, r, 64);
            stage[l] = make_uint4(0, 0, 0, 0);
            if (idx >= 0 && g_col_ok)
                stage[l] = *reinterpret_cast<const uint4 *>(B + (int64_t)idx * ldb + g_col);
        }
#pragma unroll
        for (int l = 0; l < NLD; l++) {
            const int r = l * RPI + g_row;
            const int pos = (((lane % LPR) * 16) + 32 * lds_rot<NT>(r)) & (RS - 1);
            *reinterpret_cast<uint4 *>(lds + r * RS + pos) = stage[l];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

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

    // write back: lane (j, g) holds C[w*V + j][n0 + 16t + 4g .. +3]
    const int64_t row = (int64_t)w * V + j;
    if (j >= V || row >= M) return;
    if (pslot < 0) {
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
    } else {
        float *prow = part + ((int64_t)pslot * V + j) * N;
#pragma unroll
        for (int t = 0; t < NT; t++) {
            const int col = n0 + 16 * t + 4 * g;
            if (col < N) *reinterpret_cast<float4 *>(prow + col) = make_float4(acc[t][0], acc[t][1], acc[t][2], acc[t][3]);
        }
    }
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
    for (int idx = threadIdx.x; idx < V * n4; idx += blockDim.x) {
        const int j = idx / n4, c4 = idx - j * n4;
        const int64_t row = (int64_t)w * V + j;
        if (row >= M) continue;
        float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int k = 0; k < cnt; k++) {
            const float4 v = *reinterpret_cast<const float4 *>(part + ((int64_t)(p0 + k) * V + j) * N + 4 * c4);
            sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
        }
        uint2 o;
        o.x = (uint32_t)fs_round_bits<DT>(sum.x) | ((uint32_t)fs_round_bits<DT>(sum.y) << 16);
        o.y = (uint32_t)fs_round_bits<DT>(sum.z) | ((uint32_t)fs_round_bits<DT>(sum.w) << 16);
        *reinterpret_cast<uint2 *>(C + row * ldc + 4 * c4) = o;
    }
}

template <int DT, int V>
fs_status launch(const fs_format *f, const uint16_t *vals, const uint16_t *B, int64_t N, int64_t ldb, uint16_t *C,
                 int64_t ldc, float *part, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1)
{
    if (f->n_items == 0) return FS_OK;
    const int4 *items = (const int4 *)f->items;
    const int n_items = (int)f->n_items;
    dim3 grid((unsigned)((n_items + 3) / 4), 1, 1), block(256, 1, 1);
    if (ev0) FS_HIP(hipEventRecord(ev0, st));
    if (N <= 32) {
        k_spmm<DT, V, 2><<<grid, block, 0, st>>>(items, n_items, f->vec_col, vals, B, ldb, (int)N, C, ldc, part, f->M);
    } else if (N <= 64) {
        k_spmm<DT, V, 4><<<grid, block, 0, st>>>(items, n_items, f->vec_col, vals, B, ldb, (int)N, C, ldc, part, f->M);
    } else {
        grid.y = (unsigned)((N + 127) / 128);
        k_spmm<DT, V, 8><<<grid, block, 0, st>>>(items, n_items, f->vec_col, vals, B, ldb, (int)N, C, ldc, part, f->M);
    }
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
