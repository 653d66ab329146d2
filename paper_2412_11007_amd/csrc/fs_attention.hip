// Sparse attention in one kernel:  Out = softmax_rows(scale * (X * Y^T) at A's pattern) * H.
//
// The attention GNN of the paper's end-to-end evaluation (Section 4.4) chains SDDMM (Section 3.4), a
// softmax over the stored entries of each row, and SpMM (Section 3.3).  Run as three kernels the chain
// writes the scores, reads and rewrites them, and reads them again; here a wavefront keeps them in
// registers.  Per 32-vector block of its work item it
//   * computes the V x 32 tile of scores on the matrix cores exactly as the SDDMM kernel does (gathered
//     Y rows as the left operand, the window's X rows as the right one, 16 contiguous bytes per lane
//     straight in operand layout), which leaves lane (j, g) with the scores of window row j and vectors
//     8g .. 8g+7 -- the lane's piece of the SpMM sparse operand;
//   * masks them by the pattern, updates the running row maximum m and row sum l, turns them into
//     p = 2^(t - m) (t = score * scale * log2 e) rounded to the element type, and scales the fp32
//     accumulators of the window by 2^(m_old - m_new): the usual streaming form of a softmax-weighted sum;
//   * multiplies p with the gathered rows of H exactly as the SpMM kernel does (gather -> LDS ->
//     transposed reads -> v_mfma_f32_16x16x32).
// At the end of a window the accumulators are divided by l and stored.  A window cut across work items
// stores its unnormalised fp32 tile and (m, l) per row; a second kernel merges the parts in slot order
// with the weights 2^(m_part - m_window).  No atomics: results are bit-reproducible.
//
// One pass covers up to 256 output columns, so that the scores are computed once for N <= 256.
//
// The same kernel with the softmax compiled out (SM = false) is SDDMM followed by SpMM: the weights are
// the scaled scores, rounded to the element type as the SDDMM kernel stores them, and nothing is divided.
#include <cstdlib>
#include <utility>

#include "fs_common.h"
#include "fs_tile.h"


namespace {

__device__ __forceinline__ float fs_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// KS = 32-feature steps of the score contraction (d <= 32 * KS); NT = 16-column tiles of H per pass.
// SM = false leaves the softmax out: the weights are the scaled scores themselves, rounded to the element
// type exactly as the SDDMM kernel stores them (sl2 is then the plain scale).
template <int DT, int V, int NT, int KS, int WPB, bool SM>
__global__ void __launch_bounds__(64 * WPB) __attribute__((amdgpu_waves_per_eu(NT > 8 ? 2 : 3)))
k_attention(const int4 *__restrict__ items, int n_items, const int4 *__restrict__ blk_desc, int nvec,
            const int32_t *__restrict__ vec_col, const uint32_t *__restrict__ vec_mask,
            const uint16_t *__restrict__ X, int64_t ldx, const uint16_t *__restrict__ Y, int64_t ldy, int d, float sl2,
            const uint16_t *__restrict__ H, int64_t ldh, int N,
            uint16_t *__restrict__ C, int64_t ldc, float *__restrict__ part, float *__restrict__ stats, int64_t M, int nbx,
            int slice, int n_swz)
{
    constexpr int NC = NT * 16;   // columns per pass
    constexpr int LPR = NC / 8;   // lanes that share one gathered row (16 bytes each)
    constexpr int RPI = 64 / LPR; // rows per wave-wide load
    constexpr int NLD = 32 / RPI; // wave-wide loads per 32-vector block
    constexpr int RS = NC * 2;    // LDS row stride in bytes
    constexpr int LDS_BYTES = lds_row<RS>(31) + RS;

    __shared__ __attribute__((aligned(16))) unsigned char lds_all[WPB][(LDS_BYTES + 15) / 16 * 16];

    const int pass = blockIdx.x / nbx;
    const int bx = blockIdx.x - pass * nbx;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int turn = __builtin_amdgcn_readfirstlane(fs_launch_turn<WPB>(bx, slice, n_swz) + wave);  // wave-uniform
    if (turn >= n_items) return;  // no block-wide barrier is used below
    unsigned char *lds = lds_all[wave];

    const int4 it = items[turn];  // the work list in launch order: {first block slot, blocks, first partial slot, first vector}
    const int nblk = it.y;
    if (nblk == 0) return;
    int slot = it.z;
    const int n0 = pass * NC;
    const int j = lane & 15, g = lane >> 4;

    const int4 my_desc = blk_desc[it.x + min(lane, nblk - 1)];
    auto block = [&](int i) -> BlockDesc { return fs_item_block(my_desc, i, nblk); };

    fs_f4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; t++) acc[t] = fs_f4{0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY;  // running maximum of t over the window row's entries seen so far (all four g lanes agree)
    float l_run = 0.f;        // this lane's share of the sum of 2^(t - m_run)

    // per-lane constants of the gather of H and of the transposed read
    const int g_row = lane / LPR;
    const int g_col = n0 + (lane % LPR) * 8;
    const uint32_t g_colb = (g_col < N ? g_col : 0) * 2;  // lanes past N read (never store) column 0
    const unsigned char *Hb = reinterpret_cast<const unsigned char *>(H);
    const unsigned char *Xb = reinterpret_cast<const unsigned char *>(X);
    const unsigned char *Yb = reinterpret_cast<const unsigned char *>(Y);
    const uint32_t ldh2 = (uint32_t)ldh * 2, ldx2 = (uint32_t)ldx * 2, ldy2 = (uint32_t)ldy * 2;
    const bool full_pass = n0 + NC <= N;
    const int e4 = (lane & 15) >> 2, q = lane & 3;
    const uint32_t p_lane = (uint32_t)((n0 / 16) * (V * 16) + (g * V + j) * 4) * 4;  // as in the SpMM partial tiles
    unsigned char *lds_wr = lds + lds_row<RS>(g_row) + (lane % LPR) * 16;
    const unsigned char *lds_rd = lds + lds_row<RS>(8 * g + e4) + 8 * q;
    // byte offset of this lane's features inside a row of X or Y, per 32-feature step; steps past d read
    // the row's first bytes and meet a zero X operand
    uint32_t f_off[KS];
    bool f_ok[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
        f_ok[ks] = 32 * ks + 8 * g < d;
        f_off[ks] = f_ok[ks] ? 2 * (32 * ks + 8 * g) : 0;
    }

    // Column indices of a block.  A gathered row of H is shared by 16 or 32 lanes, so every group of 16
    // lanes wants the same index for a given wave-wide load: lane i of a group holds the index for load i
    // (vector i * RPI + the group's row) and a DPP broadcast hands it out.  Vectors past the block's width
    // repeat its last one (their occupancy mask is zero, so whatever they gather is ignored).
    auto load_cols = [&](const BlockDesc &b) -> int {
        const int v = (lane & 15) * RPI + lane / LPR;
        return vec_col[max(min(b.s + min(v, b.kb - 1), nvec - 1), 0)];
    };
    // the lane that holds vector u's index in that arrangement
    auto holder = [&](int u) -> int { return (u % RPI) * LPR + u / RPI; };
    auto load_mask = [&](const BlockDesc &b) -> uint32_t {
        const uint32_t m = vec_mask[max(min(b.s + min(lane, b.kb - 1), nvec - 1), 0)];
        return lane < b.kb ? m : 0u;
    };
    // X operand of a block: lane (j, g) holds X[w*V + j][32ks + 8g .. +7]; rows past V or M and features
    // past d are zero.  The load itself is unconditional (row 0 stands in).
    fs_frag xf[KS];
    auto load_x = [&](const BlockDesc &b) {
        const int64_t xrow = (int64_t)b.w * V + j;
        const bool ok = j < V && xrow < M;
        const uint32_t xoff = __umul24((uint32_t)(ok ? xrow : 0), ldx2);
#pragma unroll
        for (int ks = 0; ks < KS; ks++) {
            xf[ks].u = *reinterpret_cast<const fs_u4 *>(Xb + xoff + f_off[ks]);
            if (!ok || !f_ok[ks]) xf[ks].u = fs_u4{0u, 0u, 0u, 0u};
        }
    };
    // Y operand: matrix row j of tile t is vector 8*(j/4) + 4t + (j%4) of the block
    uint32_t yoff[2];
    fs_frag yf[2][KS];
#define FS_YROWS(cols)                                                                           \
    {                                                                                            \
        _Pragma("unroll") for (int t = 0; t < 2; t++)                                            \
            yoff[t] = __umul24((uint32_t)__shfl(cols, holder(8 * (j >> 2) + 4 * t + (j & 3)), 64), ldy2); \
    }
#define FS_YGATHER()                                                                             \
    _Pragma("unroll") for (int t = 0; t < 2; t++)                                                \
        _Pragma("unroll") for (int ks = 0; ks < KS; ks++)                                        \
            yf[t][ks].u = *reinterpret_cast<const fs_u4 *>(Yb + yoff[t] + f_off[ks]);
    // rows of H this lane gathers for a block, as 32-bit byte offsets
    uint32_t grow[NLD];
#define FS_ROWS(cols)                                                                            \
    {                                                                                            \
        fs_for_each_index([&](auto l_) {                                                         \
            constexpr int l = decltype(l_)::value;                                               \
            grow[l] = __umul24((uint32_t)fs_row_bcast<l>(cols), ldh2) + g_colb;                  \
        }, std::make_integer_sequence<int, NLD>{});                                              \
    }
    fs_u4 stage[NLD];
#define FS_GATHER()                                                                              \
    _Pragma("unroll") for (int l = 0; l < NLD; l++)                                              \
        stage[l] = *reinterpret_cast<const fs_u4 *>(Hb + grow[l]);

    // Software pipeline: while block i is multiplied, the rows of H and of Y, the rows of X and the mask
    // of block i+1 are in flight; row numbers are worked out a step earlier, indices two steps earlier.
    BlockDesc d0 = block(0), d1 = block(1), d2 = block(2);
    const int col0 = load_cols(d0);
    const int col1 = load_cols(d1);
    int col2 = load_cols(d2);
    uint32_t msk0 = load_mask(d0);
    bool from_first = d0.first;
    load_x(d0);
    FS_YROWS(col0)
    FS_YGATHER()
    FS_YROWS(col1)
    FS_ROWS(col0)
    FS_GATHER()
    FS_ROWS(col1)

    // One block step.  MORE: another block of the item follows (its rows of Y and H are gathered here).  The
    // last step is a second instance of the same code, so that inside the loop every path issues the same
    // loads and the compiler can wait for exactly the ones a use needs: loads return in the order they were
    // issued, and a wait that cannot tell waits for everything in flight.
    // (The 256-column instantiations keep one instance and a run-time flag: twice their code measured 1 % slower.)
    int step = 0;
    auto block_step = [&](auto more_) {
        const bool MORE = more_;  // a compile-time constant where the argument is one
        const int kb = d0.kb;
        // The small loads ahead -- the indices three blocks ahead and the next block's mask -- are copied to
        // their places when the step ends; behind the gathers that copy waits for both.  The 128-column
        // instantiations issue them first (cfg 2 -3 %); the 256-column ones, with two wavefronts per SIMD and
        // sixteen loads per gather, measured 1-2 % better with the gathers in front.
        constexpr bool SMALL_FIRST = NT <= 8;
        const BlockDesc d3 = block(step + 3);
        int col3 = 0;
        uint32_t msk1 = 0;
        if constexpr (SMALL_FIRST) {
            col3 = load_cols(d3);
            msk1 = load_mask(d1);
        }
        // ---- scores of this block -> probabilities relative to the running maximum
        fs_frag sp;
        float corr;
        {
            fs_f4 sc[2];
#pragma unroll
            for (int t = 0; t < 2; t++) {
                sc[t] = fs_f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ks++) sc[t] = fs_mfma_16x16x32<DT>(yf[t][ks], xf[ks], sc[t]);
            }
            // bit c of `bits`: vector c of the block stores window row j (from the per-vector occupancy masks)
            uint32_t bits = 0;
#pragma unroll
            for (int r = 0; r < V; r++) {
                const uint32_t has = (uint32_t)__ballot((msk0 >> r) & 1u);
                bits = (j == r) ? has : bits;
            }
            const uint32_t mine = bits >> (8 * g);  // bit 4t + e: vector 8g + 4t + e
            float p[8];
            if constexpr (SM) {
                float tv[8];
                float mx = -INFINITY;
#pragma unroll
                for (int x = 0; x < 8; x++) {
                    tv[x] = ((mine >> x) & 1u) ? sc[x >> 2][x & 3] * sl2 : -INFINITY;
                    mx = fmaxf(mx, tv[x]);
                }
                mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
                mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
                const float m_new = fmaxf(m_run, mx);
                const float m_use = m_new == -INFINITY ? 0.f : m_new;  // a row without entries so far
                corr = fs_exp2(m_run - m_use);
                float ps = 0.f;
#pragma unroll
                for (int x = 0; x < 8; x++) {
                    p[x] = fs_exp2(tv[x] - m_use);
                    ps += p[x];
                }
                l_run = l_run * corr + ps;
                m_run = m_new;
            } else {
                corr = 1.f;
#pragma unroll
                for (int x = 0; x < 8; x++) p[x] = ((mine >> x) & 1u) ? sc[x >> 2][x & 3] * sl2 : 0.f;
            }
            sp.u.x = fs_pack2<DT>(p[0], p[1]);
            sp.u.y = fs_pack2<DT>(p[2], p[3]);
            sp.u.z = fs_pack2<DT>(p[4], p[5]);
            sp.u.w = fs_pack2<DT>(p[6], p[7]);
        }
        // ---- the next block's Y rows and X rows
        if (MORE) FS_YGATHER()
        load_x(d1);
        if constexpr (!SMALL_FIRST) msk1 = load_mask(d1);

        if (kb > 0) {
            // the gathered rows of H go to LDS (this is where the wave waits for the gather)
#pragma unroll
            for (int l = 0; l < NLD; l++)
                *reinterpret_cast<fs_u4 *>(lds_wr + lds_row<RS>(l * RPI)) = stage[l];
        }
        if (MORE) FS_GATHER()
        if constexpr (!SMALL_FIRST) col3 = load_cols(d3);
        FS_WAVE_SYNC();

        if (kb > 0) {
#pragma unroll
            for (int t = 0; t < NT; t++) {
                fs_frag dn;
#pragma unroll
                for (int h = 0; h < 2; h++)
                    dn.s[h] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (fs_s4 __attribute__((address_space(3))) *)(lds_rd + lds_row<RS>(4 * h) + 32 * t));
                acc[t] = fs_mfma_16x16x32<DT>(dn, sp, SM ? acc[t] * corr : acc[t]);
            }
            FS_WAVE_SYNC();
        }
        FS_ROWS(col2)
        FS_YROWS(col2)

        if (d0.last || !MORE) {
            // flush: lane (j, g) holds row j, columns n0 + 16t + 4g .. +3 of the window's weighted sum
            float l_tot = l_run + __shfl_xor(l_run, 16, 64);
            l_tot += __shfl_xor(l_tot, 32, 64);
            const bool whole = d0.last && from_first;
            if (whole) {
                const float inv = SM ? (l_tot > 0.f ? 1.0f / l_tot : 0.f) : 1.f;  // a row without entries gives zeros
                fs_round_tile_to_lds<DT, V, NT, RS>(lds, acc, j, g, inv);
                FS_WAVE_SYNC();
                fs_store_tile_rows<V, RPI, RS>(lds_wr, C, ldc, d0.w, M, N, g_row, g_col);
                FS_WAVE_SYNC();
            } else {
                // a part of a cut window: the unnormalised tile, and (m, l) per row for the merge
                fs_store_partial_tile<V, NT>(part, slot, N, p_lane, acc, j < V, full_pass, n0, g);
                if (j < V) {
                    if (SM && pass == 0 && g == 0) {
                        stats[(int64_t)slot * 2 * V + j] = m_run;
                        stats[(int64_t)slot * 2 * V + V + j] = l_tot;
                    }
                }
                slot++;
            }
#pragma unroll
            for (int t = 0; t < NT; t++) acc[t] = fs_f4{0.f, 0.f, 0.f, 0.f};
            m_run = -INFINITY;
            l_run = 0.f;
        }
        if (d0.last) from_first = true;
        d0 = d1; d1 = d2; d2 = d3;
        col2 = col3;
        msk0 = msk1;
    };
    if constexpr (NT <= 8) {
        for (; step + 1 < nblk; step++) block_step(std::true_type{});
        block_step(std::false_type{});
    } else {
        for (; step < nblk; step++) block_step(step + 1 < nblk);
    }
#undef FS_GATHER
#undef FS_ROWS
#undef FS_YGATHER
#undef FS_YROWS
}

// Merges the parts of one cut window: with m* the largest m over the parts of a row,
//   out = sum_k 2^(m_k - m*) tile_k / sum_k 2^(m_k - m*) l_k,
// tiles taken in slot order.  One wavefront per window and 32 columns -- many small workgroups, so that a hub
// window with dozens of parts is not one long-running workgroup.  Lane (row r = lane % V, q = lane / V)
// first walks the parts q, q + 64/V, ... for the row's m* and its sum (merged across the lanes of a row by
// shuffles: a fixed order), then adds the tiles at its position, sixteen loads in flight.  Tiles are read in
// their storage order (16-column tile, 4-column group, row) and the rounded rows leave through LDS as
// contiguous 16-byte pieces.
template <int DT, int V, bool SM>
__global__ void __launch_bounds__(64)
k_attention_reduce(const int4 *__restrict__ split_windows, const float *__restrict__ part, const float *__restrict__ stats,
                   int N, uint16_t *__restrict__ C, int64_t ldc, int64_t M)
{
    constexpr int CH = 32;  // columns per workgroup
    constexpr int KQ = 64 / V;
    __shared__ __attribute__((aligned(16))) uint16_t out_t[V][CH + 8];
    const int n_chunks = (N + CH - 1) / CH;
    const int4 sw = split_windows[blockIdx.x / n_chunks];
    const int w = sw.x, p0 = sw.y, cnt = sw.z;
    const int lane = threadIdx.x, r = lane % V, q = lane / V;
    const float *st = stats + (int64_t)p0 * 2 * V;
    float use = 0.f, inv = 1.f;  // of row r
    if constexpr (SM) {
        float top = -INFINITY;
        for (int k = q; k < cnt; k += KQ) top = fmaxf(top, st[(int64_t)k * 2 * V + r]);
#pragma unroll
        for (int o = V; o < 64; o <<= 1) top = fmaxf(top, __shfl_xor(top, o, 64));
        use = top == -INFINITY ? 0.f : top;
        float total = 0.f;
        for (int k = q; k < cnt; k += KQ) total += st[(int64_t)k * 2 * V + V + r] * fs_exp2(st[(int64_t)k * 2 * V + r] - use);
#pragma unroll
        for (int o = V; o < 64; o <<= 1) total += __shfl_xor(total, o, 64);
        inv = total > 0.f ? 1.0f / total : 0.f;
    }
    const int64_t tile4 = (int64_t)V * N / 4;  // float4 per partial tile
    const fs_f4 *base = reinterpret_cast<const fs_f4 *>(part) + (int64_t)p0 * tile4;
    const int c0 = (blockIdx.x % n_chunks) * CH;
    const int nc = min(CH, N - c0);  // columns of this workgroup, a multiple of 8
    const fs_f4 *src0 = base + (c0 / 4) * V;
    for (int idx = lane; idx < (nc / 4) * V; idx += 64) {  // idx % V == r: the position's row is the lane's
        const int ct = idx / (4 * V), rem = idx - ct * 4 * V, g = rem / V, j = rem - g * V;
        const fs_f4 *src = src0 + idx;
        const float *mk = st + j;
        fs_f4 sum = fs_f4{0.f, 0.f, 0.f, 0.f};
        for (int k = 0; k < cnt; k += 16) {  // sixteen loads in flight, added in slot order
            fs_f4 v[16];
            float wk[16];
#pragma unroll
            for (int u = 0; u < 16; u++) {
                const int kk = min(k + u, cnt - 1);
                v[u] = src[(int64_t)kk * tile4];
                wk[u] = SM ? mk[(int64_t)kk * 2 * V] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 16; u++)
                if (k + u < cnt) sum += SM ? v[u] * fs_exp2(wk[u] - use) : v[u];
        }
        uint2 o;
        o.x = fs_pack2<DT>(sum[0] * inv, sum[1] * inv);
        o.y = fs_pack2<DT>(sum[2] * inv, sum[3] * inv);
        *reinterpret_cast<uint2 *>(&out_t[j][16 * ct + 4 * g]) = o;
    }
    __syncthreads();
    const int c8n = nc / 8;
    for (int t = lane; t < V * c8n; t += 64) {
        const int j = t / c8n, c8 = t - j * c8n;
        const int64_t row = (int64_t)w * V + j;
        if (row < M)
            __builtin_nontemporal_store(*reinterpret_cast<const fs_u4 *>(&out_t[j][8 * c8]),
                                        reinterpret_cast<fs_u4 *>(C + row * ldc + c0 + 8 * c8));
    }
}

// WPB wavefronts (= work items) per workgroup.  A workgroup keeps its slots until its slowest wavefront is
// done: small launches, whose tail is a large part of the run, do best with one (cfg 2: -5 %), large ones
// with four (cfg 5: one per workgroup is 2 % slower).
template <int DT, int V, int NT, bool SM, int WPB>
fs_status launch_wpb(const fs_format *f, const uint16_t *X, int64_t ldx, const uint16_t *Y, int64_t ldy, int d, float sl2,
                     const uint16_t *H, int64_t ldh, int N, uint16_t *C, int64_t ldc, float *part, float *stats,
                     hipStream_t st)
{
    const int n_items = (int)f->n_items;
    const fs_launch_geometry geo = fs_launch_geometry_for(f, WPB);
    const int nbx = geo.nbx;
    const int passes = (N + NT * 16 - 1) / (NT * 16);
    const int64_t nblocks = (int64_t)nbx * passes;
    if (nblocks >= ((int64_t)1 << 31)) return FS_ERR_TOO_LARGE;
    dim3 grid((unsigned)nblocks, 1, 1), block(64 * WPB, 1, 1);
#define FS_ATTN_ARGS (const int4 *)f->items_by_cost, n_items, (const int4 *)f->blk_desc, (int)f->nvec, f->vec_col, f->vec_mask, \
                     X, ldx, Y, ldy, d, sl2, H, ldh, N, C, ldc, part, stats, f->M, nbx, geo.slice, geo.n_swz
    if (d <= 32) k_attention<DT, V, NT, 1, WPB, SM><<<grid, block, 0, st>>>(FS_ATTN_ARGS);
    else if (d <= 64) k_attention<DT, V, NT, 2, WPB, SM><<<grid, block, 0, st>>>(FS_ATTN_ARGS);
    else k_attention<DT, V, NT, 4, WPB, SM><<<grid, block, 0, st>>>(FS_ATTN_ARGS);
#undef FS_ATTN_ARGS
    FS_LAUNCH_CHECK();
    if (f->n_split_windows > 0) {
        const int64_t rblocks = f->n_split_windows * ((N + 31) / 32);  // one workgroup per window and 32 columns
        if (rblocks >= ((int64_t)1 << 31)) return FS_ERR_TOO_LARGE;
        k_attention_reduce<DT, V, SM><<<(unsigned)rblocks, 64, 0, st>>>((const int4 *)f->split_windows, part, stats, N,
                                                                       C, ldc, f->M);
        FS_LAUNCH_CHECK();
    }
    return FS_OK;
}

template <int DT, int V, int NT, bool SM>
fs_status launch_nt(const fs_format *f, const uint16_t *X, int64_t ldx, const uint16_t *Y, int64_t ldy, int d, float sl2,
                    const uint16_t *H, int64_t ldh, int N, uint16_t *C, int64_t ldc, float *part, float *stats,
                    hipStream_t st)
{
    if (f->n_items < 16384) return launch_wpb<DT, V, NT, SM, 1>(f, X, ldx, Y, ldy, d, sl2, H, ldh, N, C, ldc, part, stats, st);
    return launch_wpb<DT, V, NT, SM, 4>(f, X, ldx, Y, ldy, d, sl2, H, ldh, N, C, ldc, part, stats, st);
}

template <int DT, int V>
fs_status launch(const fs_format *f, const uint16_t *X, int64_t ldx, const uint16_t *Y, int64_t ldy, int d, float sl2,
                 const uint16_t *H, int64_t ldh, int N, uint16_t *C, int64_t ldc, float *work, hipStream_t st, bool softmax)
{
    if (f->n_items == 0) return FS_OK;
    float *part = work;
    float *stats = work + (size_t)f->n_split_items * (size_t)V * (size_t)N;
    if (softmax) {
        if (N <= 128) return launch_nt<DT, V, 8, true>(f, X, ldx, Y, ldy, d, sl2, H, ldh, N, C, ldc, part, stats, st);
        return launch_nt<DT, V, 16, true>(f, X, ldx, Y, ldy, d, sl2, H, ldh, N, C, ldc, part, stats, st);
    }
    if (N <= 128) return launch_nt<DT, V, 8, false>(f, X, ldx, Y, ldy, d, sl2, H, ldh, N, C, ldc, part, stats, st);
    return launch_nt<DT, V, 16, false>(f, X, ldx, Y, ldy, d, sl2, H, ldh, N, C, ldc, part, stats, st);
}

}  // namespace

fs_status fs_attention_launch(const fs_format *f, const void *d_X, int64_t ldx, const void *d_Y, int64_t ldy, int64_t d,
                              float scale, const void *d_H, int64_t N, int64_t ldh, void *d_out, int64_t ldo,
                              void *d_work, hipStream_t st, bool softmax)
{
    const uint16_t *X = (const uint16_t *)d_X, *Y = (const uint16_t *)d_Y, *H = (const uint16_t *)d_H;
    uint16_t *C = (uint16_t *)d_out;
    const float sl2 = softmax ? scale * 1.44269504088896340736f : scale;  // softmax: scores in units of log2
    float *work = (float *)d_work;
    if (f->dtype == FS_F16) {
        if (f->V == 4) return launch<FS_F16, 4>(f, X, ldx, Y, ldy, (int)d, sl2, H, ldh, (int)N, C, ldo, work, st, softmax);
        if (f->V == 8) return launch<FS_F16, 8>(f, X, ldx, Y, ldy, (int)d, sl2, H, ldh, (int)N, C, ldo, work, st, softmax);
        if (f->V == 16) return launch<FS_F16, 16>(f, X, ldx, Y, ldy, (int)d, sl2, H, ldh, (int)N, C, ldo, work, st, softmax);
    } else if (f->dtype == FS_BF16) {
        if (f->V == 4) return launch<FS_BF16, 4>(f, X, ldx, Y, ldy, (int)d, sl2, H, ldh, (int)N, C, ldo, work, st, softmax);
        if (f->V == 8) return launch<FS_BF16, 8>(f, X, ldx, Y, ldy, (int)d, sl2, H, ldh, (int)N, C, ldo, work, st, softmax);
        if (f->V == 16) return launch<FS_BF16, 16>(f, X, ldx, Y, ldy, (int)d, sl2, H, ldh, (int)N, C, ldo, work, st, softmax);
    }
    return FS_ERR_UNSUPPORTED;
}
