// Edge softmax on gfx950: for every row of A, the softmax of scale * value over the row's stored
// entries, on a value array in the vals_blk layout (the output of fs_sddmm, the input of fs_spmm).
// It is the normalisation step between the two in an attention GNN (the paper's end-to-end
// evaluation, Section 4.4, names the softmax layer without describing a kernel; the definition is
// the usual one).
//
// One wavefront walks one work item (the same items as fs_spmm / fs_sddmm).  Inside an item a window
// appears as a run of consecutive blocks.  A window that lies whole inside the item is finished on
// the spot: row maxima, row sums of exponentials, then the normalised values.  A window cut across
// items leaves (maximum, sum) per row in the workspace slot of each part -- the slots are numbered
// exactly like the partial tiles of fs_spmm -- and a second launch normalises the parts, each of which
// first merges the pairs of all parts of its window in a fixed order.  No atomics: results are
// bit-reproducible.
//
// Lane (j, q) = (lane % V, lane / V) handles row j and the E = V/2 vectors q*E .. q*E+E-1 of a block: for a
// full block that is one aligned 8- or 16-byte piece of the row-major tile.  A run is read twice: once
// for the statistics (a running maximum and a sum of exponentials relative to it, rescaled when the
// maximum moves), once to write the normalised values.
//
// The same walk serves the gradient of that softmax (BWD): with p the probabilities and g the gradient
// that arrives at them, both in the vals_blk layout,  ds = scale * p * (g - sum over the row of p * g).
// The row statistic is then a plain sum, kept in the second float of a workspace pair.
#include <algorithm>
#include <cmath>

#include "fs_common.h"

namespace {

constexpr int kWpb = 1;  // wavefronts (= work items) per workgroup: one measured best (cfg 5 -3 %; they share nothing)

template <int DT>
__device__ __forceinline__ float fs_to_float(uint16_t bits)
{
    if (DT == FS_F16) {
        union { uint16_t u; _Float16 h; } c;
        c.u = bits;
        return (float)c.h;
    }
    return __uint_as_float((uint32_t)bits << 16);
}

// (maximum, sum of exp(. - maximum)) of two disjoint sets of scores -> the same for their union
__device__ __forceinline__ void merge_stats(float &top, float &total, float top2, float total2)
{
    const float t = fmaxf(top, top2);
    if (t > -INFINITY) total = total * __expf(top - t) + total2 * __expf(top2 - t);
    top = t;
}

// E scaled scores of row j of a block (vectors q*E ..), -infinity where A stores nothing
template <int DT, int V>
struct BlockScores {
    static constexpr int E = V / 2;
    float v[E];
    uint16_t raw[E];
    uint32_t mk[E];
    // issue the loads of a full block (kb = 32): one aligned piece of the row, E masks
    __device__ __forceinline__ void fetch_full(const uint16_t *__restrict__ vals, const uint32_t *__restrict__ vec_mask,
                                               int s, int j, int q)
    {
        const uint16_t *p = vals + (int64_t)V * s + j * 32 + q * E;
        if constexpr (E == 2) {
            const uint32_t r = *reinterpret_cast<const uint32_t *>(p);
            raw[0] = r & 0xFFFF; raw[1] = r >> 16;
            mk[0] = vec_mask[s + q * E];
            mk[1] = vec_mask[s + q * E + 1];
        } else if constexpr (E == 4) {
            const uint2 r = *reinterpret_cast<const uint2 *>(p);
            raw[0] = r.x & 0xFFFF; raw[1] = r.x >> 16; raw[2] = r.y & 0xFFFF; raw[3] = r.y >> 16;
            const fs_u4 m = *reinterpret_cast<const fs_u4 *>(vec_mask + s + q * E);
            mk[0] = m.x; mk[1] = m.y; mk[2] = m.z; mk[3] = m.w;
        } else {
            const fs_u4 r = *reinterpret_cast<const fs_u4 *>(p);
            raw[0] = r.x & 0xFFFF; raw[1] = r.x >> 16; raw[2] = r.y & 0xFFFF; raw[3] = r.y >> 16;
            raw[4] = r.z & 0xFFFF; raw[5] = r.z >> 16; raw[6] = r.w & 0xFFFF; raw[7] = r.w >> 16;
            const fs_u4 m0 = *reinterpret_cast<const fs_u4 *>(vec_mask + s + q * E);
            const fs_u4 m1 = *reinterpret_cast<const fs_u4 *>(vec_mask + s + q * E + 4);
            mk[0] = m0.x; mk[1] = m0.y; mk[2] = m0.z; mk[3] = m0.w;
            mk[4] = m1.x; mk[5] = m1.y; mk[6] = m1.z; mk[7] = m1.w;
        }
    }
    // the same for a block of any width (row stride kb): element by element
    __device__ __forceinline__ void fetch_any(const uint16_t *__restrict__ vals, const uint32_t *__restrict__ vec_mask,
                                              int s, int kb, int j, int q)
    {
#pragma unroll
        for (int e = 0; e < E; e++) {
            const int c = q * E + e;
            const bool in = c < kb;
            mk[e] = in ? vec_mask[s + c] : 0u;
            raw[e] = in ? vals[(int64_t)V * s + j * kb + c] : (uint16_t)0;
        }
    }
    __device__ __forceinline__ void scale_and_mask(int j, float scale)
    {
#pragma unroll
        for (int e = 0; e < E; e++) v[e] = ((mk[e] >> j) & 1) ? scale * fs_to_float<DT>(raw[e]) : -INFINITY;
    }
    // BWD: the plain values, zero where A stores nothing
    __device__ __forceinline__ void plain_and_mask(int j)
    {
#pragma unroll
        for (int e = 0; e < E; e++) v[e] = ((mk[e] >> j) & 1) ? fs_to_float<DT>(raw[e]) : 0.f;
    }
    // BWD: sum of p * g over this block's share of the row
    __device__ __forceinline__ void absorb_dot(const BlockScores &g, float &total) const
    {
#pragma unroll
        for (int e = 0; e < E; e++) total = fmaf(v[e], g.v[e], total);
    }
    // BWD: scale * p * (g - dot), stored in the block's tile (row stride kb); *this holds p
    __device__ __forceinline__ void store_grad(const BlockScores &g, uint16_t *__restrict__ out, int s, int kb, int j, int q,
                                               float dot, float scale) const
    {
        float y[E];
#pragma unroll
        for (int e = 0; e < E; e++) y[e] = ((mk[e] >> j) & 1) ? scale * v[e] * (g.v[e] - dot) : 0.f;
        store_values(y, out, s, kb, j, q);
    }
    // running (maximum, sum) of a lane absorbs this block's scores
    __device__ __forceinline__ void absorb(float &top, float &total) const
    {
        float bt = v[0];
#pragma unroll
        for (int e = 1; e < E; e++) bt = fmaxf(bt, v[e]);
        if (bt > -INFINITY) {
            const float t = fmaxf(top, bt);
            float sum = total * __expf(top - t);
#pragma unroll
            for (int e = 0; e < E; e++) sum += __expf(v[e] - t);  // exp(-inf) = 0 where nothing is stored
            top = t;
            total = sum;
        }
    }
    // normalised values of this block, stored in its tile (row stride kb)
    __device__ __forceinline__ void store(uint16_t *__restrict__ out, int s, int kb, int j, int q, float top, float inv) const
    {
        float y[E];
#pragma unroll
        for (int e = 0; e < E; e++) {
            // The fast exponential returns zero where the result would be a subnormal fp32 number, a range
            // bf16 still represents: far below the maximum, evaluate e^(x+40) and scale by e^-40 (the
            // multiplication keeps subnormal results).
            const float x = v[e] - top;
            const float p = x < -80.f ? __expf(x + 40.f) * 4.24835425529158899533e-18f : __expf(x);
            y[e] = v[e] > -INFINITY ? p * inv : 0.f;
        }
        store_values(y, out, s, kb, j, q);
    }
    // E values of row j into the block's tile (row stride kb)
    __device__ __forceinline__ void store_values(const float (&y)[E], uint16_t *__restrict__ out, int s, int kb, int j, int q) const
    {
        if (kb == 32) {
            uint16_t *p = out + (int64_t)V * s + j * 32 + q * E;
            if constexpr (E == 2) {
                *reinterpret_cast<uint32_t *>(p) = fs_pack2<DT>(y[0], y[1]);
            } else if constexpr (E == 4) {
                uint2 o;
                o.x = fs_pack2<DT>(y[0], y[1]); o.y = fs_pack2<DT>(y[2], y[3]);
                *reinterpret_cast<uint2 *>(p) = o;
            } else {
                fs_u4 o;
                o.x = fs_pack2<DT>(y[0], y[1]); o.y = fs_pack2<DT>(y[2], y[3]);
                o.z = fs_pack2<DT>(y[4], y[5]); o.w = fs_pack2<DT>(y[6], y[7]);
                *reinterpret_cast<fs_u4 *>(p) = o;
            }
        } else {
#pragma unroll
            for (int e = 0; e < E; e++) {
                const int c = q * E + e;
                if (c < kb) out[(int64_t)V * s + j * kb + c] = fs_round_bits<DT>(y[e]);
            }
        }
    }
};

// PARTS = false: statistics of every run, whole windows are normalised, parts of cut windows leave
//                their statistics in the workspace.
// PARTS = true : parts of cut windows are normalised; each merges the statistics its window's parts left in
//                the workspace (a fixed order: deterministic).
// BWD          : the gradient instead: `in` holds the probabilities, `in2` the gradient that arrives at them,
//                the row statistic is sum p * g (second float of a workspace pair), the output
//                scale * p * (g - that sum).
template <int DT, int V, bool PARTS, bool BWD>
__global__ void __launch_bounds__(64 * kWpb)
k_edge_softmax(const int4 *__restrict__ items, int n_items, const int4 *__restrict__ blk_desc,
               const uint32_t *__restrict__ vec_mask, const uint16_t *__restrict__ in, const uint16_t *__restrict__ in2,
               uint16_t *__restrict__ out, float *__restrict__ stats, float scale, const int2 *__restrict__ slot_range,
               int n_slots)
{
    constexpr int E = V / 2;  // vectors per lane and block
    constexpr int B = 4;      // full blocks whose loads are issued together
    const int lane = threadIdx.x & 63;
    const int item = __builtin_amdgcn_readfirstlane(blockIdx.x * kWpb + (threadIdx.x >> 6));
    if (item >= n_items) return;
    const int4 it = items[item];  // {first block slot, blocks, first workspace slot, first vector}
    const int nblk = it.y;
    if (nblk == 0) return;
    int slot = it.z;
    const int j = lane % V, q = lane / V;
    // PARTS: where the statistics of the windows of the item's (at most two) parts lie -- slot numbers that
    // follow from the item record alone, so these loads travel together with the descriptors'
    int2 range0 = make_int2(0, 0), range1 = make_int2(0, 0);
    if constexpr (PARTS) {
        range0 = slot_range[min(slot, n_slots - 1)];
        range1 = slot_range[min(slot + 1, n_slots - 1)];
    }
    const int4 my_desc = blk_desc[it.x + min(lane, nblk - 1)];  // at most 64 blocks per item

    int a = 0;  // first block of the current run
    while (a < nblk) {
        // the run ends with the window's last block or with the item
        int b = a;
        bool ends_window = false;
        while (b < nblk && !ends_window) {
            ends_window = (__builtin_amdgcn_readlane(my_desc.y, b) & 256) != 0;
            b++;
        }
        const bool whole = ends_window && (__builtin_amdgcn_readlane(my_desc.y, a) & 512) != 0;
        if (PARTS && whole) { a = b; continue; }
        // every block of a window but its last is full
        const int nfull = a + (ends_window ? b - a - 1 : b - a);

        float top = -INFINITY, total = 0.f;
        if constexpr (!PARTS) {
            if (whole && b - a <= B) {
                // A window of at most B blocks that lies whole inside the item (most windows of a graph with
                // short rows): read once, keep the blocks in registers between the statistics and the output.
                BlockScores<DT, V> x[B], g[BWD ? B : 1];
                int kbs[B];
#pragma unroll
                for (int u = 0; u < B; u++) {
                    const int i = min(a + u, b - 1);
                    const int s = __builtin_amdgcn_readlane(my_desc.x, i);
                    kbs[u] = a + u < b ? (__builtin_amdgcn_readlane(my_desc.y, i) & 255) : 0;
                    if (kbs[u] == 32) {
                        x[u].fetch_full(in, vec_mask, s, j, q);
                        if constexpr (BWD) g[u].fetch_full(in2, vec_mask, s, j, q);
                    } else if (kbs[u] > 0) {
                        x[u].fetch_any(in, vec_mask, s, kbs[u], j, q);
                        if constexpr (BWD) g[u].fetch_any(in2, vec_mask, s, kbs[u], j, q);
                    }
                }
#pragma unroll
                for (int u = 0; u < B; u++) {
                    if (kbs[u] == 0) continue;
                    if constexpr (BWD) {
                        x[u].plain_and_mask(j);
                        g[u].plain_and_mask(j);
                        x[u].absorb_dot(g[u], total);
                    } else {
                        x[u].scale_and_mask(j, scale);
                        x[u].absorb(top, total);
                    }
                }
#pragma unroll
                for (int o = V; o < 64; o <<= 1) {
                    if constexpr (BWD) total += __shfl_xor(total, o, 64);
                    else merge_stats(top, total, __shfl_xor(top, o, 64), __shfl_xor(total, o, 64));
                }
                const float inv1 = total > 0.f ? 1.f / total : 0.f;
#pragma unroll
                for (int u = 0; u < B; u++) {
                    if (kbs[u] == 0) continue;
                    const int s = __builtin_amdgcn_readlane(my_desc.x, min(a + u, b - 1));
                    if constexpr (BWD) x[u].store_grad(g[u], out, s, kbs[u], j, q, total, scale);
                    else x[u].store(out, s, kbs[u], j, q, top, inv1);
                }
                a = b;
                continue;
            }
            int i = a;
            for (; i + B <= nfull; i += B) {  // B full blocks at a time: all loads first
                BlockScores<DT, V> x[B], g[BWD ? B : 1];
#pragma unroll
                for (int u = 0; u < B; u++) {
                    x[u].fetch_full(in, vec_mask, __builtin_amdgcn_readlane(my_desc.x, i + u), j, q);
                    if constexpr (BWD) g[u].fetch_full(in2, vec_mask, __builtin_amdgcn_readlane(my_desc.x, i + u), j, q);
                }
#pragma unroll
                for (int u = 0; u < B; u++) {
                    if constexpr (BWD) {
                        x[u].plain_and_mask(j);
                        g[u].plain_and_mask(j);
                        x[u].absorb_dot(g[u], total);
                    } else {
                        x[u].scale_and_mask(j, scale);
                        x[u].absorb(top, total);
                    }
                }
            }
            for (; i < b; i++) {
                const int s = __builtin_amdgcn_readlane(my_desc.x, i);
                const int kb = __builtin_amdgcn_readlane(my_desc.y, i) & 255;
                if (kb == 0) continue;
                BlockScores<DT, V> x, g;
                if (i < nfull) x.fetch_full(in, vec_mask, s, j, q);
                else x.fetch_any(in, vec_mask, s, kb, j, q);
                if constexpr (BWD) {
                    if (i < nfull) g.fetch_full(in2, vec_mask, s, j, q);
                    else g.fetch_any(in2, vec_mask, s, kb, j, q);
                    x.plain_and_mask(j);
                    g.plain_and_mask(j);
                    x.absorb_dot(g, total);
                } else {
                    x.scale_and_mask(j, scale);
                    x.absorb(top, total);
                }
            }
            // the lanes that share row j: lane bits above log2(V)
#pragma unroll
            for (int o = V; o < 64; o <<= 1) {
                if constexpr (BWD) total += __shfl_xor(total, o, 64);
                else merge_stats(top, total, __shfl_xor(top, o, 64), __shfl_xor(total, o, 64));
            }
            if (!whole) {
                if (q == 0) {
                    float *st = stats + (int64_t)slot * 2 * V;
                    st[j] = BWD ? 0.f : top;
                    st[V + j] = total;
                }
                slot++;
                a = b;
                continue;
            }
        } else {
            // The parts of this window left their (maximum, sum) pairs in consecutive workspace slots, whose
            // range the format keeps per slot.  Lane (j, q) merges the pairs of row j over the parts
            // q, q + 64/V, ... and the lanes of a row are merged by shuffles: a fixed order, deterministic.
            const int2 rg = slot == it.z ? range0 : range1;
            const int4 sw = make_int4(0, rg.x, rg.y, 0);  // {-, first slot, slots, -}
            const float *st = stats + (int64_t)sw.y * 2 * V;
            for (int k = q; k < sw.z; k += 64 / V) {
                if constexpr (BWD) total += st[k * 2 * V + V + j];
                else merge_stats(top, total, st[k * 2 * V + j], st[k * 2 * V + V + j]);
            }
#pragma unroll
            for (int o = V; o < 64; o <<= 1) {
                if constexpr (BWD) total += __shfl_xor(total, o, 64);
                else merge_stats(top, total, __shfl_xor(top, o, 64), __shfl_xor(total, o, 64));
            }
            slot++;
        }
        // normalised values; positions of the tile that A does not store get +0.0
        const float inv = total > 0.f ? 1.f / total : 0.f;
        int i = a;
        for (; i + B <= nfull; i += B) {
            BlockScores<DT, V> x[B], g[BWD ? B : 1];
#pragma unroll
            for (int u = 0; u < B; u++) {
                x[u].fetch_full(in, vec_mask, __builtin_amdgcn_readlane(my_desc.x, i + u), j, q);
                if constexpr (BWD) g[u].fetch_full(in2, vec_mask, __builtin_amdgcn_readlane(my_desc.x, i + u), j, q);
            }
#pragma unroll
            for (int u = 0; u < B; u++) {
                if constexpr (BWD) {
                    x[u].plain_and_mask(j);
                    g[u].plain_and_mask(j);
                    x[u].store_grad(g[u], out, __builtin_amdgcn_readlane(my_desc.x, i + u), 32, j, q, total, scale);
                } else {
                    x[u].scale_and_mask(j, scale);
                    x[u].store(out, __builtin_amdgcn_readlane(my_desc.x, i + u), 32, j, q, top, inv);
                }
            }
        }
        for (; i < b; i++) {
            const int s = __builtin_amdgcn_readlane(my_desc.x, i);
            const int kb = __builtin_amdgcn_readlane(my_desc.y, i) & 255;
            if (kb == 0) continue;
            BlockScores<DT, V> x, g;
            if (i < nfull) x.fetch_full(in, vec_mask, s, j, q);
            else x.fetch_any(in, vec_mask, s, kb, j, q);
            if constexpr (BWD) {
                if (i < nfull) g.fetch_full(in2, vec_mask, s, j, q);
                else g.fetch_any(in2, vec_mask, s, kb, j, q);
                x.plain_and_mask(j);
                g.plain_and_mask(j);
                x.store_grad(g, out, s, i < nfull ? 32 : kb, j, q, total, scale);
            } else {
                x.scale_and_mask(j, scale);
                x.store(out, s, i < nfull ? 32 : kb, j, q, top, inv);
            }
        }
        a = b;
    }
}

template <int DT, int V, bool BWD>
fs_status launch(const fs_format *f, const uint16_t *in, const uint16_t *in2, uint16_t *out, float scale, float *stats,
                 hipStream_t st)
{
    if (f->n_items == 0) return FS_OK;
    // The work list in launch order: the items that hold a part of a cut window come first (n_cut_items of
    // them), the whole windows after them, costliest first.  The second launch only needs the former.
    const int4 *items = (const int4 *)f->items_by_cost;
    const int n_items = (int)f->n_items;
    const unsigned grid = (unsigned)((n_items + kWpb - 1) / kWpb);
    k_edge_softmax<DT, V, false, BWD><<<grid, 64 * kWpb, 0, st>>>(items, n_items, (const int4 *)f->blk_desc,
                                                                  f->vec_mask, in, in2, out, stats, scale,
                                                                  (const int2 *)f->slot_range, (int)f->n_split_items);
    FS_LAUNCH_CHECK();
    const int n_cut = (int)std::min<int64_t>(f->n_cut_items, f->n_items);
    if (f->n_split_windows > 0 && n_cut > 0) {
        const unsigned grid2 = (unsigned)((n_cut + kWpb - 1) / kWpb);
        k_edge_softmax<DT, V, true, BWD><<<grid2, 64 * kWpb, 0, st>>>(items, n_cut, (const int4 *)f->blk_desc,
                                                                      f->vec_mask, in, in2, out, stats, scale,
                                                                      (const int2 *)f->slot_range, (int)f->n_split_items);
        FS_LAUNCH_CHECK();
    }
    return FS_OK;
}

template <bool BWD>
fs_status launch_any(const fs_format *f, const uint16_t *in, const uint16_t *in2, uint16_t *out, float scale, float *stats,
                     hipStream_t st)
{
    if (f->dtype == FS_F16) {
        if (f->V == 4) return launch<FS_F16, 4, BWD>(f, in, in2, out, scale, stats, st);
        if (f->V == 8) return launch<FS_F16, 8, BWD>(f, in, in2, out, scale, stats, st);
        if (f->V == 16) return launch<FS_F16, 16, BWD>(f, in, in2, out, scale, stats, st);
    } else if (f->dtype == FS_BF16) {
        if (f->V == 4) return launch<FS_BF16, 4, BWD>(f, in, in2, out, scale, stats, st);
        if (f->V == 8) return launch<FS_BF16, 8, BWD>(f, in, in2, out, scale, stats, st);
        if (f->V == 16) return launch<FS_BF16, 16, BWD>(f, in, in2, out, scale, stats, st);
    }
    return FS_ERR_UNSUPPORTED;
}

}  // namespace

fs_status fs_edge_softmax_launch(const fs_format *f, const void *d_in, void *d_out, float scale, void *d_work,
                                 hipStream_t st)
{
    return launch_any<false>(f, (const uint16_t *)d_in, nullptr, (uint16_t *)d_out, scale, (float *)d_work, st);
}

fs_status fs_edge_softmax_backward_launch(const fs_format *f, const void *d_p, const void *d_g, void *d_out, float scale,
                                          void *d_work, hipStream_t st)
{
    return launch_any<true>(f, (const uint16_t *)d_p, (const uint16_t *)d_g, (uint16_t *)d_out, scale, (float *)d_work, st);
}
