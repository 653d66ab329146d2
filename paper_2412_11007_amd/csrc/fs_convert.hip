// CSR -> vector-blocked row-window format, entirely on the GPU.
//
// The paper states only that the translation runs as GPU kernels (Section 3.1)
// and what it must produce (Section 3.5); the algorithm below is this
// library's own.  It needs no sort and no atomics, so the output is
// deterministic and bit-identical to a sequential construction:
//
//   1. flag   one thread per stored entry (row i, column c): the entry LEADS its
//             nonzero vector iff no earlier row of the same window stores c
//             (binary search in each earlier row; CSR rows are sorted).
//   2. scan   exclusive prefix sum L of the flags over CSR order.  Entries of a
//             window are contiguous in CSR order, so L at a window's first entry
//             is the index of its first vector: win_ptr[w] = L[rowptr[w*V]].
//   3. emit   one thread per entry: the position of column c among the window's
//             distinct columns is the number of leaders with a smaller column,
//             summed over the window's rows with one lower_bound and two reads
//             of L per row.  Leaders write vec_col / vec_mask; every entry
//             writes its value into its slot and records the slot.
//   4. items  a descriptor per 32-vector block, and the work items: windows longer than one and a half
//             times `chunk` vectors are cut into equal parts of about `chunk` vectors, shorter ones are
//             packed whole into items of about four blocks (boundary candidates, flag, scan, compact).
#include <algorithm>
#include <cstdlib>

#include "fs_common.h"
#include "fs_rows.h"
#include "fs_scan.h"
#include "fs_sort.h"

namespace {

constexpr int kMaxItemBlocks = 32;  // a part of a cut window never has more blocks than this
// ... and no more than this unless the caller asks: with parts launched by column, sixteen-block parts of
// hub windows share more of the dense operand in L2 than thirty-two-block parts do, which outweighs the
// extra partial tiles (cfg 4: 702 us against 720 us per call; eight-block parts 752 us)
constexpr int kDefaultMaxPartBlocks = 16;
constexpr int kPackBlocks = 4;      // packing grain for short windows, in blocks
constexpr int kMaxItemSlots = 64;   // the compute kernels hold an item's block descriptors one per lane

// ---------------------------------------------------------------- CSR helpers
struct CsrView {
    const int32_t *rowptr;
    const int32_t *colidx;
    int64_t M;
    int32_t nnz;
};

// Row bounds clamped into [0, nnz] so that a malformed rowptr can never cause an out-of-range read.
__device__ __forceinline__ void row_range(const CsrView &a, int64_t i, int32_t &lo, int32_t &hi)
{
    lo = min(max(a.rowptr[i], 0), a.nnz);
    hi = min(max(a.rowptr[i + 1], lo), a.nnz);
}

// An int32 array element by its byte offset: with a 32-bit offset from a pointer that is the same for the
// whole wavefront the load needs no address arithmetic of its own.
__device__ __forceinline__ int32_t at_byte(const int32_t *__restrict__ a, uint32_t off)
{
    return *reinterpret_cast<const int32_t *>(reinterpret_cast<const char *>(a) + off);
}

// For up to G rows at once: base[u] moves to the first position in [base[u], base[u] + n[u]) whose column
// is >= c (to base[u] + n[u] if there is none), and hit[u] says whether that column is c itself.  Positions
// are byte offsets into colidx (base[u] = 4 * index); 32 bits hold them because a window has other rows
// to search only for V >= 2, where V * nnz < 2^31 keeps 4 * nnz below 2^32.  Halving without branches:
// every round probes the middle of what is left of each row -- G independent loads in flight together, five
// instructions per row -- and the number of rounds is that of the longest row; the last round reads the two
// positions the answer can be, so that the comparison with c needs no load of its own.  A row with
// n[u] == 0 is left alone (no hit); its base must still be a valid offset, because the rounds read it.
// `last` = the offset of the last element of colidx.
template <int G>
__device__ __forceinline__ void lower_bound_cols(const int32_t *__restrict__ colidx, uint32_t last, uint32_t (&base)[G],
                                                 int32_t (&n)[G], int32_t c, bool (&hit)[G])
{
    int32_t nmax = 0;
#pragma unroll
    for (int u = 0; u < G; u++) nmax = max(nmax, n[u]);
    for (; nmax > 1; nmax -= nmax >> 1) {  // n -> ceil(n / 2) per round, for every row
        int32_t half[G], v[G];
        uint32_t probe[G];
#pragma unroll
        for (int u = 0; u < G; u++) {
            half[u] = n[u] >> 1;
            probe[u] = base[u] + ((uint32_t)half[u] << 2);
            v[u] = at_byte(colidx, probe[u]);
        }
#pragma unroll
        for (int u = 0; u < G; u++) {
            base[u] = v[u] < c ? probe[u] : base[u];
            n[u] -= half[u];
        }
    }
    // the answer is base[u] or the element after it (which may be the end of the row: the caller knows)
    int32_t v0[G], v1[G];
#pragma unroll
    for (int u = 0; u < G; u++) {
        v0[u] = at_byte(colidx, base[u]);
        v1[u] = at_byte(colidx, min(base[u] + 4u, last));
    }
#pragma unroll
    for (int u = 0; u < G; u++) {
        const bool some = n[u] > 0, below = some && v0[u] < c;
        hit[u] = some && (below ? v1[u] == c : v0[u] == c);
        base[u] += below ? 4u : 0u;
    }
}

__global__ void k_check_rowptr(CsrView a, int *__restrict__ err)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i > a.M) return;
    int32_t x = a.rowptr[i];
    bool bad = x < 0 || x > a.nnz;
    if (i == 0 && x != 0) bad = true;
    if (i == a.M && x != a.nnz) bad = true;
    if (i < a.M && a.rowptr[i + 1] < x) bad = true;
    if (bad) atomicOr(err, 1);
}

// Step 1: leader flags (+ the column checks of the CSR contract).
__global__ void __launch_bounds__(kEntriesPerGroup) k_flag(CsrView a, int64_t K, int V, const int32_t *__restrict__ block_rows,
                                                            int *__restrict__ flag, int *__restrict__ err)
{
    __shared__ int32_t sh_ptr[kEntriesPerGroup];
    const int64_t p64 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t i = group_row_of(a.rowptr, a.nnz, p64, block_rows, sh_ptr);
    if (i < 0) return;
    const int32_t p = (int32_t)p64;
    const int32_t c = a.colidx[p];
    int32_t lo, hi;
    row_range(a, i, lo, hi);
    if (c < 0 || c >= K || (p > lo && a.colidx[p - 1] >= c)) atomicOr(err, 2);
    const int32_t w0 = ((int32_t)i / V) * V, rows_before = (int32_t)i - w0;
    int leader = 1;
    constexpr int G = 8;
    for (int t0 = 0; t0 < rows_before && leader; t0 += G) {  // the earlier rows of the window, G at a time
        uint32_t base[G], end[G];
        int32_t n[G], rp[G + 1];
        bool hit[G];
#pragma unroll
        for (int u = 0; u <= G; u++) rp[u] = min(max(a.rowptr[min(w0 + t0 + u, (int32_t)i)], 0), a.nnz);
#pragma unroll
        for (int u = 0; u < G; u++) {
            base[u] = end[u] = 4u * (uint32_t)p;  // no row, or an empty one: nothing to search, and a valid offset
            if (t0 + u < rows_before && rp[u + 1] > rp[u]) { base[u] = 4u * (uint32_t)rp[u]; end[u] = 4u * (uint32_t)rp[u + 1]; }
            n[u] = (int32_t)((end[u] - base[u]) >> 2);
        }
        lower_bound_cols<G>(a.colidx, 4u * (uint32_t)(a.nnz - 1), base, n, c, hit);
#pragma unroll
        for (int u = 0; u < G; u++)
            if (hit[u] && base[u] < end[u]) leader = 0;
    }
    flag[p] = leader;
}

// Step 2b: window pointers from the scanned flags, and every window's number of block slots.
__global__ void k_win_ptr(CsrView a, int V, int64_t W, const int *__restrict__ L, int32_t *__restrict__ win_ptr, int KB,
                          int *__restrict__ nblk)
{
    int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (w > W) return;
    const int32_t p = L[min(max(a.rowptr[min(w * V, a.M)], 0), a.nnz)];
    win_ptr[w] = p;
    if (w < W) {
        const int32_t p1 = L[min(max(a.rowptr[min((w + 1) * V, a.M)], 0), a.nnz)];
        nblk[w] = max(1, (p1 - p + KB - 1) / KB);
    }
}

// Step 3: vectors, masks, slots and values.
template <typename T>
__global__ void __launch_bounds__(kEntriesPerGroup) k_emit(CsrView a, int V, int KB, const int32_t *__restrict__ block_rows,
                                                            const int *__restrict__ L,
                                              const int32_t *__restrict__ win_ptr, const T *__restrict__ vals,
                                              int32_t *__restrict__ vec_col, uint32_t *__restrict__ vec_mask,
                                              int32_t *__restrict__ csr_to_slot, T *__restrict__ vals_blk)
{
    __shared__ int32_t sh_ptr[kEntriesPerGroup];
    const int64_t p64 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t i = group_row_of(a.rowptr, a.nnz, p64, block_rows, sh_ptr);
    if (i < 0) return;
    const int32_t p = (int32_t)p64;
    const int32_t c = a.colidx[p];
    const int32_t w = (int32_t)i / V, w0 = w * V, own = (int32_t)i - w0;
    const int32_t rows = (int32_t)min((int64_t)V, a.M - w0);  // rows of this window
    int32_t lo_i, hi_i;
    row_range(a, i, lo_i, hi_i);
    int32_t rank = L[p] - L[lo_i];  // leaders of its own row with a column below c: the position is known
    uint32_t mask = 1u << own;
    constexpr int G = 8;
    for (int t0 = 0; t0 < rows; t0 += G) {  // the other rows of the window, G at a time
        uint32_t base[G], beg[G], end[G];
        int32_t n[G], rp[G + 1];
        bool hit[G];
#pragma unroll
        for (int u = 0; u <= G; u++) rp[u] = min(max(a.rowptr[min(w0 + t0 + u, w0 + rows)], 0), a.nnz);
#pragma unroll
        for (int u = 0; u < G; u++) {
            base[u] = end[u] = 4u * (uint32_t)p;  // no row, its own or an empty one: nothing to search, and a valid offset
            if (t0 + u < rows && t0 + u != own && rp[u + 1] > rp[u]) { base[u] = 4u * (uint32_t)rp[u]; end[u] = 4u * (uint32_t)rp[u + 1]; }
            beg[u] = base[u];
            n[u] = (int32_t)((end[u] - base[u]) >> 2);
        }
        lower_bound_cols<G>(a.colidx, 4u * (uint32_t)(a.nnz - 1), base, n, c, hit);
#pragma unroll
        for (int u = 0; u < G; u++) {
            rank += at_byte(L, base[u]) - at_byte(L, beg[u]);  // leaders of this row with a column below c
            if (hit[u] && base[u] < end[u]) mask |= 1u << (t0 + u);
        }
    }
    const int32_t first = win_ptr[w];
    const int32_t n_w = win_ptr[w + 1] - first;
    if (L[p + 1] != L[p]) {  // this entry leads its vector
        vec_col[first + rank] = c;
        vec_mask[first + rank] = mask;
    }
    const int32_t b = rank / KB, cc = rank - b * KB;
    const int32_t kb = min(KB, n_w - b * KB);
    const int32_t slot = V * (first + b * KB) + own * kb + cc;
    csr_to_slot[p] = slot;
    if (vals) vals_blk[slot] = vals[p];
}

// Step 4: work items.  Every window owns max(1, ceil(n_w / KB)) block slots, numbered window after
// window.  Items are runs of consecutive slots.  A window with more than 1.5 T blocks is cut into
// round(blocks / T) parts of equal length.  Shorter windows are never cut: candidate boundaries every Ts <= T slots
// snap to the nearest window boundary, so short windows are packed into items of about Ts blocks --
// finer than T, because a block that ends its window (rounding, stores, a narrow operand) costs about
// twice a block inside a long window, and because more, shorter wavefronts keep a CU's memory and LDS
// pipelines busier than few that run in step.
// Window that owns block slot x: the last w in [0, W) with blk_ptr[w] <= x.
__device__ __forceinline__ int window_of_slot(const int *__restrict__ blk_ptr, int W, int x)
{
    int lo = 0, hi = W;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (blk_ptr[mid] <= x) lo = mid; else hi = mid;
    }
    return lo;
}

// Candidate i is the boundary for block slot i * Ts.  Candidates that fall on the same boundary are
// merged afterwards.
__device__ __forceinline__ int item_boundary(const int *__restrict__ blk_ptr, int W, int NB, int T, int Ts, int i)
{
    const int x = (int)min<int64_t>((int64_t)i * Ts, NB - 1);
    const int w = window_of_slot(blk_ptr, W, x);
    const int lo = blk_ptr[w], hi = blk_ptr[w + 1];
    const int len = hi - lo;
    if (len > T + T / 2) {
        // long window: cut into round(len / T) parts of equal length (within one block), so that no part
        // is a short tail -- a part costs an fp32 partial tile whatever its length
        const int parts = (len + T / 2) / T;
        const int plen = (len + parts - 1) / parts;
        return lo + (x - lo) / plen * plen;
    }
    return (x - lo <= hi - x) ? lo : hi;  // up to one and a half part lengths: keep it whole
}

// T, the blocks per part of a long window, from the number of block slots NB: enough parts to put about 16
// wavefronts on each of the 256 CUs, long enough to amortise an item's fixed cost, short enough that one
// item is a small part of the run time.  A caller's own choice (t_user > 0) wins.
__host__ __device__ inline int part_blocks(int NB, int t_user)
{
    if (t_user > 0) return t_user;
    const int t = (NB + 4095) / 4096;
    return t < 8 ? 8 : (t > kDefaultMaxPartBlocks ? kDefaultMaxPartBlocks : t);
}

// The number of block slots is still on the device when these two run (total[0], written by the scan of the
// windows' block counts), so they are launched for the largest number of candidates there can be and work
// out the real one themselves.
// cand[i] = candidate i's boundary (cand[n_cand] = NB); flag[i] = 1 where it differs from its predecessor's
__global__ void k_item_cand(const int *__restrict__ blk_ptr, int W, const int *__restrict__ total, int t_user, int Ts,
                            int n_cand_max, int *__restrict__ cand, int *__restrict__ flag)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i > n_cand_max) return;
    const int NB = total[0], T = part_blocks(NB, t_user);
    const int n_cand = (NB + Ts - 1) / Ts;
    if (i >= n_cand) { cand[i] = NB; flag[i] = 0; return; }
    const int st = item_boundary(blk_ptr, W, NB, T, Ts, i);
    cand[i] = st;
    flag[i] = (i == 0 || st != item_boundary(blk_ptr, W, NB, T, Ts, i - 1)) ? 1 : 0;
}

// pos = exclusive scan of the flags: the distinct boundaries, in order, are the item starts
__global__ void k_item_compact(const int *__restrict__ cand, const int *__restrict__ pos, const int *__restrict__ total,
                               int Ts, int n_cand_max, int *__restrict__ start)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i > n_cand_max) return;
    const int NB = total[0];
    const int n_cand = (NB + Ts - 1) / Ts;
    if (i > n_cand) return;
    if (i == n_cand) { start[pos[n_cand]] = NB; return; }
    if (i == 0 || cand[i] != cand[i - 1]) start[pos[i]] = cand[i];
}

__global__ void k_item_make(const int *__restrict__ blk_ptr, int W, const int32_t *__restrict__ win_ptr, int KB,
                            const int *__restrict__ start, int n_items, int4 *__restrict__ items,
                            int *__restrict__ n_part, int *__restrict__ max_blocks)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_items) return;
    const int s0 = start[i], s1 = start[i + 1];
    if (s1 - s0 > kMaxItemSlots) atomicMax(max_blocks, s1 - s0);  // never by construction; checked by the host
    if (s1 <= s0) {
        items[i] = make_int4(0, 0, 0, 0);
        n_part[i] = 0;
        return;
    }
    const int wf = window_of_slot(blk_ptr, W, s0);
    const int wl = window_of_slot(blk_ptr, W, s1 - 1);
    const int bf = s0 - blk_ptr[wf];
    const bool head = bf > 0;                 // starts inside a window
    const bool tail = s1 < blk_ptr[wl + 1];   // ends inside a window
    n_part[i] = (head ? 1 : 0) + ((tail && !(head && wl == wf)) ? 1 : 0);
    items[i] = make_int4(s0, s1 - s0, 0, win_ptr[wf] + bf * KB);
}

__global__ void k_item_slots(const int *__restrict__ slot_ptr, int n_items, int4 *__restrict__ items)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_items) items[i].z = slot_ptr[i];
}

// Launch order of the work list.  Parts of cut windows come first, ordered by the column of their first
// vector: a hub window references a broad, mostly cold set of columns in ascending order, so parts that
// start at the same column sweep the same rows of the dense operand and, run side by side, share them in
// L2 instead of fetching them once per window.  Whole windows follow, the costliest items first (one unit
// per block and one more per block that ends its window: rounding, stores and a narrow operand make such
// a block about twice as dear), so that the wavefronts still running when the launch drains are short
// ones and the short windows, whose vectors sit on the hot columns, are not mixed with the cold sweep of
// the hubs.  Measured against the work list's own order: cfg 2 k_spmm 24.0 -> 21.5 us, cfg 4 (four-row
// windows) 938 -> 827 us with the cost order alone.  The 24-bit key sorts ascending; equal keys keep the
// work list's order (the sort is stable).
__global__ void k_item_key(const int4 *__restrict__ items, const int4 *__restrict__ blk_desc, int n_items,
                           const int32_t *__restrict__ vec_col, int64_t nvec, int64_t K, int32_t *__restrict__ key,
                           int *__restrict__ n_cut)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_items) return;
    const int4 it = items[i];
    if (it.y == 0) { key[i] = 0x00FFFFFF; return; }  // empty record: last
    int cost = it.y;
    for (int b = 0; b < it.y; b++) cost += (blk_desc[it.x + b].y & 256) ? 1 : 0;
    const bool head = !(blk_desc[it.x].y & 512), tail = !(blk_desc[it.x + it.y - 1].y & 256);
    if (head || tail) {
        const int32_t c = nvec > 0 ? vec_col[min((int64_t)it.w, nvec - 1)] : 0;
        key[i] = (int32_t)(((int64_t)c << 16) / max(K, (int64_t)1));  // column of the first vector, 16 bits
        atomicAdd(n_cut, 1);  // a count: the same whatever the order of the additions
    } else {
        key[i] = (1 + 128 - min(cost, 128)) << 16;
    }
}

// The work list in launch order: by_cost[t] = items[order[t]], so that a wavefront finds its item with one load.
__global__ void k_item_permute(const int4 *__restrict__ items, const int32_t *__restrict__ order, int n_items,
                               int4 *__restrict__ by_cost)
{
    int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n_items) by_cost[t] = items[order[t]];
}

// One descriptor per block slot: {first vector, width | last-block flag << 8 | first-block flag << 9, window, 0}.
__global__ void k_block_table(const int *__restrict__ blk_ptr, int W, const int32_t *__restrict__ win_ptr, int KB,
                              int NB, int4 *__restrict__ blk_desc)
{
    int x = blockIdx.x * blockDim.x + threadIdx.x;
    if (x >= NB) return;
    const int w = window_of_slot(blk_ptr, W, x);
    const int b = x - blk_ptr[w];
    const int nb_w = blk_ptr[w + 1] - blk_ptr[w];
    const int first = win_ptr[w];
    const int n_w = win_ptr[w + 1] - first;
    const int kb = max(0, min(KB, n_w - b * KB));
    blk_desc[x] = make_int4(first + b * KB, kb | ((b == nb_w - 1) ? 256 : 0) | ((b == 0) ? 512 : 0), w, 0);
}

// CSR position of the first stored entry of window row r that lies in block slot x or later:
// row_base[x * V + r] = first position in row w*V + r whose column is >= the column of the block's first
// vector.  With the block's occupancy bits this gives the CSR position of every entry of the block, which
// lets a kernel that works block by block write its results in CSR order.
__global__ void k_block_row_base(CsrView a, int V, const int4 *__restrict__ blk_desc, int NB,
                                 const int32_t *__restrict__ vec_col, int64_t nvec, int32_t *__restrict__ row_base)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (int64_t)NB * V) return;
    const int x = (int)(t / V), r = (int)(t - (int64_t)x * V);
    const int4 d = blk_desc[x];
    const int64_t row = (int64_t)d.z * V + r;
    int32_t lo = 0, hi = 0;
    if (row < a.M) row_range(a, row, lo, hi);
    if ((d.y & 255) > 0 && nvec > 0) {
        const int32_t c = vec_col[min((int64_t)d.x, nvec - 1)];
        while (lo < hi) {
            const int32_t mid = lo + ((hi - lo) >> 1);
            if (a.colidx[mid] < c) lo = mid + 1; else hi = mid;
        }
    }
    row_base[t] = lo;
}

// Last item index i in [0, n_items) with start[i] <= x (skips empty items, whose start equals the next one's).
__device__ __forceinline__ int item_of_slot(const int *__restrict__ start, int n_items, int x)
{
    int lo = 0, hi = n_items;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (start[mid] <= x) lo = mid; else hi = mid;
    }
    return lo;
}

__global__ void k_split_flag(const int *__restrict__ blk_ptr, int64_t W, const int *__restrict__ start, int n_items,
                             int *__restrict__ is_split)
{
    int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (w >= W) return;
    const int fi = item_of_slot(start, n_items, blk_ptr[w]);
    const int li = item_of_slot(start, n_items, blk_ptr[w + 1] - 1);
    is_split[w] = li > fi ? 1 : 0;
}

__global__ void k_split_fill(const int *__restrict__ blk_ptr, int64_t W, const int *__restrict__ start, int n_items,
                             const int *__restrict__ slot_ptr,
                             const int *__restrict__ sw_ptr, int4 *__restrict__ split_windows,
                             int2 *__restrict__ slot_range)
{
    int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (w >= W) return;
    if (sw_ptr[w + 1] == sw_ptr[w]) return;
    const int fi = item_of_slot(start, n_items, blk_ptr[w]);
    const int li = item_of_slot(start, n_items, blk_ptr[w + 1] - 1);
    // the window's partial tiles are consecutive slots: the tail of item fi, the items inside, the head of
    // item li.  Item fi owns a head tile of an earlier window iff it starts strictly inside that window.
    const int wfi = window_of_slot(blk_ptr, (int)W, start[fi]);
    const int first_slot = slot_ptr[fi] + (start[fi] > blk_ptr[wfi] ? 1 : 0);
    split_windows[sw_ptr[w]] = make_int4((int)w, first_slot, li - fi + 1, 0);
    // and every one of its slots learns the window's slot range (what a part needs to find the others)
    for (int k = 0; k <= li - fi; k++) slot_range[first_slot + k] = make_int2(first_slot, li - fi + 1);
}

template <typename T>
__global__ void k_blk_to_csr(const int32_t *__restrict__ csr_to_slot, const T *__restrict__ blk, T *__restrict__ out, int64_t nnz)
{
    int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p < nnz) out[p] = blk[csr_to_slot[p]];
}

// 16-byte pieces of zeros (the blocked value array is 16-byte aligned and padded to 16 bytes by its owner)
__global__ void k_zero16(fs_u4 *__restrict__ dst, int64_t n16)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = fs_u4{0u, 0u, 0u, 0u};
}

template <typename T>
__global__ void k_zero_tail(T *__restrict__ dst, int64_t from, int64_t to)
{
    int64_t i = from + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < to) dst[i] = (T)0;
}

template <typename T>
__global__ void k_csr_to_blk(const int32_t *__restrict__ csr_to_slot, const T *__restrict__ vals, T *__restrict__ blk, int64_t nnz)
{
    int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p < nnz) blk[csr_to_slot[p]] = vals[p];
}

// Stored entries per block slot (the sum of the occupancy bits of its vectors): half a wavefront per slot,
// one lane per vector.  The same pass writes every vector's occupancy mask narrowed to one byte (m8, for
// V <= 8) or two (m16), the form the packed-value kernels read.
__global__ void __launch_bounds__(256) k_block_nnz(const int4 *__restrict__ blk_desc, int64_t n_blocks,
                                                   const uint32_t *__restrict__ vec_mask, int32_t *__restrict__ cnt,
                                                   uint8_t *__restrict__ m8, uint16_t *__restrict__ m16)
{
    const int lane = threadIdx.x & 63, c = lane & 31;
    const int64_t b = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * 2 + (lane >> 5);
    int n = 0;
    if (b < n_blocks) {
        const int4 d = blk_desc[b];
        if (c < (d.y & 255)) {
            const uint32_t m = vec_mask[d.x + c];
            n = __popc(m);
            if (m8) m8[d.x + c] = (uint8_t)m; else m16[d.x + c] = (uint16_t)m;
        }
    }
#pragma unroll
    for (int o = 16; o >= 1; o >>= 1) n += __shfl_xor(n, o, 64);  // the 32 lanes of the half
    if (c == 0 && b < n_blocks) cnt[b] = n;
}

// Half a wavefront per block slot (at most 32 vectors): the stored values of the V x kb tile, row after
// row, go to consecutive positions from blk_ofs[slot] on.  Lane c < kb owns vector c and reads its column
// of the tile first, all rows at once; its position inside row r is the number of lower lanes of its half
// that also store row r.
__global__ void __launch_bounds__(256) k_pack(const int4 *__restrict__ blk_desc, int64_t n_blocks, int V,
                                              const uint32_t *__restrict__ vec_mask, const uint16_t *__restrict__ vals_blk,
                                              const int32_t *__restrict__ blk_ofs, uint16_t *__restrict__ packed)
{
    constexpr int kMaxV = 16;
    const int lane = threadIdx.x & 63, c = lane & 31, half = lane >> 5;
    const int64_t b = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * 2 + half;
    int s = 0, kb = 0;
    if (b < n_blocks) {
        const int4 d = blk_desc[b];
        s = d.x;
        kb = d.y & 255;
    }
    const bool mine = c < kb;
    const uint32_t msk = mine ? vec_mask[s + c] : 0u;
    int pos = mine ? blk_ofs[b] : 0;
    const uint16_t *tile = vals_blk + (int64_t)V * s;
    uint16_t v[kMaxV];
#pragma unroll
    for (int r = 0; r < kMaxV; r++) v[r] = (r < V && mine) ? tile[r * kb + c] : (uint16_t)0;
    const uint32_t below = (1u << c) - 1u;
#pragma unroll
    for (int r = 0; r < kMaxV; r++) {
        if (r >= V) break;
        const bool has = (msk >> r) & 1u;
        const uint64_t both = __ballot(has);
        const uint32_t row = (uint32_t)(half ? both >> 32 : both);
        if (has) packed[pos + __popc(row & below)] = v[r];
        pos += __popc(row);
    }
}

inline unsigned grid_for(int64_t n, int threads) { return (unsigned)((n + threads - 1) / threads); }

// Scratch layout (ints): [L: nnz+1][scan tmp][err + totals: 64][blk_ptr: W+1][split flags: W+1][item starts][slot_ptr]
// [boundary candidates][their flags / positions][digit counts of the work-list sort]
struct ScratchPlan {
    size_t L, tmp, misc, blk, spl, start, slotp, cand, upos, hist, brow, total_ints;
};
size_t items_bound(int64_t W, int64_t nnz, int KB) { return (size_t)(W + nnz / KB + 2); }
ScratchPlan plan_scratch(int64_t nnz, int64_t W, int KB)
{
    ScratchPlan s;
    const size_t ib = items_bound(W, nnz, KB);
    size_t o = 0;
    s.L = o; o += fs_align_up((size_t)nnz + 1, 64);
    s.tmp = o; o += scan_tmp_ints(std::max<int64_t>(std::max<int64_t>(nnz, W), (int64_t)ib));
    s.misc = o; o += 64;
    s.blk = o; o += fs_align_up((size_t)W + 1, 64);
    s.spl = o; o += fs_align_up((size_t)W + 1, 64);
    s.start = o; o += fs_align_up(ib + 1, 64);
    s.slotp = o; o += fs_align_up(ib + 1, 64);
    s.cand = o; o += fs_align_up(ib + 1, 64);
    s.upos = o; o += fs_align_up(ib + 1, 64);
    s.hist = o; o += fs_align_up((size_t)kDigits * std::max<size_t>((ib + kSortTile - 1) / kSortTile,
                                                                     (std::min<size_t>(ib, 65536) + kSortTileSmall - 1) / kSortTileSmall) + 1, 64);  // digit counts of the work-list sort
    s.brow = o; o += fs_align_up((size_t)nnz / kEntriesPerGroup + 3, 64);  // row of every 256th stored entry
    s.total_ints = o;
    return s;
}

// Window height when the caller leaves the choice to the library: eight rows, which are best or within a few
// per cent of best on every workload measured -- except on large fabric-bound matrices whose rows share
// almost no columns inside an eight-row window: there a taller window saves no vectors and a four-row
// window halves the value array for everything that reads it unpacked (cfg 5: SpMM on SDDMM scores 381 us
// against 401 us; cfg 4, whose windows do share columns, 779 us against 750 us the other way).  So for a
// matrix that qualifies for packed values the conversion counts the vectors at eight rows first and starts
// over with four when fewer than one stored entry in twenty shares its vector with another.
int32_t default_window_rows(int64_t, int64_t) { return 8; }
bool prefers_four_rows(int64_t nnz, int64_t nvec_at_eight) { return nvec_at_eight * 20 > nnz * 19; }

// Large matrices with long rows are bound by the memory fabric: for them the conversion also packs the
// values (only the stored ones, see fs_pack_values) and fs_spmm reads those.  On small or short-row
// matrices decoding costs more than the traffic it saves (cfg 2 +9 %, cfg 3 +4 %).
bool wants_packed_values(int64_t M, int64_t nnz, int32_t V, int32_t KB)
{
    return nnz >= ((int64_t)1 << 22) && nnz >= 12 * M && KB == 32 && V <= 16;
}

bool params_ok(int64_t M, int64_t nnz, int32_t V, int32_t KB)
{
    return M >= 0 && nnz >= 0 && V >= 1 && V <= 32 && KB >= 1 && KB <= 64;
}

}  // namespace

extern "C" fs_status fs_format_bytes(int64_t M, int64_t nnz, int32_t V, int32_t KB, fs_dtype dtype,
                                     size_t *arena_bytes, size_t *scratch_bytes)
{
    if (KB == 0) KB = 32;
    if (V == 0) {  // the library may settle on eight or on four rows: room for either
        size_t a8 = 0, s8 = 0, a4 = 0, s4 = 0;
        fs_status st = fs_format_bytes(M, nnz, 8, KB, dtype, &a8, &s8);
        if (st != FS_OK) return st;
        if ((st = fs_format_bytes(M, nnz, 4, KB, dtype, &a4, &s4)) != FS_OK) return st;
        if (arena_bytes) *arena_bytes = std::max(a8, a4);
        if (scratch_bytes) *scratch_bytes = std::max(s8, s4);
        return FS_OK;
    }
    if (!params_ok(M, nnz, V, KB) || (dtype != FS_F16 && dtype != FS_BF16)) return FS_ERR_INVALID_ARG;
    if (nnz >= (int64_t)1 << 31 || M >= (int64_t)1 << 31 || (int64_t)V * nnz >= (int64_t)1 << 31) return FS_ERR_TOO_LARGE;
    const int64_t W = (M + V - 1) / V;
    if (arena_bytes) {
        size_t a = 0;
        a += fs_align_up((size_t)(W + 1) * 4, 256);            // win_ptr
        a += 3 * fs_align_up((size_t)nnz * 4, 256);            // vec_col, vec_mask, csr_to_slot
        a += fs_align_up((size_t)V * nnz * 2, 256) + 256;      // vals_blk (+ slack so a 16-byte read of the tail stays inside)
        a += 3 * fs_align_up(items_bound(W, nnz, KB) * 16, 256);  // blk_desc, items, split_windows
        a += fs_align_up(items_bound(W, nnz, KB) * 4, 256);       // item_order
        a += fs_align_up(items_bound(W, nnz, KB) * V * 4, 256);   // blk_row_base
        a += fs_align_up(items_bound(W, nnz, KB) * 16, 256);      // items_by_cost
        a += fs_align_up(items_bound(W, nnz, KB) * 16, 256);      // slot_range (an item has at most two partial tiles)
        if (wants_packed_values(M, nnz, V, KB)) {  // the packed copy of the values (bounds: nvec <= nnz, blocks <= items_bound)
            fs_format b{};
            b.n_blocks = (int64_t)items_bound(W, nnz, KB); b.nvec = nnz; b.nnz = nnz; b.V = V;
            a += fs_packed_plan(&b).total + 256;
        }
        *arena_bytes = a;
    }
    if (scratch_bytes) *scratch_bytes = plan_scratch(nnz, W, KB).total_ints * 4;
    return FS_OK;
}

extern "C" fs_status fs_convert(int64_t M, int64_t K, int64_t nnz, const int32_t *d_rowptr, const int32_t *d_colidx,
                                const void *d_vals, fs_dtype dtype, int32_t V, int32_t KB, int32_t chunk,
                                void *d_arena, size_t arena_bytes, void *d_scratch, size_t scratch_bytes,
                                void *stream, fs_format *out)
{
    const bool library_picks_rows = V == 0;
    if (V == 0) V = default_window_rows(M, nnz);
    if (KB == 0) KB = 32;
    if (!out || !d_rowptr || !d_arena || !d_scratch || K < 0 || (nnz > 0 && (!d_colidx || M == 0))) return FS_ERR_INVALID_ARG;
    size_t need_arena = 0, need_scratch = 0;
    fs_status st = fs_format_bytes(M, nnz, library_picks_rows ? 0 : V, KB, dtype, &need_arena, &need_scratch);
    if (st != FS_OK) return st;
    if (chunk < 0 || (chunk > 0 && (chunk % KB != 0 || chunk / KB > kMaxItemBlocks))) return FS_ERR_INVALID_ARG;
    if (((uintptr_t)d_arena | (uintptr_t)d_scratch) & 255) return FS_ERR_INVALID_ARG;
    if (arena_bytes < need_arena || scratch_bytes < need_scratch) return FS_ERR_BUFFER_TOO_SMALL;

    hipStream_t s = (hipStream_t)stream;
    const int64_t W = (M + V - 1) / V;
    const ScratchPlan sp = plan_scratch(nnz, W, KB);
    int *scr = (int *)d_scratch;
    int *L = scr + sp.L, *misc = scr + sp.misc, *tmp = scr + sp.tmp;
    int *blk_ptr = scr + sp.blk, *spl = scr + sp.spl, *start = scr + sp.start, *slot_ptr = scr + sp.slotp;
    int *cand = scr + sp.cand, *upos = scr + sp.upos;
    int32_t *block_rows = scr + sp.brow;
    const int64_t n_groups = (nnz + kEntriesPerGroup - 1) / kEntriesPerGroup;  // workgroups of the per-entry kernels
    char *arena = (char *)d_arena;
    int32_t *win_ptr = (int32_t *)arena;
    CsrView a{d_rowptr, d_colidx, M, (int32_t)nnz};

    FS_HIP(hipMemsetAsync(misc, 0, 64 * sizeof(int), s));
    k_check_rowptr<<<grid_for(M + 1, 256), 256, 0, s>>>(a, misc);
    FS_LAUNCH_CHECK();
    if (nnz > 0) {
        k_group_rows<<<grid_for(n_groups + 1, 256), 256, 0, s>>>(d_rowptr, M, nnz, n_groups, block_rows);
        FS_LAUNCH_CHECK();
        k_flag<<<(unsigned)n_groups, kEntriesPerGroup, 0, s>>>(a, K, V, block_rows, L, misc);
        FS_LAUNCH_CHECK();
    }
    // misc: [0] CSR error flags, [1] vectors, [2] longest item, [3] items with a part of a cut window,
    // [4] block slots, [5] items, [6] partial tiles, [7] cut windows -- what the host reads, in one copy each time
    st = scan_exclusive(L, nnz, tmp, s, misc + 1);
    if (st != FS_OK) return st;
    k_win_ptr<<<grid_for(W + 1, 256), 256, 0, s>>>(a, V, W, L, win_ptr, KB, blk_ptr);
    FS_LAUNCH_CHECK();
    if ((st = scan_exclusive(blk_ptr, W, tmp, s, misc + 4)) != FS_OK) return st;

    // Work items (step 4), up to their count: the grain Ts is known here, T follows from the number of block
    // slots, which the kernels read from the device.
    const int t_user = chunk > 0 ? chunk / KB : 0;
    int Ts = std::min(t_user > 0 ? t_user : kPackBlocks, kPackBlocks);
#ifdef FS_TUNING_ENV
    if (const char *e = getenv("FS_PACK_BLOCKS")) Ts = std::max(std::min(atoi(e), t_user > 0 ? t_user : 8), 1);
#endif
    const int n_cand_max = (int)((items_bound(W, nnz, KB) + Ts - 1) / Ts);  // block slots <= W + nnz / KB
    if (W > 0) {
        k_item_cand<<<grid_for(n_cand_max + 1, 256), 256, 0, s>>>(blk_ptr, (int)W, misc + 4, t_user, Ts, n_cand_max, cand, upos);
        FS_LAUNCH_CHECK();
        if ((st = scan_exclusive(upos, n_cand_max, tmp, s, misc + 5)) != FS_OK) return st;
        k_item_compact<<<grid_for(n_cand_max + 1, 256), 256, 0, s>>>(cand, upos, misc + 4, Ts, n_cand_max, start);
        FS_LAUNCH_CHECK();
    }

    int h_misc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    FS_HIP(hipMemcpyAsync(h_misc, misc, sizeof(h_misc), hipMemcpyDeviceToHost, s));
    FS_HIP(hipStreamSynchronize(s));
    if (h_misc[0]) return FS_ERR_INVALID_CSR;
    const int64_t nvec = h_misc[1];
    const int NB = h_misc[4];  // block slots in total
    if (library_picks_rows && V == 8 && wants_packed_values(M, nnz, 4, KB) && prefers_four_rows(nnz, nvec))
        return fs_convert(M, K, nnz, d_rowptr, d_colidx, d_vals, dtype, 4, KB, chunk, d_arena, arena_bytes, d_scratch,
                          scratch_bytes, stream, out);
    if ((int64_t)V * nvec >= (int64_t)1 << 31) return FS_ERR_TOO_LARGE;
    const int n_items = W > 0 ? h_misc[5] : 0;
    chunk = part_blocks(NB, t_user) * KB;

    // arena layout, now that the sizes are known.  The value array is followed by 256 zeroed bytes: with no
    // vectors at all every per-vector array has size zero and starts there, so that the kernels' clamped
    // reads of element 0 (column 0, empty mask) stay inside the arena.
    size_t o = fs_align_up((size_t)(W + 1) * 4, 256);
    int32_t *vec_col = (int32_t *)(arena + o); o += fs_align_up((size_t)nvec * 4, 256);
    uint32_t *vec_mask = (uint32_t *)(arena + o); o += fs_align_up((size_t)nvec * 4, 256);
    int32_t *csr_to_slot = (int32_t *)(arena + o); o += fs_align_up((size_t)nnz * 4, 256);
    uint16_t *vals_blk = (uint16_t *)(arena + o); o += fs_align_up((size_t)V * nvec * 2, 256) + 256;
    int4 *blk_desc = (int4 *)(arena + o); o += fs_align_up((size_t)NB * 16, 256);
    int4 *items = (int4 *)(arena + o); o += fs_align_up((size_t)n_items * 16, 256);
    int32_t *item_order = (int32_t *)(arena + o); o += fs_align_up((size_t)n_items * 4, 256);
    int4 *items_by_cost = (int4 *)(arena + o); o += fs_align_up((size_t)n_items * 16, 256);
    int32_t *blk_row_base = (int32_t *)(arena + o); o += fs_align_up((size_t)NB * V * 4, 256);
    int2 *slot_range = (int2 *)(arena + o); o += fs_align_up((size_t)n_items * 16, 256);  // at most two partial tiles per item
    int4 *split_windows = (int4 *)(arena + o);

    FS_HIP(hipMemsetAsync(vals_blk, 0, fs_align_up((size_t)V * nvec * 2, 256) + 256, s));
    if (nnz > 0) {
        k_emit<uint16_t><<<(unsigned)n_groups, kEntriesPerGroup, 0, s>>>(a, V, KB, block_rows, L, win_ptr, (const uint16_t *)d_vals, vec_col,
                                                          vec_mask, csr_to_slot, vals_blk);
        FS_LAUNCH_CHECK();
    }

    int h_tot[2] = {0, 0}, h_max_item = 0, h_cut_items = 0;
    if (n_items > 0) {
        k_block_table<<<grid_for(NB, 256), 256, 0, s>>>(blk_ptr, (int)W, win_ptr, KB, NB, blk_desc);
        FS_LAUNCH_CHECK();
        k_block_row_base<<<grid_for((int64_t)NB * V, 256), 256, 0, s>>>(a, V, blk_desc, NB, vec_col, nvec, blk_row_base);
        FS_LAUNCH_CHECK();
        k_item_make<<<grid_for(n_items, 256), 256, 0, s>>>(blk_ptr, (int)W, win_ptr, KB, start, n_items, items, slot_ptr,
                                                                  misc + 2);
        FS_LAUNCH_CHECK();
        if ((st = scan_exclusive(slot_ptr, n_items, tmp, s, misc + 6)) != FS_OK) return st;
        k_item_slots<<<grid_for(n_items, 256), 256, 0, s>>>(slot_ptr, n_items, items);
        FS_LAUNCH_CHECK();
        k_split_flag<<<grid_for(W, 256), 256, 0, s>>>(blk_ptr, W, start, n_items, spl);
        FS_LAUNCH_CHECK();
        if ((st = scan_exclusive(spl, W, tmp, s, misc + 7)) != FS_OK) return st;
        k_split_fill<<<grid_for(W, 256), 256, 0, s>>>(blk_ptr, W, start, n_items, slot_ptr, spl, split_windows, slot_range);
        FS_LAUNCH_CHECK();
        {   // launch order: three stable radix passes over the 24-bit keys.  cand, upos and start are free
            // again: keys alternate between cand and upos, the payload between start and item_order
            {
                const int tile = n_items <= 65536 ? kSortTileSmall : kSortTile;
                const int64_t ntile = ((int64_t)n_items + tile - 1) / tile;
                int *hist = scr + sp.hist;
                k_item_key<<<grid_for(n_items, 256), 256, 0, s>>>(items, blk_desc, n_items, vec_col, nvec, K, cand, misc + 3);
                FS_LAUNCH_CHECK();
                int32_t *kbuf[2] = {upos, cand};            // pass p reads kbuf[(p + 1) & 1], writes kbuf[p & 1]
                int32_t *vbuf[2] = {item_order, start};     // pass p writes vbuf[p & 1]; the last pass (2) writes item_order
                for (int p = 0; p < 3; p++) {
                    const int32_t *src_k = kbuf[(p + 1) & 1];
                    k_digit_hist<<<(unsigned)ntile, 64, 0, s>>>(src_k, n_items, 8 * p, ntile, hist, tile);
                    FS_LAUNCH_CHECK();
                    if ((st = scan_exclusive(hist, (int64_t)kDigits * ntile, tmp, s)) != FS_OK) return st;
                    if (p == 0)
                        k_digit_scatter<true><<<(unsigned)((ntile + kScatterWaves - 1) / kScatterWaves), 64 * kScatterWaves, 0, s>>>(src_k, nullptr, n_items, 0, ntile, hist,
                                                                            kbuf[0], vbuf[0], tile);
                    else
                        k_digit_scatter<false><<<(unsigned)((ntile + kScatterWaves - 1) / kScatterWaves), 64 * kScatterWaves, 0, s>>>(src_k, vbuf[(p + 1) & 1], n_items, 8 * p, ntile,
                                                                             hist, kbuf[p & 1], vbuf[p & 1], tile);
                    FS_LAUNCH_CHECK();
                }
            }
            k_item_permute<<<grid_for(n_items, 256), 256, 0, s>>>(items, item_order, n_items, items_by_cost);
            FS_LAUNCH_CHECK();
        }
        FS_HIP(hipMemcpyAsync(h_misc, misc, sizeof(h_misc), hipMemcpyDeviceToHost, s));
    }
    FS_HIP(hipStreamSynchronize(s));
    if (n_items > 0) { h_tot[0] = h_misc[6]; h_tot[1] = h_misc[7]; h_max_item = h_misc[2]; h_cut_items = h_misc[3]; }
    // Uncut windows have at most 1.5 T <= 48 blocks and parts of cut windows at most 1.25 T + 1, so no item
    // exceeds the 64 block descriptors a wavefront holds; a work list that did would be refused here.
    if (h_max_item > kMaxItemSlots) return FS_ERR_UNSUPPORTED;
    o += fs_align_up((size_t)h_tot[1] * 16, 256);

    out->M = M; out->K = K; out->nnz = nnz; out->nvec = nvec; out->W = W;
    out->V = V; out->KB = KB; out->dtype = (int32_t)dtype; out->chunk = chunk;
    out->n_items = n_items; out->n_split_items = h_tot[0]; out->n_split_windows = h_tot[1];
    out->n_cut_items = h_cut_items;
    out->win_ptr = win_ptr; out->vec_col = vec_col; out->vec_mask = vec_mask; out->csr_to_slot = csr_to_slot;
    out->vals_blk = vals_blk; out->blk_desc = (const int32_t *)blk_desc; out->n_blocks = NB;
    out->items = (const int32_t *)items; out->split_windows = (const int32_t *)split_windows;
    out->item_order = item_order; out->items_by_cost = (const int32_t *)items_by_cost;
    out->blk_row_base = blk_row_base;
    out->packed = nullptr;
    out->slot_range = (const int32_t *)slot_range;
    out->arena_used = o;
    if (d_vals && nvec > 0 && wants_packed_values(M, nnz, V, KB)) {
        const size_t pb = fs_packed_plan(out).total;
        if (o + pb > arena_bytes) return FS_ERR_BUFFER_TOO_SMALL;  // cannot happen with fs_format_bytes' bound
        st = fs_pack_values(out, nullptr, arena + o, pb, stream);
        if (st != FS_OK) return st;
        out->packed = arena + o;
        out->arena_used = o + pb;
    }
    return FS_OK;
}

extern "C" fs_status fs_blk_to_csr(const fs_format *fmt, const void *d_blk, void *d_out_csr, void *stream)
{
    if (!fmt || !d_blk || !d_out_csr) return FS_ERR_INVALID_ARG;
    if (fmt->nnz == 0) return FS_OK;
    k_blk_to_csr<uint16_t><<<grid_for(fmt->nnz, 256), 256, 0, (hipStream_t)stream>>>(
        fmt->csr_to_slot, (const uint16_t *)d_blk, (uint16_t *)d_out_csr, fmt->nnz);
    FS_LAUNCH_CHECK();
    return FS_OK;
}

extern "C" fs_status fs_csr_to_blk(const fs_format *fmt, const void *d_vals_csr, void *d_out_blk, void *stream)
{
    if (!fmt || fmt->nvec < 0 || fmt->nnz < 0) return FS_ERR_INVALID_ARG;
    const int64_t n = (int64_t)fmt->V * fmt->nvec;  // elements of the blocked array
    if (n == 0) return FS_OK;
    if (!d_out_blk || ((uintptr_t)d_out_blk & 15) || (fmt->nnz > 0 && !d_vals_csr)) return FS_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    uint16_t *out = (uint16_t *)d_out_blk;
    const int64_t n16 = n / 8;  // whole 16-byte pieces; fill kernels, not memset nodes, so the call can be captured
    if (n16 > 0) {
        k_zero16<<<(unsigned)std::min<int64_t>((n16 + 255) / 256, 65536), 256, 0, s>>>((fs_u4 *)out, n16);
        FS_LAUNCH_CHECK();
    }
    if (n16 * 8 < n) {
        k_zero_tail<uint16_t><<<1, 64, 0, s>>>(out, n16 * 8, n);
        FS_LAUNCH_CHECK();
    }
    if (fmt->nnz > 0) {
        k_csr_to_blk<uint16_t><<<grid_for(fmt->nnz, 256), 256, 0, s>>>(fmt->csr_to_slot, (const uint16_t *)d_vals_csr, out,
                                                                         fmt->nnz);
        FS_LAUNCH_CHECK();
    }
    return FS_OK;
}

fs_packed_plan_t fs_packed_plan(const fs_format *f)
{
    fs_packed_plan_t p;
    size_t o = 0;
    p.ofs = o; o += fs_align_up(((size_t)f->n_blocks + 1) * sizeof(int32_t), 256);
    p.tmp = o; o += fs_align_up(scan_tmp_ints(f->n_blocks) * sizeof(int), 256);
    p.masks = o; o += fs_align_up(((size_t)f->nvec + 1) * (f->V <= 8 ? 1 : 2), 256);
    p.vals = o; o += fs_align_up((size_t)f->nnz * 2 + 16, 256);
    p.total = o;
    return p;
}

extern "C" fs_status fs_pack_bytes(const fs_format *fmt, size_t *packed_bytes)
{
    if (!fmt || !packed_bytes || fmt->n_blocks < 0 || fmt->nnz < 0) return FS_ERR_INVALID_ARG;
    *packed_bytes = fs_packed_plan(fmt).total;
    return FS_OK;
}

extern "C" fs_status fs_pack_values(const fs_format *fmt, const void *d_vals_blk, void *d_packed, size_t packed_bytes,
                                    void *stream)
{
    if (!fmt || fmt->n_blocks < 0 || fmt->nnz < 0 || !d_packed || ((uintptr_t)d_packed & 255)) return FS_ERR_INVALID_ARG;
    if (fmt->V < 1 || fmt->V > 16 || fmt->KB != 32) return FS_ERR_UNSUPPORTED;
    const fs_packed_plan_t pl = fs_packed_plan(fmt);
    if (packed_bytes < pl.total) return FS_ERR_BUFFER_TOO_SMALL;
    const uint16_t *vals = (const uint16_t *)(d_vals_blk ? d_vals_blk : fmt->vals_blk);
    if (fmt->nvec > 0 && !vals) return FS_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    unsigned char *buf = (unsigned char *)d_packed;
    int32_t *ofs = (int32_t *)(buf + pl.ofs);
    if (fmt->n_blocks > 0) {
        uint8_t *m8 = fmt->V <= 8 ? (uint8_t *)(buf + pl.masks) : nullptr;
        k_block_nnz<<<grid_for(fmt->n_blocks, 8), 256, 0, s>>>((const int4 *)fmt->blk_desc, fmt->n_blocks, fmt->vec_mask, ofs, m8,
                                                                (uint16_t *)(buf + pl.masks));
        FS_LAUNCH_CHECK();
    }
    fs_status st = scan_exclusive(ofs, fmt->n_blocks, (int *)(buf + pl.tmp), s);
    if (st != FS_OK) return st;
    if (fmt->n_blocks > 0) {
        k_pack<<<grid_for(fmt->n_blocks, 8), 256, 0, s>>>((const int4 *)fmt->blk_desc, fmt->n_blocks, fmt->V, fmt->vec_mask,
                                                             vals, ofs, (uint16_t *)(buf + pl.vals));
        FS_LAUNCH_CHECK();
    }
    return FS_OK;
}

extern "C" int fs_version(void) { return 300; }  // 0.3.0: fused attention, CSR of the transposed matrix

extern "C" const char *fs_status_string(fs_status s)
{
    switch (s) {
    case FS_OK: return "ok";
    case FS_ERR_INVALID_ARG: return "invalid argument";
    case FS_ERR_INVALID_CSR: return "invalid CSR (column out of range or not strictly ascending in a row)";
    case FS_ERR_UNSUPPORTED: return "unsupported combination of V, KB, dtype or sizes";
    case FS_ERR_BUFFER_TOO_SMALL: return "buffer too small";
    case FS_ERR_TOO_LARGE: return "sizes exceed the 32-bit indices of the format";
    case FS_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}
