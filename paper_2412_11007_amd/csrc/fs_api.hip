// Argument checking for the compute entry points of the C ABI; the kernels live in
// fs_spmm.hip / fs_sddmm.hip / fs_softmax.hip / fs_attention.hip, conversion and utilities in fs_convert.hip.
#include <algorithm>
#include <mutex>

#include "fs_common.h"
#include "fs_tile.h"

// Workspace of fs_spmm_static: the fp32 partial tiles of cut windows live here instead of in a caller's
// buffer.  One copy per GPU, held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; the device address it yields (per device) is what the kernels are given.
#define FS_STATIC_WORK_BYTES ((size_t)32 << 20)
static __device__ __align__(256) unsigned char scratch[FS_STATIC_WORK_BYTES];

namespace {

constexpr int FS_MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[FS_MAX_DEVICES];  // device address of `scratch` on each GPU, looked up on first use

// Address of the current device's copy of `scratch`.
fs_status static_workspace(void **out)
{
    int dev = -1;
    FS_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= FS_MAX_DEVICES) return FS_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        FS_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return FS_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return FS_OK;
}

bool format_ok(const fs_format *f)
{
    return f && f->M >= 0 && f->K >= 0 && f->nvec >= 0 && f->n_items >= 0 && f->n_items < ((int64_t)1 << 31) &&
           (f->n_items == 0 || (f->items && f->items_by_cost && f->win_ptr && f->blk_desc)) && (f->nvec == 0 || (f->vec_col && f->vec_mask));
}

bool kernels_support(const fs_format *f)
{
    return (f->V == 4 || f->V == 8 || f->V == 16) && f->KB == 32 && (f->dtype == FS_F16 || f->dtype == FS_BF16) &&
           f->chunk > 0 && f->chunk % 32 == 0;
}

bool aligned(const void *p, size_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

__global__ void __launch_bounds__(256) k_copy16(uint4 *__restrict__ dst, const uint4 *__restrict__ src, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// Measurement aid: the buffer is cut into 16 KiB chunks; in every repeat a workgroup reads one chunk (a
// wavefront 1 KiB per load instruction), a different one each time but always one whose index is congruent to
// its own modulo 8 -- workgroups go to the XCDs round robin, so an XCD keeps re-reading its own eighth of the
// buffer, which its L2 holds after the first sweep, while a CU never finds a chunk in its L1 again.
__global__ void __launch_bounds__(256) k_read16(const fs_u4 *__restrict__ src, unsigned n_chunks, int repeats, uint32_t *__restrict__ sink)
{
    uint32_t x = 0;
    for (int r = 0; r < repeats; r++) {
        const unsigned chunk = (blockIdx.x + 8u * 37u * (unsigned)r) % n_chunks;  // n_chunks is a multiple of 8
        const fs_u4 *p = src + (size_t)chunk * 1024 + threadIdx.x;
        fs_u4 v[4];
#pragma unroll
        for (int u = 0; u < 4; u++) v[u] = p[u * 256];
#pragma unroll
        for (int u = 0; u < 4; u++) x ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = x;
}

// Measurement aid: nothing but the gather of fs_spmm, in fs_spmm's own launch order.  One wavefront per work
// item, four per workgroup, placed like the SpMM kernel's; per block it reads the column indices and loads
// the rows of B they name exactly as that kernel does -- 16 bytes per lane, 16 lanes per 128-column piece of a
// row, eight wave-wide loads per 32 vectors and pass -- and folds what it read into one word per lane, written
// once at the end.
__global__ void __launch_bounds__(256) k_gather_probe(const int4 *__restrict__ items, int n_items, const int4 *__restrict__ blk_desc,
                                                      const int32_t *__restrict__ vec_col, int nvec,
                                                      const uint16_t *__restrict__ B, int64_t ldb, int N, int nbx, int slice, int n_swz,
                                                      uint32_t *__restrict__ sink)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int pass = blockIdx.x / nbx, bx = blockIdx.x - pass * nbx;
    const int turn = fs_launch_turn<4>(bx, slice, n_swz) + wave;
    uint32_t x = 0;
    if (turn < n_items) {
        const int4 it = items[turn];
        const int col = pass * 128 + (lane & 15) * 8;
        const int64_t colb = col < N ? col : 0;
        for (int b = 0; b < it.y; b++) {
            const int4 d = blk_desc[it.x + b];
            const int kb = d.y & 255;
            if (kb == 0) continue;
            const int my = vec_col[min(d.x + min(lane & 31, kb - 1), nvec - 1)];
            fs_u4 v[8];
#pragma unroll
            for (int u = 0; u < 8; u++) {
                const int r = __shfl(my, u * 4 + (lane >> 4), 64);
                v[u] = *reinterpret_cast<const fs_u4 *>(B + (int64_t)r * ldb + colb);
            }
#pragma unroll
            for (int u = 0; u < 8; u++) x ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
        }
    }
    sink[((size_t)blockIdx.x * 256 + threadIdx.x) & (1024 * 256 - 1)] = x;  // any slot: the word only keeps the loads alive
}

}  // namespace

extern "C" fs_status fs_gather_probe(const fs_format *fmt, const void *d_B, int64_t N, int64_t ldb, void *d_sink,
                                     size_t sink_bytes, void *stream)
{
    if (!format_ok(fmt) || N < 0 || ldb < N) return FS_ERR_INVALID_ARG;
    if (!kernels_support(fmt)) return FS_ERR_UNSUPPORTED;
    if (N == 0 || fmt->n_blocks == 0 || fmt->nvec == 0) return FS_OK;
    if (!d_B || !d_sink || N % 8 || ldb % 8 || !aligned(d_B, 16) || !aligned(d_sink, 4)) return FS_ERR_INVALID_ARG;
    if (sink_bytes < (size_t)1024 * 256 * sizeof(uint32_t)) return FS_ERR_BUFFER_TOO_SMALL;
    const fs_launch_geometry geo = fs_launch_geometry_for(fmt, 4);
    const int64_t nblocks = (int64_t)geo.nbx * ((N + 127) / 128);
    if (nblocks >= ((int64_t)1 << 31)) return FS_ERR_TOO_LARGE;
    k_gather_probe<<<(unsigned)nblocks, 256, 0, (hipStream_t)stream>>>((const int4 *)fmt->items_by_cost, (int)fmt->n_items,
                                                                        (const int4 *)fmt->blk_desc, fmt->vec_col, (int)fmt->nvec,
                                                                        (const uint16_t *)d_B, ldb, (int)N, geo.nbx, geo.slice,
                                                                        geo.n_swz, (uint32_t *)d_sink);
    FS_LAUNCH_CHECK();
    return FS_OK;
}

extern "C" fs_status fs_spmm_workspace_bytes(const fs_format *fmt, int64_t N, size_t *work_bytes)
{
    if (!format_ok(fmt) || !work_bytes || N < 0) return FS_ERR_INVALID_ARG;
    *work_bytes = (size_t)fmt->n_split_items * (size_t)fmt->V * (size_t)N * sizeof(float);
    return FS_OK;
}

extern "C" fs_status fs_spmm_timed(const fs_format *fmt, const void *d_vals, const void *d_B, int64_t N, int64_t ldb,
                                   void *d_C, int64_t ldc, void *d_work, size_t work_bytes, void *stream,
                                   void *ev_before_main, void *ev_after_main)
{
    if (!format_ok(fmt) || N < 0 || ldb < N || ldc < N) return FS_ERR_INVALID_ARG;
    if (!kernels_support(fmt)) return FS_ERR_UNSUPPORTED;
    if (N == 0 || fmt->M == 0) return FS_OK;
    if (!d_B || !d_C) return FS_ERR_INVALID_ARG;
    if (N % 8 || ldb % 8 || ldc % 8 || !aligned(d_B, 16) || !aligned(d_C, 16)) return FS_ERR_INVALID_ARG;
    if (N >= ((int64_t)1 << 24) || ldc >= ((int64_t)1 << 24) || ldb >= ((int64_t)1 << 30)) return FS_ERR_TOO_LARGE;
    const void *vals = d_vals ? d_vals : fmt->vals_blk;
    if (fmt->nvec > 0 && (!vals || !aligned(vals, 16))) return FS_ERR_INVALID_ARG;
    size_t need = 0;
    fs_spmm_workspace_bytes(fmt, N, &need);
    if (need > 0 && (!d_work || !aligned(d_work, 16))) return FS_ERR_INVALID_ARG;
    if (work_bytes < need) return FS_ERR_BUFFER_TOO_SMALL;
    return fs_spmm_launch(fmt, d_vals, d_B, N, ldb, d_C, ldc, d_work, (hipStream_t)stream,
                          (hipEvent_t)ev_before_main, (hipEvent_t)ev_after_main);
}

extern "C" fs_status fs_spmm_packed(const fs_format *fmt, const void *d_packed, const void *d_B, int64_t N, int64_t ldb,
                                    void *d_C, int64_t ldc, void *d_work, size_t work_bytes, void *stream)
{
    if (!format_ok(fmt) || N < 0 || ldb < N || ldc < N) return FS_ERR_INVALID_ARG;
    if (!kernels_support(fmt)) return FS_ERR_UNSUPPORTED;
    if (N == 0 || fmt->M == 0) return FS_OK;
    if (!d_B || !d_C || !d_packed || !aligned(d_packed, 256)) return FS_ERR_INVALID_ARG;
    if (N % 8 || ldb % 8 || ldc % 8 || !aligned(d_B, 16) || !aligned(d_C, 16)) return FS_ERR_INVALID_ARG;
    if (N >= ((int64_t)1 << 24) || ldc >= ((int64_t)1 << 24) || ldb >= ((int64_t)1 << 30)) return FS_ERR_TOO_LARGE;
    size_t need = 0;
    fs_spmm_workspace_bytes(fmt, N, &need);
    if (need > 0 && (!d_work || !aligned(d_work, 16))) return FS_ERR_INVALID_ARG;
    if (work_bytes < need) return FS_ERR_BUFFER_TOO_SMALL;
    return fs_spmm_packed_launch(fmt, d_packed, d_B, N, ldb, d_C, ldc, d_work, (hipStream_t)stream, nullptr, nullptr);
}

extern "C" fs_status fs_spmm(const fs_format *fmt, const void *d_vals, const void *d_B, int64_t N, int64_t ldb,
                             void *d_C, int64_t ldc, void *d_work, size_t work_bytes, void *stream)
{
    return fs_spmm_timed(fmt, d_vals, d_B, N, ldb, d_C, ldc, d_work, work_bytes, stream, nullptr, nullptr);
}

extern "C" fs_status fs_spmm_static(const fs_format *fmt, const void *d_vals, const void *d_B, int64_t N, int64_t ldb,
                                    void *d_C, int64_t ldc, void *stream)
{
    size_t need = 0;
    const fs_status s = fs_spmm_workspace_bytes(fmt, N, &need);
    if (s != FS_OK) return s;
    if (need > FS_STATIC_WORK_BYTES) return FS_ERR_TOO_LARGE;
    void *work = nullptr;
    if (need > 0) {  // partial tiles are written whole before they are read: nothing to clear
        const fs_status a = static_workspace(&work);
        if (a != FS_OK) return a;
    }
    return fs_spmm_timed(fmt, d_vals, d_B, N, ldb, d_C, ldc, work, need, stream, nullptr, nullptr);
}

extern "C" fs_status fs_sddmm(const fs_format *fmt, const void *d_X, int64_t ldx, const void *d_Y, int64_t ldy,
                              int64_t d, void *d_out_blk, void *d_out_csr, void *stream)
{
    if (!format_ok(fmt) || d < 0 || ldx < d || ldy < d) return FS_ERR_INVALID_ARG;
    if (!kernels_support(fmt)) return FS_ERR_UNSUPPORTED;
    if (fmt->nvec == 0) return FS_OK;
    if (!d_X || !d_Y || (!d_out_blk && !d_out_csr)) return FS_ERR_INVALID_ARG;
    if (d % 8 || ldx % 8 || ldy % 8 || !aligned(d_X, 16) || !aligned(d_Y, 16) || !aligned(d_out_blk, 16) ||
        !aligned(d_out_csr, 2))
        return FS_ERR_INVALID_ARG;
    if (d_out_csr && !fmt->blk_row_base) return FS_ERR_INVALID_ARG;
    if (d >= ((int64_t)1 << 24)) return FS_ERR_TOO_LARGE;
    return fs_sddmm_launch(fmt, d_X, ldx, d_Y, ldy, d, d_out_blk, d_out_csr, (hipStream_t)stream);
}

extern "C" fs_status fs_edge_softmax_workspace_bytes(const fs_format *fmt, size_t *work_bytes)
{
    if (!format_ok(fmt) || !work_bytes) return FS_ERR_INVALID_ARG;
    *work_bytes = (size_t)fmt->n_split_items * 2 * (size_t)fmt->V * sizeof(float);
    return FS_OK;
}

extern "C" fs_status fs_edge_softmax(const fs_format *fmt, const void *d_in_blk, void *d_out_blk, float scale,
                                     void *d_work, size_t work_bytes, void *stream)
{
    if (!format_ok(fmt) || !(scale == scale) || scale - scale != 0.f) return FS_ERR_INVALID_ARG;  // NaN, infinity
    if (!kernels_support(fmt)) return FS_ERR_UNSUPPORTED;
    if (fmt->nvec == 0) return FS_OK;
    if (!d_in_blk || !d_out_blk) return FS_ERR_INVALID_ARG;
    size_t need = 0;
    fs_edge_softmax_workspace_bytes(fmt, &need);
    if (need > 0 && (!d_work || !aligned(d_work, 4))) return FS_ERR_INVALID_ARG;
    if (work_bytes < need) return FS_ERR_BUFFER_TOO_SMALL;
    return fs_edge_softmax_launch(fmt, d_in_blk, d_out_blk, scale, d_work, (hipStream_t)stream);
}

extern "C" fs_status fs_edge_softmax_backward(const fs_format *fmt, const void *d_p_blk, const void *d_g_blk, float scale,
                                              void *d_out_blk, void *d_work, size_t work_bytes, void *stream)
{
    if (!format_ok(fmt) || !(scale == scale) || scale - scale != 0.f) return FS_ERR_INVALID_ARG;  // NaN, infinity
    if (!kernels_support(fmt)) return FS_ERR_UNSUPPORTED;
    if (fmt->nvec == 0) return FS_OK;
    if (!d_p_blk || !d_g_blk || !d_out_blk) return FS_ERR_INVALID_ARG;
    size_t need = 0;
    fs_edge_softmax_workspace_bytes(fmt, &need);
    if (need > 0 && (!d_work || !aligned(d_work, 4))) return FS_ERR_INVALID_ARG;
    if (work_bytes < need) return FS_ERR_BUFFER_TOO_SMALL;
    return fs_edge_softmax_backward_launch(fmt, d_p_blk, d_g_blk, d_out_blk, scale, d_work, (hipStream_t)stream);
}

extern "C" fs_status fs_attention_workspace_bytes(const fs_format *fmt, int64_t N, size_t *work_bytes)
{
    if (!format_ok(fmt) || !work_bytes || N < 0) return FS_ERR_INVALID_ARG;
    // per part of a cut window: an fp32 V x N tile, and a maximum and a sum per row
    *work_bytes = (size_t)fmt->n_split_items * (size_t)fmt->V * ((size_t)N + 2) * sizeof(float);
    return FS_OK;
}

static fs_status attention_call(const fs_format *fmt, const void *d_X, int64_t ldx, const void *d_Y, int64_t ldy,
                                int64_t d, float scale, const void *d_H, int64_t N, int64_t ldh, void *d_out,
                                int64_t ldo, void *d_work, size_t work_bytes, void *stream, bool softmax)
{
    if (!format_ok(fmt) || d < 0 || N < 0 || ldx < d || ldy < d || ldh < N || ldo < N) return FS_ERR_INVALID_ARG;
    if (!(scale == scale) || scale - scale != 0.f) return FS_ERR_INVALID_ARG;  // NaN, infinity
    if (!kernels_support(fmt) || d > 128) return FS_ERR_UNSUPPORTED;
    if (N == 0 || fmt->M == 0) return FS_OK;
    if (!d_X || !d_Y || !d_H || !d_out) return FS_ERR_INVALID_ARG;
    if (d % 8 || N % 8 || ldx % 8 || ldy % 8 || ldh % 8 || ldo % 8 || !aligned(d_X, 16) || !aligned(d_Y, 16) ||
        !aligned(d_H, 16) || !aligned(d_out, 16))
        return FS_ERR_INVALID_ARG;
    if (N >= ((int64_t)1 << 24) || ldo >= ((int64_t)1 << 24)) return FS_ERR_TOO_LARGE;
    // the kernel addresses X, Y and H with 32-bit byte offsets formed by a 24-bit multiply
    const int64_t lim24 = (int64_t)1 << 24, lim32 = (int64_t)1 << 32;
    if (fmt->M >= lim24 || fmt->K >= lim24 || ldx * 2 >= lim24 || ldy * 2 >= lim24 || ldh * 2 >= lim24 ||
        fmt->M * ldx * 2 >= lim32 || fmt->K * ldy * 2 >= lim32 || fmt->K * ldh * 2 >= lim32)
        return FS_ERR_UNSUPPORTED;
    size_t need = 0;
    fs_attention_workspace_bytes(fmt, N, &need);
    if (need > 0 && (!d_work || !aligned(d_work, 16))) return FS_ERR_INVALID_ARG;
    if (work_bytes < need) return FS_ERR_BUFFER_TOO_SMALL;
    return fs_attention_launch(fmt, d_X, ldx, d_Y, ldy, d, scale, d_H, N, ldh, d_out, ldo, d_work, (hipStream_t)stream,
                               softmax);
}

extern "C" fs_status fs_attention(const fs_format *fmt, const void *d_X, int64_t ldx, const void *d_Y, int64_t ldy,
                                  int64_t d, float scale, const void *d_H, int64_t N, int64_t ldh, void *d_out,
                                  int64_t ldo, void *d_work, size_t work_bytes, void *stream)
{
    return attention_call(fmt, d_X, ldx, d_Y, ldy, d, scale, d_H, N, ldh, d_out, ldo, d_work, work_bytes, stream, true);
}

extern "C" fs_status fs_sddmm_spmm(const fs_format *fmt, const void *d_X, int64_t ldx, const void *d_Y, int64_t ldy,
                                   int64_t d, float scale, const void *d_H, int64_t N, int64_t ldh, void *d_out,
                                   int64_t ldo, void *d_work, size_t work_bytes, void *stream)
{
    return attention_call(fmt, d_X, ldx, d_Y, ldy, d, scale, d_H, N, ldh, d_out, ldo, d_work, work_bytes, stream, false);
}

extern "C" fs_status fs_read_bytes(const void *d_src, size_t bytes, int32_t repeats, void *d_sink, size_t sink_bytes, void *stream)
{
    if (!d_src || !d_sink || bytes % (8 * 16384) || repeats < 1 || !aligned(d_src, 16) || !aligned(d_sink, 4)) return FS_ERR_INVALID_ARG;
    if (bytes == 0) return FS_OK;
    if (bytes / 16384 > 0xFFFFFFFFu) return FS_ERR_TOO_LARGE;
    const unsigned grid = 256 * 8;  // eight workgroups of four wavefronts on each of the 256 CUs
    if (sink_bytes < (size_t)grid * 256 * sizeof(uint32_t)) return FS_ERR_BUFFER_TOO_SMALL;
    k_read16<<<grid, 256, 0, (hipStream_t)stream>>>((const fs_u4 *)d_src, (unsigned)(bytes / 16384), repeats, (uint32_t *)d_sink);
    FS_LAUNCH_CHECK();
    return FS_OK;
}

extern "C" fs_status fs_copy_bytes(void *d_dst, const void *d_src, size_t bytes, void *stream)
{
    if (!d_dst || !d_src || bytes % 16 || !aligned(d_dst, 16) || !aligned(d_src, 16)) return FS_ERR_INVALID_ARG;
    if (bytes == 0) return FS_OK;
    const size_t n16 = bytes / 16;
    const unsigned grid = (unsigned)std::min<size_t>((n16 + 255) / 256, 256 * 32);
    k_copy16<<<grid, 256, 0, (hipStream_t)stream>>>((uint4 *)d_dst, (const uint4 *)d_src, n16);
    FS_LAUNCH_CHECK();
    return FS_OK;
}
