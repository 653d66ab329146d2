// Shared host/device helpers of the HIP library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "flashsparse.h"
#include "flashsparse_measure.h"

#define FS_WAVE 64

// Check a HIP runtime call inside a function returning fs_status.
#define FS_HIP(call)                          \
    do {                                      \
        hipError_t e__ = (call);              \
        if (e__ != hipSuccess) {              \
            (void)hipGetLastError();          \
            return FS_ERR_HIP;                \
        }                                     \
    } while (0)

// After a kernel launch.
#define FS_LAUNCH_CHECK()                     \
    do {                                      \
        if (hipGetLastError() != hipSuccess)  \
            return FS_ERR_HIP;                \
    } while (0)

static inline size_t fs_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Vector types for the matrix-core builtins.
typedef _Float16 fs_h8 __attribute__((ext_vector_type(8)));
typedef __bf16 fs_b8 __attribute__((ext_vector_type(8)));
typedef short fs_s4 __attribute__((ext_vector_type(4)));
typedef float fs_f4 __attribute__((ext_vector_type(4)));
// Native 16-byte vector: unlike HIP's uint4 class it is copied by plain loads and stores, which keeps
// arrays of it in registers.
typedef uint32_t fs_u4 __attribute__((ext_vector_type(4)));

// 16 bytes of raw 16-bit elements; reinterpreted per element type at the MFMA call.
union fs_frag {
    fs_u4 u;
    fs_h8 h;
    fs_b8 b;
    uint16_t e[8];
    fs_s4 s[2];
};

// fp32 -> 16-bit storage, round to nearest even.
__device__ __forceinline__ uint16_t fs_f32_to_f16_bits(float x)
{
    _Float16 h = (_Float16)x;  // v_cvt_f16_f32, RNE
    return __builtin_bit_cast(uint16_t, h);
}
__device__ __forceinline__ uint16_t fs_f32_to_bf16_bits(float x)
{
    uint32_t u = __builtin_bit_cast(uint32_t, x);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);  // quiet NaN
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
template <int DT>
__device__ __forceinline__ uint16_t fs_round_bits(float x)
{
    return DT == FS_BF16 ? fs_f32_to_bf16_bits(x) : fs_f32_to_f16_bits(x);
}

// Two fp32 values -> two 16-bit storage values in one dword (a in the low half), round to nearest even.
// Written as a vector conversion so that it becomes a single v_cvt_pk_{f16,bf16}_f32.
typedef float fs_f2 __attribute__((ext_vector_type(2)));
typedef _Float16 fs_h2 __attribute__((ext_vector_type(2)));
typedef __bf16 fs_b2 __attribute__((ext_vector_type(2)));
template <int DT>
__device__ __forceinline__ uint32_t fs_pack2(float a, float b)
{
    const fs_f2 v = {a, b};
    if constexpr (DT == FS_BF16)
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, fs_b2));
    else
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, fs_h2));
}

// D(16x16 fp32) += A(16x32) * B(32x16) on the matrix core.
// Operand layout (lane l, r = l % 16, g = l / 16):
//   a holds A[r][8g .. 8g+7], b holds B[8g .. 8g+7][r], acc[e] is D[4g+e][r].
template <int DT>
__device__ __forceinline__ fs_f4 fs_mfma_16x16x32(const fs_frag &a, const fs_frag &b, fs_f4 acc)
{
    if constexpr (DT == FS_BF16)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.b, b.b, acc, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(a.h, b.h, acc, 0, 0, 0);
}

// Layout of the caller's buffer behind fs_pack_values / fs_spmm_packed (byte offsets, each 256-byte
// aligned): first value of every block slot (n_blocks + 1 int32), scratch of the prefix sum, the
// per-vector occupancy masks narrowed to one byte (V <= 8) or two, the stored values (nnz 16-bit
// elements and 16 spare bytes, because a lane reads 16 bytes from any element on).
struct fs_packed_plan_t {
    size_t ofs, tmp, masks, vals, total;
};
fs_packed_plan_t fs_packed_plan(const fs_format *fmt);

// internal entry points of the per-operator translation units
fs_status fs_spmm_packed_launch(const fs_format *fmt, const void *d_packed, const void *d_B, int64_t N, int64_t ldb,
                                void *d_C, int64_t ldc, void *d_work, hipStream_t stream, hipEvent_t ev0, hipEvent_t ev1);
fs_status fs_spmm_launch(const fs_format *fmt, const void *d_vals, const void *d_B, int64_t N, int64_t ldb,
                         void *d_C, int64_t ldc, void *d_work, hipStream_t stream, hipEvent_t ev0, hipEvent_t ev1);
fs_status fs_sddmm_launch(const fs_format *fmt, const void *d_X, int64_t ldx, const void *d_Y, int64_t ldy,
                          int64_t d, void *d_out_blk, void *d_out_csr, hipStream_t stream);
fs_status fs_attention_launch(const fs_format *fmt, const void *d_X, int64_t ldx, const void *d_Y, int64_t ldy, int64_t d,
                              float scale, const void *d_H, int64_t N, int64_t ldh, void *d_out, int64_t ldo,
                              void *d_work, hipStream_t stream, bool softmax);
fs_status fs_edge_softmax_launch(const fs_format *fmt, const void *d_in_blk, void *d_out_blk, float scale,
                                 void *d_work, hipStream_t stream);
fs_status fs_edge_softmax_backward_launch(const fs_format *fmt, const void *d_p_blk, const void *d_g_blk, void *d_out_blk,
                                          float scale, void *d_work, hipStream_t st);
