/*
 * The library from plain C: no Python, no torch, only the C ABI of flashsparse.h and the HIP runtime
 * for device memory.  Converts a small CSR matrix, runs SpMM and SDDMM, and checks both against loops
 * on the host.  All values are small multiples of 1/2, so every product and sum is exact in fp32 and
 * in fp16 and the comparison is bit for bit.  Also: the CSR of the transposed matrix (bit for bit against
 * a counting placement on the host) and the fused attention call (against a double-precision loop, to
 * 1e-2 of sum a|h|).  Exit code 0 = everything matched.
 *
 * Build (done by paper_2412_11007_amd/build.py):
 *   gcc -std=c99 -D__HIP_PLATFORM_AMD__ -I/opt/rocm/include -Iinclude tests/c_abi_example.c \
 *       -Lpaper_2412_11007_amd -lflashsparse_hip -L/opt/rocm/lib -lamdhip64 -o tests/c_abi_example
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "flashsparse.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %d at line %d\n", (int)e_, __LINE__); return 2; } } while (0)
#define CHECK_FS(x) do { fs_status s_ = (x); if (s_ != FS_OK) { printf("%s at line %d\n", fs_status_string(s_), __LINE__); return 3; } } while (0)

/* fp16 bits of a multiple of 1/2 with magnitude below 2048 (exact), and back */
static uint16_t half_bits(double v)
{
    uint16_t sign = 0;
    int e = 0;
    double m;
    if (v == 0) return 0;
    if (v < 0) { sign = 0x8000; v = -v; }
    m = v;
    while (m >= 2.0) { m /= 2.0; e++; }
    while (m < 1.0) { m *= 2.0; e--; }
    return (uint16_t)(sign | ((e + 15) << 10) | (uint16_t)((m - 1.0) * 1024.0));
}
static double half_value(uint16_t h)
{
    int e = (h >> 10) & 31, f = h & 1023;
    double v = e == 0 ? f / 1024.0 / 16384.0 : (1.0 + f / 1024.0);
    int i;
    if (e > 0) { for (i = 15; i < e; i++) v *= 2.0; for (i = e; i < 15; i++) v /= 2.0; }
    return (h & 0x8000) ? -v : v;
}

int main(void)
{
    enum { M = 43, K = 57, N = 24, D = 16 };
    static const double vals_set[6] = {-2.0, -1.0, -0.5, 0.5, 1.0, 1.5};
    int32_t rowptr[M + 1], *colidx;
    uint16_t *vals, B[K * N], X[M * D], Y[K * D];
    int i, j, p, nnz = 0, t;

    /* pattern: row i stores columns c with (7*i + 3*c) % 11 < 2, plus one long row */
    rowptr[0] = 0;
    for (i = 0; i < M; i++) {
        for (j = 0; j < K; j++) if (i == 20 || (7 * i + 3 * j) % 11 < 2) nnz++;
        rowptr[i + 1] = nnz;
    }
    colidx = (int32_t *)malloc(sizeof(int32_t) * nnz);
    vals = (uint16_t *)malloc(sizeof(uint16_t) * nnz);
    for (i = 0, p = 0; i < M; i++)
        for (j = 0; j < K; j++)
            if (i == 20 || (7 * i + 3 * j) % 11 < 2) { colidx[p] = j; vals[p] = half_bits(vals_set[(i + 2 * j) % 6]); p++; }
    for (i = 0; i < K * N; i++) B[i] = half_bits((double)((i * 5) % 9 - 4));
    for (i = 0; i < M * D; i++) X[i] = half_bits((double)((i * 3) % 5 - 2));
    for (i = 0; i < K * D; i++) Y[i] = half_bits((double)((i * 5) % 7 - 3) / 2.0);

    /* device buffers */
    int32_t *d_rowptr, *d_colidx;
    uint16_t *d_vals, *d_B, *d_C, *d_X, *d_Y, *d_scores, *d_scores_csr;
    void *d_arena, *d_scratch, *d_work = NULL;
    size_t arena_bytes, scratch_bytes, work_bytes;
    fs_format fmt;
    CHECK_FS(fs_format_bytes(M, nnz, 0, 0, FS_F16, &arena_bytes, &scratch_bytes));
    CHECK_HIP(hipMalloc((void **)&d_rowptr, sizeof rowptr));
    CHECK_HIP(hipMalloc((void **)&d_colidx, sizeof(int32_t) * nnz));
    CHECK_HIP(hipMalloc((void **)&d_vals, sizeof(uint16_t) * nnz));
    CHECK_HIP(hipMalloc((void **)&d_B, sizeof B));
    CHECK_HIP(hipMalloc((void **)&d_C, sizeof(uint16_t) * M * N));
    CHECK_HIP(hipMalloc((void **)&d_X, sizeof X));
    CHECK_HIP(hipMalloc((void **)&d_Y, sizeof Y));
    CHECK_HIP(hipMalloc(&d_arena, arena_bytes));
    CHECK_HIP(hipMalloc(&d_scratch, scratch_bytes));
    CHECK_HIP(hipMemcpy(d_rowptr, rowptr, sizeof rowptr, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_colidx, colidx, sizeof(int32_t) * nnz, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_vals, vals, sizeof(uint16_t) * nnz, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_B, B, sizeof B, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_X, X, sizeof X, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_Y, Y, sizeof Y, hipMemcpyHostToDevice));

    /* chunk = 32 cuts the long row's window into one-block parts: the partial-tile path runs too */
    CHECK_FS(fs_convert(M, K, nnz, d_rowptr, d_colidx, d_vals, FS_F16, 0, 0, 32, d_arena, arena_bytes, d_scratch,
                        scratch_bytes, NULL, &fmt));
    CHECK_FS(fs_spmm_workspace_bytes(&fmt, N, &work_bytes));
    if (work_bytes) CHECK_HIP(hipMalloc(&d_work, work_bytes));
    CHECK_FS(fs_spmm(&fmt, NULL, d_B, N, N, d_C, N, d_work, work_bytes, NULL));
    CHECK_HIP(hipMalloc((void **)&d_scores, sizeof(uint16_t) * fmt.V * fmt.nvec));
    CHECK_HIP(hipMalloc((void **)&d_scores_csr, sizeof(uint16_t) * nnz));
    uint16_t *d_scores_csr2;  /* CSR order straight from the kernel, compared with the re-ordered blocked output below */
    CHECK_HIP(hipMalloc((void **)&d_scores_csr2, sizeof(uint16_t) * nnz));
    CHECK_FS(fs_sddmm(&fmt, d_X, D, d_Y, D, D, d_scores, d_scores_csr2, NULL));
    CHECK_FS(fs_blk_to_csr(&fmt, d_scores, d_scores_csr, NULL));

    /* CSR of the transposed matrix, and the attention chain as one call (B serves as H) */
    int32_t *d_rowptr_t, *d_colidx_t, *d_perm;
    uint16_t *d_att;
    void *d_tscratch, *d_awork = NULL;
    size_t tscratch_bytes, awork_bytes;
    const float att_scale = 0.25f;
    CHECK_FS(fs_csr_transpose_bytes(M, K, nnz, &tscratch_bytes));
    CHECK_HIP(hipMalloc((void **)&d_rowptr_t, sizeof(int32_t) * (K + 1)));
    CHECK_HIP(hipMalloc((void **)&d_colidx_t, sizeof(int32_t) * nnz));
    CHECK_HIP(hipMalloc((void **)&d_perm, sizeof(int32_t) * nnz));
    CHECK_HIP(hipMalloc(&d_tscratch, tscratch_bytes));
    CHECK_FS(fs_csr_transpose(M, K, nnz, d_rowptr, d_colidx, d_rowptr_t, d_colidx_t, d_perm, d_tscratch, tscratch_bytes, NULL));
    CHECK_FS(fs_attention_workspace_bytes(&fmt, N, &awork_bytes));
    if (awork_bytes) CHECK_HIP(hipMalloc(&d_awork, awork_bytes));
    CHECK_HIP(hipMalloc((void **)&d_att, sizeof(uint16_t) * M * N));
    CHECK_FS(fs_attention(&fmt, d_X, D, d_Y, D, D, att_scale, d_B, N, N, d_att, N, d_awork, awork_bytes, NULL));
    CHECK_HIP(hipDeviceSynchronize());

    /* host references */
    uint16_t C[M * N], *scores = (uint16_t *)malloc(sizeof(uint16_t) * nnz);
    int bad = 0;
    CHECK_HIP(hipMemcpy(C, d_C, sizeof C, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(scores, d_scores_csr2, sizeof(uint16_t) * nnz, hipMemcpyDeviceToHost));
    {
        uint16_t *again = (uint16_t *)malloc(sizeof(uint16_t) * nnz);
        CHECK_HIP(hipMemcpy(again, d_scores_csr, sizeof(uint16_t) * nnz, hipMemcpyDeviceToHost));
        if (memcmp(again, scores, sizeof(uint16_t) * nnz) != 0) { printf("SDDMM: CSR-order output differs from the re-ordered blocked output\n"); return 1; }
        free(again);
    }
    for (i = 0; i < M; i++)
        for (j = 0; j < N; j++) {
            double acc = 0;
            for (p = rowptr[i]; p < rowptr[i + 1]; p++) acc += half_value(vals[p]) * half_value(B[colidx[p] * N + j]);
            if (half_value(C[i * N + j]) != acc) bad++;
        }
    for (i = 0; i < M; i++)
        for (p = rowptr[i]; p < rowptr[i + 1]; p++) {
            double acc = 0;
            for (t = 0; t < D; t++) acc += half_value(X[i * D + t]) * half_value(Y[colidx[p] * D + t]);
            if (half_value(scores[p]) != acc) bad++;
        }
    /* transposed CSR: walk A's rows in order and append every entry to the list of its column */
    {
        int32_t rowptr_t[K + 2], next[K], *colidx_t = (int32_t *)malloc(sizeof(int32_t) * nnz);
        int32_t *perm = (int32_t *)malloc(sizeof(int32_t) * nnz), *got = (int32_t *)malloc(sizeof(int32_t) * nnz);
        int32_t got_ptr[K + 1];
        memset(rowptr_t, 0, sizeof rowptr_t);
        for (p = 0; p < nnz; p++) rowptr_t[colidx[p] + 1]++;
        for (j = 0; j < K; j++) { rowptr_t[j + 1] += rowptr_t[j]; next[j] = rowptr_t[j]; }
        for (i = 0; i < M; i++)
            for (p = rowptr[i]; p < rowptr[i + 1]; p++) { colidx_t[next[colidx[p]]] = i; perm[next[colidx[p]]++] = p; }
        CHECK_HIP(hipMemcpy(got_ptr, d_rowptr_t, sizeof got_ptr, hipMemcpyDeviceToHost));
        if (memcmp(got_ptr, rowptr_t, sizeof got_ptr)) bad++;
        CHECK_HIP(hipMemcpy(got, d_colidx_t, sizeof(int32_t) * nnz, hipMemcpyDeviceToHost));
        if (memcmp(got, colidx_t, sizeof(int32_t) * nnz)) bad++;
        CHECK_HIP(hipMemcpy(got, d_perm, sizeof(int32_t) * nnz, hipMemcpyDeviceToHost));
        if (memcmp(got, perm, sizeof(int32_t) * nnz)) bad++;
    }
    /* attention: softmax over each row's stored entries of att_scale * x.y, times the rows of B */
    {
        uint16_t att[M * N];
        CHECK_HIP(hipMemcpy(att, d_att, sizeof att, hipMemcpyDeviceToHost));
        for (i = 0; i < M; i++) {
            double top = -1e300, total = 0, w[K];
            for (p = rowptr[i]; p < rowptr[i + 1]; p++) {
                w[p - rowptr[i]] = att_scale * half_value(scores[p]);  /* the scores were checked exactly above */
                if (w[p - rowptr[i]] > top) top = w[p - rowptr[i]];
            }
            for (p = rowptr[i]; p < rowptr[i + 1]; p++) total += w[p - rowptr[i]] = exp(w[p - rowptr[i]] - top);
            for (j = 0; j < N; j++) {
                double acc = 0, mag = 0;
                for (p = rowptr[i]; p < rowptr[i + 1]; p++) {
                    double h = half_value(B[colidx[p] * N + j]);
                    acc += w[p - rowptr[i]] / total * h;
                    mag += w[p - rowptr[i]] / total * fabs(h);
                }
                if (fabs(half_value(att[i * N + j]) - acc) > 1e-2 * mag + 1e-7) bad++;
            }
        }
    }
    printf("flashsparse %d: M=%d K=%d nnz=%d nvec=%lld items=%lld cut windows=%lld: %s\n", fs_version(), M, K, nnz,
           (long long)fmt.nvec, (long long)fmt.n_items, (long long)fmt.n_split_windows, bad ? "MISMATCH" : "OK");
    return bad ? 1 : 0;
}
