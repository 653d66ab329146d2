/*
 * CPU oracle for sparse-times-dense (SpMM) and sampled dense-dense (SDDMM).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the yardstick the GPU library is
 * checked against; nothing in the product path may call it.  It shares no
 * code, header, table or helper with the HIP sources.
 *
 * Both operators reach, up to rounding order, a result with a plain
 * definition, so the oracle is that definition written out over CSR, with
 * every stored 16-bit input widened exactly to double and every sum carried
 * in double:
 *
 *   SpMM  (paper Section 2.2: a sparse matrix A multiplied by a dense B)
 *       C[i][j] = sum over stored entries p of row i of  A.val[p] * B[A.col[p]][j]
 *   SDDMM (paper Section 3.4: two dense inputs, output sparse by sampling)
 *       out[p]  = sum over t < d of  X[i][t] * Y[A.col[p]][t]     for every stored entry p of row i
 *       The stored values of A play no part: A only supplies the sampling pattern.
 *
 *   Edge softmax (the softmax layer of the attention GNN in the paper's
 *   end-to-end evaluation, Section 4.4; the paper names it without giving a
 *   kernel, so this is the textbook definition over the stored entries of a row)
 *       out[p]  = exp(scale*v[p]) / sum over stored entries q of row i of exp(scale*v[q])
 *
 *   CSR of the transposed matrix (index work only; for the A^T * dC of a
 *   backward pass): see oracle_csr_transpose.
 *
 * Next to each result the oracle emits the matching sum of absolute products
 * (the "scale"), which a comparison can use as the denominator of a relative
 * error that stays meaningful when terms cancel.
 *
 * Plain C, one loop nest per operator, rows spread over OpenMP threads.
 */
#include <stdint.h>
#include <stddef.h>
#include <math.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F16 = 0, ORACLE_BF16 = 1 };

/* IEEE binary16 -> double, exact (subnormals, infinities and NaN included). */
static double half_bits_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1F;
    int frac = h & 0x3FF;
    double v;
    if (expo == 0)
        v = ldexp((double)frac, -24); /* subnormal or zero: frac * 2^-24 */
    else if (expo == 31)
        v = frac ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)frac / 1024.0, expo - 15);
    return sign ? -v : v;
}

/* bfloat16 is the upper half of an IEEE binary32. */
static double bf16_bits_to_double(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static double widen(uint16_t bits, int dtype)
{
    return dtype == ORACLE_BF16 ? bf16_bits_to_double(bits) : half_bits_to_double(bits);
}

int oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Exposed so that tests can pin the widening against numpy's own conversion. */
double oracle_widen(uint16_t bits, int dtype) { return widen(bits, dtype); }

/*
 * SpMM over a list of rows.
 *   rows == NULL : rows 0..n_rows-1 (use n_rows = M for the whole product)
 *   rows != NULL : the n_rows row numbers given; output row q belongs to rows[q]
 * C and S are n_rows x N, row-major, leading dimension N.  S may be NULL.
 * Returns 0, or 1 when an index is out of range.
 */
int oracle_spmm(int64_t M, int64_t K, int64_t N,
                const int32_t *rowptr, const int32_t *colidx, const uint16_t *vals,
                const uint16_t *B, int64_t ldb, int dtype,
                const int64_t *rows, int64_t n_rows,
                double *C, double *S)
{
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 16) reduction(| : bad)
    for (int64_t q = 0; q < n_rows; q++) {
        int64_t i = rows ? rows[q] : q;
        double *c = C + q * N;
        double *s = S ? S + q * N : NULL;
        for (int64_t j = 0; j < N; j++) c[j] = 0.0;
        if (s) for (int64_t j = 0; j < N; j++) s[j] = 0.0;
        if (i < 0 || i >= M) { bad |= 1; continue; }
        for (int32_t p = rowptr[i]; p < rowptr[i + 1]; p++) {
            int64_t k = colidx[p];
            if (k < 0 || k >= K) { bad |= 1; continue; }
            double a = widen(vals[p], dtype);
            const uint16_t *brow = B + k * ldb;
            for (int64_t j = 0; j < N; j++) {
                double prod = a * widen(brow[j], dtype);
                c[j] += prod;
                if (s) s[j] += fabs(prod);
            }
        }
    }
    return bad;
}

/*
 * SDDMM over a list of rows of A (same row-list convention as oracle_spmm).
 * out and S are indexed by CSR position p (length nnz); only the positions of
 * the listed rows are written.  S may be NULL.
 */
int oracle_sddmm(int64_t M, int64_t K, int64_t d,
                 const int32_t *rowptr, const int32_t *colidx,
                 const uint16_t *X, int64_t ldx, const uint16_t *Y, int64_t ldy, int dtype,
                 const int64_t *rows, int64_t n_rows,
                 double *out, double *S)
{
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 16) reduction(| : bad)
    for (int64_t q = 0; q < n_rows; q++) {
        int64_t i = rows ? rows[q] : q;
        if (i < 0 || i >= M) { bad |= 1; continue; }
        const uint16_t *x = X + i * ldx;
        for (int32_t p = rowptr[i]; p < rowptr[i + 1]; p++) {
            int64_t k = colidx[p];
            if (k < 0 || k >= K) { bad |= 1; continue; }
            const uint16_t *y = Y + k * ldy;
            double acc = 0.0, sc = 0.0;
            for (int64_t t = 0; t < d; t++) {
                double prod = widen(x[t], dtype) * widen(y[t], dtype);
                acc += prod;
                sc += fabs(prod);
            }
            out[p] = acc;
            if (S) S[p] = sc;
        }
    }
    return bad;
}

/*
 * Softmax over the stored entries of each row of A (same row-list convention
 * as oracle_spmm), of scale * value.  The row maximum is subtracted before
 * exponentiating, which leaves the quotient unchanged and keeps exp in range.
 * out is indexed by CSR position p; only the positions of the listed rows are
 * written; a row without stored entries writes nothing.
 */
int oracle_edge_softmax(int64_t M, const int32_t *rowptr, const uint16_t *vals, int dtype, double scale,
                        const int64_t *rows, int64_t n_rows, double *out)
{
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 64) reduction(| : bad)
    for (int64_t q = 0; q < n_rows; q++) {
        int64_t i = rows ? rows[q] : q;
        if (i < 0 || i >= M) { bad |= 1; continue; }
        int32_t p0 = rowptr[i], p1 = rowptr[i + 1];
        if (p1 <= p0) continue;
        double top = -INFINITY, total = 0.0;
        for (int32_t p = p0; p < p1; p++) {
            double t = scale * widen(vals[p], dtype);
            if (t > top) top = t;
        }
        for (int32_t p = p0; p < p1; p++) total += exp(scale * widen(vals[p], dtype) - top);
        for (int32_t p = p0; p < p1; p++) out[p] = exp(scale * widen(vals[p], dtype) - top) / total;
    }
    return bad;
}

/*
 * CSR of the transposed matrix (needed for A^T * dC, the backward pass of
 * C = A * B in the end-to-end training of the paper's Section 4.4).  The
 * definition: entry (i, k) of A is entry (k, i) of A^T; row k of A^T lists
 * its entries by ascending i.  Walking A's rows in order and appending each
 * entry to the list of its column yields exactly that order.
 *   rowptr_t[K+1], colidx_t[nnz] : the result
 *   perm[nnz]                    : perm[q] = position in A's CSR order of the
 *                                  entry at position q of A^T's CSR order
 * Returns nonzero if a column index is outside [0, K).
 */
int oracle_csr_transpose(int64_t M, int64_t K, const int32_t *rowptr, const int32_t *colidx,
                         int32_t *rowptr_t, int32_t *colidx_t, int32_t *perm)
{
    for (int64_t k = 0; k <= K; k++) rowptr_t[k] = 0;
    for (int64_t i = 0; i < M; i++)
        for (int32_t p = rowptr[i]; p < rowptr[i + 1]; p++) {
            if (colidx[p] < 0 || colidx[p] >= K) return 1;
            rowptr_t[colidx[p] + 1]++; /* entries per column, shifted by one */
        }
    for (int64_t k = 0; k < K; k++) rowptr_t[k + 1] += rowptr_t[k];
    /* next free position of every row of A^T; restored to row starts afterwards */
    for (int64_t i = 0; i < M; i++)
        for (int32_t p = rowptr[i]; p < rowptr[i + 1]; p++) {
            int32_t q = rowptr_t[colidx[p]]++;
            colidx_t[q] = (int32_t)i;
            perm[q] = p;
        }
    for (int64_t k = K; k > 0; k--) rowptr_t[k] = rowptr_t[k - 1];
    rowptr_t[0] = 0;
    return 0;
}

/*
 * Sparse attention, the SDDMM -> edge softmax -> SpMM chain of the attention
 * GNN in the paper's Section 4.4 written as one definition, with nothing
 * rounded in between:
 *   t[p]      = scale * sum over f < d of X[i][f] * Y[col[p]][f]      for the stored entries p of row i
 *   a[p]      = exp(t[p]) / sum over the stored entries q of row i of exp(t[q])
 *   out[i][n] = sum over p of a[p] * H[col[p]][n]
 * S[i][n] = sum over p of a[p] * |H[col[p]][n]| is the matching magnitude.
 * A row without stored entries gives zeros.  Same row-list convention as
 * oracle_spmm: out and S have n_rows rows.
 */
int oracle_attention(int64_t M, int64_t K, const int32_t *rowptr, const int32_t *colidx,
                     const uint16_t *X, int64_t ldx, const uint16_t *Y, int64_t ldy, int64_t d, int dtype,
                     double scale, const uint16_t *H, int64_t ldh, int64_t N,
                     const int64_t *rows, int64_t n_rows, double *out, double *S)
{
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 16) reduction(| : bad)
    for (int64_t q = 0; q < n_rows; q++) {
        int64_t i = rows ? rows[q] : q;
        double *o = out + q * N, *s = S ? S + q * N : NULL;
        for (int64_t n = 0; n < N; n++) { o[n] = 0.0; if (s) s[n] = 0.0; }
        if (i < 0 || i >= M) { bad |= 1; continue; }
        int32_t p0 = rowptr[i], p1 = rowptr[i + 1];
        if (p1 <= p0) continue;
        const uint16_t *x = X + i * ldx;
        /* pass 1: the largest t; pass 2: the normaliser; pass 3: the weighted rows of H */
        double top = -INFINITY, total = 0.0;
        int ok = 1;
        for (int32_t p = p0; p < p1; p++) {
            int64_t k = colidx[p];
            if (k < 0 || k >= K) { ok = 0; break; }
            double t = 0.0;
            for (int64_t f = 0; f < d; f++) t += widen(x[f], dtype) * widen(Y[k * ldy + f], dtype);
            t *= scale;
            if (t > top) top = t;
        }
        if (!ok) { bad |= 1; continue; }
        for (int32_t p = p0; p < p1; p++) {
            int64_t k = colidx[p];
            double t = 0.0;
            for (int64_t f = 0; f < d; f++) t += widen(x[f], dtype) * widen(Y[k * ldy + f], dtype);
            total += exp(scale * t - top);
        }
        for (int32_t p = p0; p < p1; p++) {
            int64_t k = colidx[p];
            double t = 0.0;
            for (int64_t f = 0; f < d; f++) t += widen(x[f], dtype) * widen(Y[k * ldy + f], dtype);
            double a = exp(scale * t - top) / total;
            for (int64_t n = 0; n < N; n++) {
                double h = widen(H[k * ldh + n], dtype);
                o[n] += a * h;
                if (s) s[n] += a * fabs(h);
            }
        }
    }
    return bad;
}
