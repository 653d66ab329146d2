/*
 * flashsparse_measure.h -- measurement aids exported by libflashsparse_hip.so next to the product
 * interface of flashsparse.h.  They exist for the benchmark and for profiler calibration; no
 * computation of the library depends on them.  Conventions (status codes, d_ = device pointer,
 * stream passed as void*) as in flashsparse.h.
 */
#ifndef FLASHSPARSE_MEASURE_H
#define FLASHSPARSE_MEASURE_H

#include "flashsparse.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * fs_spmm with two hipEvent_t handles (passed as void*, either may be NULL) that the
 * library records on `stream` immediately before and immediately after its main
 * kernel, i.e. excluding the small kernel that adds the partial tiles of cut
 * windows.  For measurement: lets a caller time the main kernel with HIP events
 * exactly as a profiler's kernel trace sees it.  Otherwise identical to fs_spmm.
 */
fs_status fs_spmm_timed(const fs_format *fmt, const void *d_vals,
                        const void *d_B, int64_t N, int64_t ldb,
                        void *d_C, int64_t ldc,
                        void *d_work, size_t work_bytes, void *stream,
                        void *ev_before_main, void *ev_after_main);

/*
 * Measurement aid: the gather of fs_spmm and nothing else.  Loads, work item by work item in fs_spmm's launch
 * order and placement, the rows of B the column indices name -- with the load instructions and lane mapping of
 * the SpMM kernel's 128-column pass -- and discards them (one word per lane goes to d_sink so that the loads are kept).  Its
 * duration is what this machine needs just to bring the method's operand rows to the registers for this
 * matrix: the floor under fs_spmm's time that no change to the rest of the kernel can go below.
 *   d_sink : 1 MiB (1024 * 256 * 4 bytes), 4-byte aligned.  N % 8 == 0, ldb % 8 == 0, d_B 16-byte aligned.
 * Asynchronous on `stream`.
 */
fs_status fs_gather_probe(const fs_format *fmt, const void *d_B, int64_t N, int64_t ldb,
                          void *d_sink, size_t sink_bytes, void *stream);

/*
 * Measurement aid: a plain streaming copy of `bytes` bytes (a multiple of 16,
 * both pointers 16-byte aligned) from d_src to d_dst.  Its HBM traffic is
 * known exactly (bytes read + bytes written), which calibrates a profiler's
 * byte counters against the figures they report for the kernels above.
 */
fs_status fs_copy_bytes(void *d_dst, const void *d_src, size_t bytes, void *stream);

/*
 * Measurement aid: 2048 workgroups each read one 16 KiB chunk of the buffer per repeat, `repeats` times in
 * one kernel, and discard what they read; a workgroup's chunks change from repeat to repeat but stay in the
 * eighth of the buffer that belongs to its XCD.  With a buffer that fits the L2s (16 MiB: 2 MiB per XCD) the
 * rate, 2048 * 16384 * repeats / duration, is the bandwidth the L2s deliver to the compute units -- the
 * ceiling for a kernel whose operands are cache-resident, as the gathers of the small workloads are.
 *   bytes  : a multiple of 131072 (eight chunks); d_src 16-byte aligned.
 *   d_sink : 2 MiB (2048 * 256 * 4 bytes), 4-byte aligned.
 */
fs_status fs_read_bytes(const void *d_src, size_t bytes, int32_t repeats, void *d_sink, size_t sink_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* FLASHSPARSE_MEASURE_H */
