/*
 * maskkv_bench.h - C ABI of libmaskkv_bench.so, the measurement companion of libmaskkv.so.
 *
 * Nothing here is part of the MaskKV method (arXiv 2510.09309) or of the product library: these calls exist so
 * that a benchmark harness can (a) quote kernel rates against what the same box sustains on one resource at a
 * time and (b) time the stages inside one maskkv_score call.  Conventions as in maskkv.h: DEVICE / HOST pointers,
 * work is enqueued on the given stream (hipStream_t as void*), nothing is allocated, freed or synchronised,
 * every call returns a maskkv_status and enqueues nothing on failure.
 */
#ifndef MASKKV_BENCH_H
#define MASKKV_BENCH_H

#include "maskkv.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Detail of the calling thread's most recent maskkv_bench_probe failure ("" if none). */
const char* maskkv_bench_last_error(void);

/*
 * Enqueues one kernel that exercises a single resource.
 *   which = 0  bf16 matrix pipe, constant operands: every wave of `groups` 256-thread workgroups issues 4*iters
 *              v_mfma_f32_32x32x16_bf16 from registers;                       *work = floating-point operations
 *   which = 1  v_exp_f32: every lane issues 8*iters exponentials;                          *work = exponentials
 *   which = 2  streaming copy of `bytes` from src to dst (grid-stride, 16-byte pieces);  *work = bytes read + written
 *   which = 3  streaming read of `bytes` from src (folded into one word per thread);      *work = bytes read
 *   which = 4  the scoring kernels' instruction mix from registers: per iteration every wave issues 16 MFMAs and
 *              every lane 32 x (fma, v_exp_f32, add);                  *work = floating-point operations of the MFMAs
 *   which = 5  bf16 matrix pipe on data: per iteration every wave issues two chains of eight MFMAs that start
 *              from zero, with operands from 24 register sets loaded from src (24 KiB: fill it with the bit
 *              patterns a kernel really sees; the matrix pipe's sustained rate depends on them);
 *                                                                                *work = floating-point operations
 *   which = 6  the scoring kernels' form-and-reduce pipeline on data, from registers: per iteration every wave
 *              forms two 32x32 logits blocks (16 MFMAs, operands as for which = 5) into one accumulator pair and
 *              takes the exponentials of the pair formed one iteration earlier (32 x (multiply, v_exp_f32, add)
 *              per lane); iterations run in pairs;                *work = floating-point operations of the MFMAs
 *   which = 7  do the two pipes of a SIMD serve different waves at the same time?  512-thread workgroups (waves w
 *              and w + 4 share a SIMD): per iteration waves 0-3 issue the sixteen MFMAs of which = 5, waves 4-7
 *              32 x (multiply, v_exp_f32, add) per lane; iterations run in pairs;
 *                                                                 *work = floating-point operations of the MFMAs
 *   which = 8  as 7, the matrix waves alone (waves 4-7 exit at once);                                 *work as for 7
 *   which = 9  as 7, the vector waves alone (waves 0-3 exit at once);                           *work = exponentials
 * dst: DEVICE of dst_bytes bytes; for which != 2 it receives one 32-bit word per launched thread, for which = 2 it
 * is the copy target.  src: DEVICE, 16-byte aligned; `bytes` a multiple of 16 (which = 2, 3) or at least 24576
 * (which = 5 ... 9); ignored otherwise.  work: HOST double, may be NULL.  groups: workgroups launched (256 threads
 * each, 512 for which >= 7), 1..2^20.  MASKKV_EINVAL on any violation.
 */
int maskkv_bench_probe(int which, int32_t iters, const void* src, void* dst, int64_t bytes, int64_t dst_bytes,
                       int32_t groups, void* stream, double* work);

/*
 * maskkv_score (same arguments, same result, same kernels: it calls the body of maskkv_score in libmaskkv.so)
 * with timing marks.  events: HOST array of 4 hipEvent_t (each may be NULL), created by the caller with timing
 * enabled; they are recorded on the stream before pass 1 (row statistics), before the merge, before pass 2
 * (column sums) and after pass 2.  Errors are reported through maskkv_last_error() of libmaskkv.so.
 */
int maskkv_bench_score_marked(const maskkv_desc* desc, const maskkv_tensor* Q_mask, const maskkv_tensor* K_full,
                              float scale, float* scores, int64_t score_stride, float* prompt_mass,
                              void* workspace, size_t workspace_bytes, void* stream, void* const* events);

#ifdef __cplusplus
}
#endif
#endif /* MASKKV_BENCH_H */
