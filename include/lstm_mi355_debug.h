/*
 * lstm_mi355_debug.h — diagnostic entry points of liblstm_mi355.so: launch timing for benchmarks,
 * single kernels for kernel tests and micro-benchmarks, the workspace plan for host-side checks.
 * None of them is part of the training step; the product interface is lstm_mi355.h.
 */
#ifndef LSTM_MI355_DEBUG_H
#define LSTM_MI355_DEBUG_H

#include "lstm_mi355.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Per-kernel-class launch timing for benchmarks.  When enabled, every launch
 * the library enqueues is bracketed by two HIP events recorded on the caller's
 * stream (events are created on first use and reused).  lstm_timing_enable
 * also clears the accumulated numbers.  lstm_timing_read waits for the
 * recorded work, then returns for one class the number of timed launches, the
 * summed event-to-event duration in ms, and the summed algorithmic flops
 * (GEMM classes: 2*M*N*K) and bytes (streaming classes) of those launches.
 * Classes: 0 whole-sequence GEMMs, 1 per-time-step recurrent GEMMs, 2 gate
 * pointwise kernels, 3 auxiliary kernels, 4 grad_average, 5 master_update.
 * All out-pointers are host memory.  Not thread-safe with respect to
 * concurrently running entry points on other threads' streams. */
int lstm_timing_enable(int32_t on);
int lstm_timing_read(int32_t kernel_class, int64_t *launches, double *total_ms, double *flops, double *bytes);

/* One whole-sequence GEMM through the dispatch the training step uses, for kernel tests and
 * micro-benchmarks.  All pointers device.  C: lp [M,N] row-major, out.
 *   layout 0: C = A B^T, row-major A[M,K], B[N,K]
 *   layout 1: C = A^T B, row-major A[K,M], B[K,N]   (16-bit types, M, N >= 192, multiples of 8)
 *   layout 2/3/4: operands in 64x64 blocks as written by lstm_debug_pack_blocked, with
 *                 (A rows, B rows) indexing (M, N) / (M, K) / (K, K)   (16-bit types, M, N >= 192)
 *   layout 5: as 4 on the second (K,K) kernel   (K a multiple of 128; with splits > 1 the contraction is cut
 *             into that many equal parts, K a multiple of 128 * splits)
 *   layout 6: as 5, every 64x64 block of both operands in the fragment order given below for a 64-row tile
 * splitk_ws: fp32 [splits, M, N] or NULL with splits <= 1. */
int lstm_debug_gemm(int32_t dtype, int32_t layout, int32_t M, int32_t N, int32_t K, const void *A, const void *B, void *C,
                    float *splitk_ws, int32_t splits, void *stream);

/* The whole-sequence GEMM on operands in packed (MFMA-fragment) order, C = A B^T (+ bias): 16-bit types, M and
 * rows_per_step multiples of 64 (M a multiple of rows_per_step), K a multiple of 256, N a multiple of 8.
 * All pointers device.  Element (row, k) of a 64-row tile's 64-wide K chunk lies at
 * ((k/16 * nblk + row/32) * 64 + 32 * (k/8 % 2) + row % 32) * 8 + k % 8 inside the chunk, nblk = 2 for A, 4 for B.
 *   A: the rows of one time step (rows_per_step of them) as [64-row tile][K/64][chunk of 64 x 64]; consecutive
 *      time steps a_step_stride elements apart.
 *   B: [128-row tile][K/64][chunk of 128 x 64].  gate_h = 0: row n of B produces column n of C.  gate_h = H
 *      (N = 4H): row 32 g + r of tile j produces column g H + 32 j + r (the order the recurrent kernels keep
 *      their weights in).
 *   bias: lp [N] or NULL.  C: lp [M, N] row-major, out. */
int lstm_debug_gemm_stream(int32_t dtype, int32_t M, int32_t N, int32_t K, int32_t rows_per_step, int64_t a_step_stride,
                           int32_t gate_h, const void *A, const void *B, const void *bias, void *C, void *stream);
/* Enqueues a loop of `iters` x 8 independent 32x32x16 MFMAs per wavefront (256 workgroups of 8
 * wavefronts) whose operands stay in registers: the rate the matrix pipes sustain on the given
 * operand values, which depends on the values through the chip's power management.
 *   operands: device, 256*512*2 fragments of 16 bytes (8 lp values each), read once
 *   sink:     device, 1 float (never written in practice)
 *   flops:    host, out (may be NULL): floating-point operations the launch performs
 * 16-bit types only; 1 <= iters <= 2^22.  The caller times the launch. */
int lstm_debug_mfma_rate(int32_t dtype, const void *operands, int32_t iters, float *sink, double *flops, void *stream);

/* dst (64x64 blocks, zero padded to whole blocks: ceil(rows/64)*ceil(cols/64)*4096 elements) =
 * src (row-major [rows, cols]).  Both device. */
int lstm_debug_pack_blocked(int32_t dtype, const void *src, int32_t rows, int32_t cols, void *dst, void *stream);

/* The regions lstm_forward / lstm_backward use inside the caller's reserve and scratch buffers for cfg, in
 * the order the plan hands them out (host only, nothing is enqueued).  For region i < min(*count,
 * max_regions): which[i] = 0 (reserve) or 1 (scratch), offsets[i] and bytes[i] in bytes.  *count receives
 * the total number of regions.  Regions of one buffer never overlap and end inside the size
 * lstm_workspace_bytes reports.  All pointers host. */
int lstm_debug_plan_regions(const lstm_config *cfg, int32_t max_regions, int32_t *which, size_t *offsets, size_t *bytes,
                            int32_t *count);

#ifdef __cplusplus
}
#endif
#endif /* LSTM_MI355_DEBUG_H */
