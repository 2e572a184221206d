/*
 * libstreambp - test and measurement hooks.  NOT part of the product boundary in streambp.h, and unlike it these calls
 * keep process-wide state and (the profile calls) allocate: HIP events and host memory.  They exist for the unit tests
 * of the GEMM family, for A/B runs against the shape-agnostic kernels and for per-launch timing in the benchmark
 * (paper Sec. 4.2 reports backward time; the roofline block of the benchmark needs it per kernel).
 * None of them may be called while another thread is inside a streambp_* entry point.
 */
#ifndef STREAMBP_DEBUG_H
#define STREAMBP_DEBUG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Route every GEMM / every attention call through the shape-agnostic kernels (process-wide switch). */
void streambp_debug_force_generic(int gemm_on, int attn_on);

/* Which optional fusions the layer entry points use (process-wide switch, for A/B timing; results agree to rounding):
 * bit 0: SwiGLU adjoint in the epilogue of the dact = dy W_down GEMM instead of an elementwise pass;
 * bit 1: rotary embedding of q, and its adjoint on dq, inside the attention kernels instead of two elementwise passes;
 * bit 2: the LM head's logits GEMM stores bf16 softmax numerators exp(z - max of the 256-column block) straight into the
 *        chunk's dz buffer (plus the block statistics and the target logits) instead of fp32 logits, and the row kernel
 *        finishes dz in place (bf16 heads whose shapes the MFMA kernel takes; otherwise ignored).
 * The default is what measured fastest on MI355X. */
void streambp_debug_set_fusions(int mask);
int streambp_debug_get_fusions(void);

/* One GEMM through the library's dispatcher: C[M,N] (=|+=) op(A) op(B) [+ op(A2) op(B2)], fp32 accumulation.
 *   A(m,k) = ta ? A[k*lda+m] : A[m*lda+k];  B(k,n) = tb ? B[n*ldb+k] : B[k*ldb+n];  in_dt / out_dt: SBP_F32 or SBP_BF16.
 *   scratch: optional device fp32 buffer for split-K partial tiles;  row_stats: optional device [M, N/256] pairs
 *   (max, sum of exp(c - max)) per row and block of 256 columns (store form C = A B^T with fp32 C only).
 * All tensor pointers are device pointers.  Returns 1 if the MFMA kernel ran, 0 if the shape-agnostic one did, -5 on a
 * launch error. */
int streambp_debug_gemm(int M, int N, int K, int ta, int tb, int in_dt, int out_dt, int acc, const void *A, const void *B,
                        void *C, long long lda, long long ldb, long long ldc, void *scratch, size_t scratch_bytes,
                        void *hip_stream, const void *A2, const void *B2, void *row_stats);

/* The softmax-numerator form of the store C = A B^T (A [M,K], B [N,K], bf16): E[m,n] (bf16, leading dimension lde) =
 * exp(c[m,n] - max of row m over the 256-column block of n), stats [M, ceil(N/256)] = (that max, sum of the block's
 * exponentials) and target_value[m] = c[m, targets[row_index ? row_index[m] : m]] in fp32 (entries whose target lies
 * outside [0, N) are left untouched).  Device pointers; row_index may be NULL.  Returns 1 if the MFMA kernel ran it, 0 if
 * it cannot take the problem (nothing is written then), -5 on a launch error. */
int streambp_debug_gemm_numerators(int M, int N, int K, const void *A, const void *B, void *E, long long lda, long long ldb,
                                   long long lde, void *stats, const int32_t *targets, const int32_t *row_index,
                                   float *target_value, void *hip_stream);

/* Weight-gradient form over n <= 8 reduction segments: C[M,N] += sum_s A_s^T B_s with A_s [K_s, M], B_s [K_s, N];
 * A, B, rows_dev are host arrays of n device pointers (rows_dev, optional, and its entries, optional: device int32
 * row counts that limit K_s at run time).  Returns 1 if one segmented MFMA launch did it, 0 otherwise, negative on error. */
int streambp_debug_gemm_dw_segments(int n, int M, int N, const int *K, const void *const *A, const void *const *B,
                                    const int *const *rows_dev, void *C, long long lda, long long ldb, long long ldc,
                                    int in_dt, int out_dt, void *hip_stream);

/* Per-launch timing with HIP events recorded on the launch stream around each GEMM kernel / attention launch sequence.
 * begin: CREATES 2*max_records events, allocates host records and switches recording on (returns 0; -1 if already on).
 * end: synchronises the events, fills the caller's host arrays of streambp_debug_profile_kinds() entries (launch count,
 * summed milliseconds, summed flops of launches with host-known sizes, summed upper-bound flops of launches whose row
 * count lives on the device), destroys the events and frees the records. */
int streambp_debug_profile_kinds(void);
int streambp_debug_profile_begin(int max_records);
int streambp_debug_profile_end(long long *count, double *ms, double *work, double *work_bounded);

/* What the matrix pipe sustains without global memory traffic: `workgroups` workgroups of 8 wavefronts (two per SIMD) each
 * issue `iters` rounds of eight independent v_mfma_f32_32x32x16_bf16 on operand fragments taken from `operands` (device,
 * 32768 bf16 values the caller filled: zeros, ones, random ...); `lds_reads` (0, 6 or 8) of the eight A fragments of a round
 * are re-read from LDS every round (1 KB per wave and read, conflict-free) - the GEMM main loop reads 6 fragments per 8
 * products, the attention backward 8 - the rest stay in registers.  The sums of the accumulators go to `sink` (device,
 * workgroups * 512 floats) so that nothing is optimised away.  2 * 32*32*16 * 8 * iters * 8 * workgroups flops per launch.
 * On MI355X the rate depends on the operand VALUES (the chip is power-managed): the benchmark reports it next to the GEMM
 * rates as the ceiling real data leaves.  Returns 0, -1 / -2 on a bad argument, -5 on a launch error. */
int streambp_debug_mfma_rate(const void *operands, float *sink, int workgroups, int iters, int lds_reads, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* STREAMBP_DEBUG_H */
