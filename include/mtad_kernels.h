/*
 * mtad_kernels.h - component entry points of libmtad: single kernels of the hot path, exported so that each
 * can be checked and timed on its own at the real shapes.  Same conventions as mtad.h (device pointers are
 * borrowed, work is only enqueued on `stream`, status codes of mtad_status).
 */
#ifndef MTAD_KERNELS_H
#define MTAD_KERNELS_H

#include "mtad.h"

#ifdef __cplusplus
extern "C" {
#endif

/* The few-row matrix product of every projection, FFN matrix and the lm_head of a pass (the weight stream the
 * paper's cost argument is about, Section 4: time and energy are dominated by reading the weights once per run).
 * Y[r][n] (+)= sum_k X[r][k] * W[n][k], r < R.  dtype 1: W bfloat16 [N][K] tile-packed (mtad_pack_matrix,
 * MTAD_PACK_PLAIN); X two bfloat16 planes [2][R][K]
 * (hi, lo) whose sum is the activation; float32 accumulation (N % 16 == 0, K % 32 == 0, R <= 256);
 * dtype 0: W, X float32 (K % 4 == 0).  Y float32 [R][ldy], ldy >= N, ldy % 4 == 0.
 * accumulate != 0 adds to Y (the residual connection).  This is the product kernel of the passes with its plain store
 * epilogue.  ctx may be NULL; with a context whose bound workspace covers the shape (it does for the context's own
 * model shapes) products with few output strips and more than 8 rows also split the reduction dimension over
 * workgroups, and products of many rows (65 or more, or 25 or more with at least 16384 outputs) take the kernel that
 * stages both operands through LDS, as in the passes. */
int mtad_k_gemm(mtad_ctx *ctx, int32_t dtype, const void *W, const void *X, float *Y, int32_t R, int32_t N, int32_t K, int32_t ldy,
                int32_t accumulate, void *stream);

/* The same product with the activation terms in the order the kernel-per-step passes keep them in (dtype 1 only):
 * x_order MTAD_X_PLANES is mtad_k_gemm; MTAD_X_FRAGMENTS is the B-operand fragment order of the 16x16x32 bfloat16
 * matrix instruction, 8 rows at a time.  With kt = k / 32, kg = (k % 32) / 8, e = k % 8 and plane 0 = hi, 1 = lo, the
 * element (plane, r, k) lies at
 *   R <= 24: ((((kt * 4 + kg) * 2 + plane) * R + r) * 8 + e                                   (128 R bytes per k tile)
 *   R >  24: ((((kt * G + r / 8) * 64 + kg * 16 + plane * 8 + r % 8) * 8 + e,  G = ceil(R / 8)   (K/32 * G fragments of 1 KiB;
 *            the buffer holds G * 8 rows, the slots of rows past R are not read into results).
 * A product then reads whole cache lines per fragment.  X: device, 4 * K * (R <= 24 ? R : 8 * G) bytes.  Other arguments, errors
 * and kernel choice as mtad_k_gemm; with 25 rows or more and a context's workspace the many-row kernel reads X directly. */
enum { MTAD_X_PLANES = 0, MTAD_X_FRAGMENTS = 1 };
int mtad_k_gemm_x(mtad_ctx *ctx, int32_t dtype, const void *W, const void *X, float *Y, int32_t R, int32_t N, int32_t K, int32_t ldy,
                  int32_t accumulate, int32_t x_order, void *stream);

/* out[row][i] = h[row][i] / sqrt(mean_i h[row][i]^2 + eps) * g[i]; out is two
 * bfloat16 planes [2][rows][d] (hi, lo; dtype 1) or float32 [rows][d] (dtype 0). */
int mtad_k_rmsnorm(int32_t dtype, const float *h, const float *g, void *out, int32_t rows, int32_t d, float eps,
                   void *stream);

/* lse[row] = log sum_v exp(logits[row][v]) (the normaliser that turns a logits row into a row of P, Algorithm 1). */
int mtad_k_row_lse(const float *logits, float *lse, int32_t rows, int32_t vocab, void *stream);

/* The warping step of mtad_set_warp on given rows, in place: logits [rows][vocab] become rows of log p~ (minus infinity
 * outside the support), lse[row] becomes 0.  1 <= top_k <= 16, top_p > 0. */
int mtad_k_warp_rows(float *logits, float *lse, int32_t rows, int32_t vocab, int32_t top_k, float top_p, void *stream);

/* The selection part of one beam step (Section 2.1, Eq. 2) on given draft logits [batch][rows_per_seq][vocab] and
 * their row logsumexps: candidate (r, v) scores hist.cum_logq[step-1][r] + (logits[r][v] - lse[r]) (at step 0 the
 * only live beam is row catchup_cnt-1 with score 0); writes hist[.][step][.].  `len` = committed draft tokens per
 * sequence (only keys the sampling noise).  Needs a context with a bound workspace. */
int mtad_k_beam_topb(mtad_ctx *ctx, const float *logits, const float *lse, mtad_beam *hist, int32_t step,
                     const int32_t *catchup_cnt, const int32_t *len, int32_t rows_per_seq, int32_t vocab,
                     int32_t sample_beam, uint64_t seed, void *stream);

/* mtad_k_beam_topb for callers that cannot allocate device memory or bind a workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same inputs, outputs and results; the shapes a context would carry
 * (batch, gamma, beam) are arguments, and the scratch of the two-stage selection (the stage-1 winners) lives in a
 * device array inside the library: 256 KiB per GPU, present from the first call on that GPU until the process ends.  The
 * call allocates nothing and only enqueues work on `stream`.
 * Limits: batch <= MTAD_STATIC_TOPB_MAX_BATCH (MTAD_ECAP beyond it), beam <= MTAD_MAX_BEAM, rows_per_seq >= gamma + 1 at
 * step 0 and >= beam afterwards (the rows the kernels read), vocab >= beam.
 * All calls on one GPU share that GPU's array: two calls whose work overlaps in time on one GPU (different streams or
 * threads) race; calls on one stream, or otherwise ordered, are safe, and nothing has to be cleared between them. */
#define MTAD_STATIC_TOPB_MAX_BATCH 64
int mtad_k_beam_topb_static(const float *logits, const float *lse, mtad_beam *hist, int32_t batch, int32_t gamma, int32_t beam,
                            int32_t step, const int32_t *catchup_cnt, const int32_t *len, int32_t rows_per_seq, int32_t vocab,
                            int32_t sample_beam, uint64_t seed, void *stream);

/* Streaming copy of `bytes` bytes (a multiple of 16, both pointers 16-byte aligned).  It moves exactly `bytes` in
 * and `bytes` out, which makes it the reference for scaling the hardware's byte counters and for the bandwidth
 * that perfectly coalesced traffic reaches on the device (the paper's cost model, Section 4, prices runs by
 * their global-memory traffic). */
int mtad_k_copy(const void *src, void *dst, int64_t bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MTAD_KERNELS_H */
