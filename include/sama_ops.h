/*
 * sama_ops.h -- op-level entry points of libsama: the individual kernels of the hot path, exposed for
 * per-kernel parity tests and roofline measurements.  Same conventions as sama.h: DEVICE pointers, work is
 * enqueued on the given hipStream_t (NULL = default stream) and not waited for, no allocation.
 */
#ifndef SAMA_OPS_H
#define SAMA_OPS_H

#include <stddef.h>
#include <stdint.h>
#include "sama.h"

#ifdef __cplusplus
extern "C" {
#endif

/* C[M x N] = A . (B + B2) on the bf16 matrix cores with fp32 accumulation: the contraction behind every linear
 * layer of the base learner (forward X W^T, dgrad dY W, wgrad dY^T X; Sec. 3.3 counts these passes).
 * a_trans = 0: A stored [M][K] (lda >= K); 1: stored [K][M] (lda >= M).
 * b_trans = 1: B stored [N][K] (ldb >= K), i.e. a weight matrix [out x in] used forward; 0: stored [K][N].
 * B2: optional second bf16 term of the weight (the low half of a two-term split), same storage as B, or NULL.
 * bias: optional fp32 [N] added to every row.  Outputs: C32 (fp32) and/or C16 (bf16), row stride ldc; either may
 * be NULL.  Requirements: K % 64 == 0, M % 8 == 0, N % 8 == 0, lda/ldb % 8 == 0, ldc % 4 == 0, 16-byte aligned
 * pointers.  Returns SAMA_EINVAL otherwise (nothing is launched). */
sama_status sama_op_gemm_bf16(const void* A, int64_t lda, int32_t a_trans, const void* B, const void* B2, int64_t ldb,
                              int32_t b_trans, int32_t M, int32_t N, int32_t K, const float* bias, float* C32, void* C16,
                              int64_t ldc, void* hip_stream);

/* `count` (1..4) independent contractions of the form above in ONE launch: the + and the - pass of Eq. 5 stacked, or the
 * four weight gradients of an encoder layer.  Every array is a HOST array of `count` entries; A[k], B[k], B2[k], C32[k]
 * are DEVICE pointers (B2 either given for every problem or NULL itself); operands are dense (lda = K or M, ldb = K
 * or N, ldc = N as the storage flags imply).  The problems share a_trans / b_trans; shapes may differ.  Same
 * requirements and error behaviour as sama_op_gemm_bf16. */
sama_status sama_op_gemm_bf16_batch(int32_t count, const void* const* A, const void* const* B, const void* const* B2,
                                    float* const* C32, const int32_t* M, const int32_t* N, const int32_t* K,
                                    int32_t a_trans, int32_t b_trans, void* hip_stream);

/* Base solver update, Adam form (Sec. 2; Kingma & Ba Alg. 1 with bias correction at step t >= 1), over n fp32
 * elements in place; theta16 (bf16 [n16], n16 <= n) receives the rounded leading part of theta, or NULL.  With
 * weight_decay != 0 the L2 term is added in front of the solver and g is overwritten with g + weight_decay * theta
 * (the gradient the solver was given, which the adaptation of Eq. 4 needs); with 0 g is only read. */
sama_status sama_op_adam(float* g, float* m, float* v, float* theta, void* theta16, int64_t n, int64_t n16,
                         int64_t t, float lr, float beta1, float beta2, float eps, float weight_decay, void* hip_stream);

/* Adaptation fused with the step size (Eq. 4-5, App. C): vdir = (du_adam/dg) . gmeta from the post-update moments at
 * step t, then scalars[0] = alpha / ||vdir||_2, scalars[1] = ||vdir||_2, status[0] = 1 if the norm is zero or not
 * finite (else 0).  partial: DEVICE scratch of 65536 doubles. */
sama_status sama_op_adapt_norm(const float* g, const float* m, const float* v, const float* gmeta, float* vdir,
                               double* partial, int64_t n, int64_t t, float lr, float beta1, float beta2, float eps,
                               float alpha, float* scalars, int64_t* status, void* hip_stream);

/* sama_op_adapt_norm for callers that cannot allocate or pass device scratch: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments without `partial`, same results bit for bit: the
 * partial sums live in a 512 KB array inside the library's device image (one copy per GPU, held until the process
 * ends) whose address is resolved once per device at the first call there.  The call allocates nothing.  n must not
 * exceed SAMA_OP_STATIC_MAX_N; a larger n returns SAMA_EINVAL, launches nothing, and sama_op_last_error() says why.
 * Every call on a GPU shares that GPU's array: calls that overlap in time on one GPU (different streams or threads)
 * race on it -- serialise them, or use sama_op_adapt_norm with separate scratch buffers.  Nothing in the array needs
 * clearing between calls (each call overwrites the entries it reads). */
#define SAMA_OP_STATIC_MAX_N ((int64_t)1 << 29)
sama_status sama_op_adapt_norm_static(const float* g, const float* m, const float* v, const float* gmeta, float* vdir,
                                      int64_t n, int64_t t, float lr, float beta1, float beta2, float eps, float alpha,
                                      float* scalars, int64_t* status, void* hip_stream);
/* Text of the last error of an op-level call on this thread (HOST string owned by the library, "" if none); set by
 * sama_op_adapt_norm_static. */
const char* sama_op_last_error(void);

/* Low halves of theta +- eps v against the bf16 working copy (Eq. 5): lo_p/lo_m[k] = bf16((theta[k] +- eps v[k]) -
 * float(bf16(theta[k]))), eps read from DEVICE eps_ptr. */
sama_status sama_op_perturb_lo(const float* theta, const float* vdir, const float* eps_ptr, void* lo_p, void* lo_m,
                               int64_t n16, void* hip_stream);

/* theta <- theta - eps v (end of Sec. 3.2), refreshing theta16 like sama_op_adam. */
sama_status sama_op_nudge(float* theta, const float* vdir, const float* eps_ptr, void* theta16, int64_t n, int64_t n16,
                          void* hip_stream);

/* Diagnostic switches, process-wide, for tests and profiling.  They take effect from the next launch and are not
 * thread-safe.
 *  - sama_dev_gemm_shape(id): every bf16 GEMM launch uses block tile `id`: 1..7 are the single-term tiles (a hi+lo
 *    problem then runs as one contraction over the concatenated operands, which rounds differently from the hi+lo
 *    tiles), 11..15 the hi+lo tiles (single-term problems ignore them); 0 = the heuristic (default).  Within a class
 *    every tile gives the same bits.
 *  - sama_dev_side_stream(0): the encoder's backward passes keep every launch on the context's stream instead of
 *    running weight gradients and optimizer slices on the library's second stream (a per-kernel profile wants one
 *    stream); 1 = default.  Changes no result bit.
 *  - sama_dev_side_sink(0): the optimizer and adaptation slices wait for the end of the backward pass instead of
 *    following each layer's gradients; 1 = default.  Changes no result bit. */
void sama_dev_gemm_shape(int32_t id);
void sama_dev_side_stream(int32_t on);
void sama_dev_side_sink(int32_t on);

#ifdef __cplusplus
}
#endif
#endif /* SAMA_OPS_H */
