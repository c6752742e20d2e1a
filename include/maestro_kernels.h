/*
 * maestro_kernels.h -- kernel-level entry points of the section-compute library.
 *
 * These are the individual steps that ms_section_forward / ms_section_forward_backward /
 * ms_kd_loss_forward_backward (maestro_section.h) are composed of, exported so that each
 * kernel can be checked against the CPU oracle and timed against its roofline on its own.
 * The paper inherits its per-GPU layer compute from an existing framework and describes
 * none of it (Sec. 4, experimental setup); the operations are the textbook definitions
 * fixed by the workload shapes.  Same conventions as maestro_section.h: all data
 * pointers are device memory owned by the caller, `dtype` is an ms_dtype (bf16 storage
 * with fp32 math, or fp32), calls enqueue on `stream` and return an ms_status.
 */
#ifndef MAESTRO_KERNELS_H
#define MAESTRO_KERNELS_H

#include "maestro_section.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Kernel selection of the bf16 GEMMs, for measurements and tests (host-side switch, affects later launches
 * from any thread; not meant to be changed while launches are being issued).  tile: 0 = automatic (by shape),
 * 128 or 256 = force that workgroup tile for the direct-to-LDS kernels, -1 = use only the generic kernel.
 * mfma16: 1 = v_mfma_f32_16x16x32_bf16, 0 = v_mfma_f32_32x32x16_bf16, -1 = default.  The process-wide defaults
 * come from the environment (MS_GEMM_TILE, MS_GEMM_MFMA16). */
ms_status ms_k_gemm_config(int32_t tile, int32_t mfma16);

/* C[M,N] = alpha * sum_k A(m,k) B(n,k) (+ bias[n]) (+ residual[m,n]), optionally C += .
 * trans_a = 0: A is [M,K] row-major (lda); 1: A is stored [K,M] (lda).
 * trans_b = 0: B is [N,K] row-major (ldb); 1: B is stored [K,N] (ldb).
 * c_fp32: C is fp32 regardless of dtype.  accumulate (needs c_fp32): C += result; with
 * split_k > 1 the K range is divided over that many workgroups that add atomically.
 * bias / residual are `dtype` (NULL = none), residual has leading dimension ldr and is fp32
 * instead if residual_fp32 != 0 (the residual stream of a bf16 section is kept in fp32).
 * bf16 needs K % 8 == 0 for a non-transposed operand, M (resp. N) % 8 == 0 for a
 * transposed one, and 16-byte aligned rows. */
ms_status ms_k_gemm(int32_t dtype, int32_t trans_a, int32_t trans_b, int32_t M, int32_t N, int32_t K,
                    float alpha, const void *A, int64_t lda, const void *B, int64_t ldb, void *C,
                    int64_t ldc, int32_t c_fp32, int32_t accumulate, const void *bias,
                    const void *residual, int64_t ldr, int32_t residual_fp32, int32_t split_k, void *stream);

/* Gate/up projection of a SwiGLU FFN with the activation fused into the GEMM (bf16 only):
 *   gate_up[M, 2F] = round(A[M,K] W[2F,K]^T)  (W rows: F gate rows, then F up rows; written if gate_up != NULL)
 *   act[M, F]      = silu(gate) * up, evaluated on the rounded pre-activations (what a separate kernel would read).
 * Needs K % 64 == 0, F % 4 == 0, 16-byte aligned rows; MS_ERR_UNSUPPORTED otherwise (the caller then runs
 * ms_k_gemm + ms_k_act_forward). */
ms_status ms_k_gemm_swiglu(int32_t M, int32_t F, int32_t K, const void *A, int64_t lda, const void *W, int64_t ldw,
                           void *act, int64_t ldact, void *gate_up, int64_t ldgu, void *stream);

/* kind 0: RMSNorm y = x rstd g; kind 1: LayerNorm y = (x - mean) rstd g + b.
 * mean (kind 1 only) and rstd are fp32 [n] outputs kept for the backward pass.
 * x_fp32 != 0: x is fp32 although dtype is bf16 (g, b, y stay bf16). */
ms_status ms_k_norm_forward(int32_t kind, int32_t dtype, int32_t x_fp32, int32_t n, int32_t d, float eps,
                            const void *x, const void *g, const void *b, void *y, float *mean,
                            float *rstd, void *stream);
/* dx = norm backward of dy (+ add, if add != NULL);  dg += sum_t dy xhat;  db += sum_t dy.
 * dg / db fp32 [d], accumulated.  scratch: fp32, ms_k_norm_backward_scratch_bytes(d). */
size_t ms_k_norm_backward_scratch_bytes(int32_t d);
ms_status ms_k_norm_backward(int32_t kind, int32_t dtype, int32_t x_fp32, int32_t n, int32_t d, const void *dy,
                             const void *x, const void *g, const float *mean, const float *rstd,
                             const void *add, void *dx, float *dg, float *db, void *scratch,
                             void *stream);

/* pos[t] = t - cu_seqlens[b(t)]: position of each packed token inside its sequence. */
ms_status ms_k_positions(int32_t n_tokens, int32_t n_seqs, const int32_t *cu_seqlens, int32_t *pos,
                         void *stream);
/* table[p, i] = (cos, sin)(p * base^(-2i/head_dim)), p < max_pos, i < head_dim/2; angles in fp64. */
ms_status ms_k_rope_table(int32_t max_pos, int32_t head_dim, float base, float *table, void *stream);
/* In-place half-split rotary embedding of the first n_heads heads of every row of
 * x[n, row_stride]; inverse != 0 rotates by the negative angle (backward pass). */
ms_status ms_k_rope(int32_t dtype, int32_t n, int32_t n_heads, int32_t head_dim, int64_t row_stride,
                    void *x, const int32_t *pos, const float *table, int32_t inverse, void *stream);

/* kind 0 SwiGLU: up[n, 2f] = [gate | up] -> a[n, f] = silu(gate) * up.
 * kind 1 GELU (erf): up[n, f] -> a[n, f]. */
ms_status ms_k_act_forward(int32_t kind, int32_t dtype, int32_t n, int32_t f, const void *up, void *a,
                           void *stream);
ms_status ms_k_act_backward(int32_t kind, int32_t dtype, int32_t n, int32_t f, const void *da,
                            const void *up, void *dup, void *stream);

/* x[t, :] = table[ids[t], :]; out_fp32 != 0 widens a bf16 table row to fp32 on the way.  An id outside
 * [0, vocab) embeds as a row of zeros and receives no gradient (never an out-of-bounds access). */
ms_status ms_k_embedding_forward(int32_t dtype, int32_t out_fp32, int32_t n, int32_t d, int32_t vocab,
                                 const int32_t *ids, const void *table, void *x, void *stream);
/* d_table[ids[t], :] += dx[t, :]  (fp32, atomic). */
ms_status ms_k_embedding_backward(int32_t dtype, int32_t n, int32_t d, int32_t vocab, const int32_t *ids,
                                  const void *dx, float *d_table, void *stream);

/* out[j] += sum_t x[t, j]  (fp32 [c], accumulated).  scratch as for the norm backward with d = c. */
ms_status ms_k_colsum(int32_t dtype, int32_t n, int32_t c, const void *x, float *out, void *scratch,
                      void *stream);

/* Softmax attention per sequence on packed tokens.  qkv[n, (nq + 2 nkv) hd]: per row all Q
 * heads, all K heads, all V heads.  o[n, nq hd].  lse[nq, n] fp32 = log-sum-exp of the scaled
 * scores (kept for the backward pass).  causal != 0 masks keys after the query.
 * max_seqlen: upper bound of the sequence lengths in cu_seqlens (sizes the launch). */
ms_status ms_k_attention_forward(int32_t dtype, int32_t causal, int32_t n_q_heads, int32_t n_kv_heads,
                                 int32_t head_dim, int32_t n_tokens, int32_t n_seqs, int32_t max_seqlen,
                                 const int32_t *cu_seqlens, const void *qkv, void *o, float *lse,
                                 void *stream);
/* dqkv[n, (nq + 2 nkv) hd] from d_o, with dK / dV summed over each KV head's query group.
 * scratch: ms_k_attention_backward_scratch_bytes(...) bytes. */
size_t ms_k_attention_backward_scratch_bytes(int32_t dtype, int32_t n_q_heads, int32_t n_kv_heads,
                                             int32_t head_dim, int32_t n_tokens);
ms_status ms_k_attention_backward(int32_t dtype, int32_t causal, int32_t n_q_heads, int32_t n_kv_heads,
                                  int32_t head_dim, int32_t n_tokens, int32_t n_seqs, int32_t max_seqlen,
                                  const int32_t *cu_seqlens, const void *qkv, const void *o,
                                  const float *lse, const void *d_o, void *dqkv, void *scratch,
                                  void *stream);

/* Per-kernel timing for roofline reports.  ms_profile_enable(1) makes the launchers bracket each
 * kernel launch with HIP events on the launch stream (host-side objects only; at most 16384
 * launches are kept, later ones are not recorded); ms_profile_enable(0) stops recording and
 * frees the events.  ms_profile_read synchronises the recorded events and returns, for one
 * kernel class, the number of launches, their summed duration in milliseconds and their summed
 * algorithmic work (flops for matrix-core kernels, bytes for memory-bound kernels).
 * Classes: 0 gemm NT, 1 gemm NN/TN/TT, 2 attention forward, 3 attention backward, 4 norm forward,
 * 5 norm backward, 6 activation forward, 7 activation backward, 8 rotary embedding,
 * 9 KD statistics, 10 KD logit gradient, 11 embedding / column sums / conversions. */
#define MS_PROFILE_CLASSES 12
ms_status ms_profile_enable(int32_t on);
ms_status ms_profile_read(int32_t kernel_class, int64_t *launches, double *total_ms, double *total_work);

/* Plain device copy of `bytes` bytes (a known-traffic kernel for calibrating counters). */
ms_status ms_k_copy(const void *src, void *dst, size_t bytes, void *stream);

/* Register-resident bf16 MFMA loop on every CU (no memory traffic in the loop): the matrix-core rate the chip
 * sustains at its clocks under load, as a reference beside the published peak.  Each of `workgroups` x 8 waves
 * issues iters x 8 independent v_mfma_f32_32x32x16_bf16 (mfma16 = 0) or iters x 16 independent
 * v_mfma_f32_16x16x32_bf16 (mfma16 = 1: the same flops); sink_dev (>= workgroups * 512 floats) receives one value
 * per lane so that the loop is not removed.  Algorithmic flops = workgroups * 8 * iters * 8 * 32768.
 * random_operands = 0: small constants in the operand registers (lowest bit activity); 1: pseudo-random signs
 * and mantissas with magnitudes 2^-4 .. 2^4, as real weights and activations have.  The chip's power management
 * lowers the clock under the second, so the two rates bracket what a bf16 kernel can reach on real data. */
ms_status ms_k_mfma_probe(int32_t workgroups, int32_t iters, int32_t random_operands, int32_t mfma16, float *sink_dev,
                          void *stream);

/* Clock monitor: one wave that runs for about `microseconds` (1 .. 1000000; bounded by a poll count as well) and
 * writes to out_dev[0] the shader-clock cycles and to out_dev[1] the ticks of the constant 100 MHz counter that
 * passed meanwhile: average shader clock = 100 MHz * out_dev[0] / out_dev[1].  Launched on a second stream it
 * reports the clock the chip's power management grants while the kernels of another stream run. */
ms_status ms_k_clock_monitor(int32_t microseconds, int64_t *out_dev, void *stream);

#ifdef __cplusplus
}
#endif
#endif
