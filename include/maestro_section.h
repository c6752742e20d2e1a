/*
 * maestro_section.h -- C ABI of one GPU's section compute on MI355X (gfx950).
 *
 * A "section" is a stack of transformer layers with an execution mode (paper
 * Sec. 3.1): a frozen teacher section runs forward only, a student or vision
 * encoder section runs forward and backward (Sec. 2.2, Sec. 2.1).  A section
 * consumes one packed variable-length micro-batch per call; each section has
 * its own micro-batch size (Sec. 3.2), so the token count is a per-call
 * argument.  The distillation loss takes the two hidden-state tensors and the
 * two lm_head matrices, because the teacher's output layer is colocated with
 * the student and logits never cross a section boundary (Sec. 3.1, Sec. 4.2).
 *
 * Conventions for every entry point
 *   - Pointers named *_dev / documented "device" are device memory, everything
 *     else is host memory.  The caller owns every buffer; the library neither
 *     allocates nor frees device memory.
 *   - Activations are row-major [tokens, features] ("packed"); sequence b is
 *     rows cu_seqlens[b] .. cu_seqlens[b+1]-1.  Weights are row-major
 *     [out_features, in_features].
 *   - dtype MS_BF16: activations, weights and activation gradients are bf16,
 *     accumulation is fp32, weight gradients / statistics / loss are fp32.
 *     dtype MS_F32: everything is fp32.
 *   - Calls only enqueue work on `stream` and return; no call synchronises.
 *   - Return value: MS_OK or a negative ms_status.  Argument and shape errors
 *     are detected on the host before anything is launched; ms_last_error()
 *     gives a thread-local message for the last failure.
 *   - Weight gradients are accumulated (+=) into the caller's fp32 buffers, so
 *     several micro-batches can be summed before an optimizer step (training
 *     equivalence, Sec. 3).  The caller zeroes them.
 *   - Kernels that accumulate with floating-point atomics (embedding gradient,
 *     split-K weight gradients) are not bitwise reproducible run to run.
 *   - Calls that share a workspace must not overlap in time.
 */
#ifndef MAESTRO_SECTION_H
#define MAESTRO_SECTION_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MS_OK = 0,
    MS_ERR_INVALID_ARG = -1,  /* null pointer, negative size, malformed cu_seqlens   */
    MS_ERR_SHAPE = -2,        /* inconsistent dimensions                             */
    MS_ERR_WORKSPACE = -3,    /* workspace smaller than ms_*_workspace_bytes says    */
    MS_ERR_UNSUPPORTED = -4,  /* e.g. head_dim not in {64, 80, 128}, d % 8 != 0      */
    MS_ERR_HIP = -5           /* a HIP runtime call failed                           */
} ms_status;

typedef enum { MS_F32 = 0, MS_BF16 = 1 } ms_dtype;

/* MS_DECODER: RMSNorm, rotary positions, SwiGLU FFN, causal attention, no biases.
 * MS_ENCODER: LayerNorm, exact GELU MLP, bidirectional attention, biases, no rotary. */
typedef enum { MS_DECODER = 0, MS_ENCODER = 1 } ms_arch;

typedef struct {
    int32_t arch;        /* ms_arch                                                  */
    int32_t dtype;       /* ms_dtype                                                 */
    int32_t n_layers;
    int32_t d_model;
    int32_t n_q_heads;
    int32_t n_kv_heads;  /* divides n_q_heads (grouped-query attention)              */
    int32_t head_dim;    /* 64, 80 or 128                                            */
    int32_t d_ffn;
    int32_t vocab;       /* > 0: x_in is int32 token ids [N]; 0: embeddings [N, d]   */
    float norm_eps;
    float rope_base;
} ms_section_config;

/* Device pointers of one layer.  Matrices are [out, in]:
 *   w_qkv  [(n_q + 2 n_kv) * head_dim, d]  rows: all Q heads, all K heads, all V heads
 *   w_o    [d, n_q * head_dim]
 *   w_up   decoder [2 d_ffn, d] (gate rows then up rows); encoder [d_ffn, d]
 *   w_down [d, d_ffn]
 * Bias and norm-shift pointers are used by MS_ENCODER only (ignored, may be NULL, for
 * MS_DECODER).  In an ms_section_grads the same fields point to fp32 buffers of the
 * same shapes. */
typedef struct {
    void *norm1_g, *norm1_b, *w_qkv, *b_qkv, *w_o, *b_o;
    void *norm2_g, *norm2_b, *w_up, *b_up, *w_down, *b_down;
} ms_layer_ptrs;

typedef struct {
    void *embedding;               /* [vocab, d] (NULL when vocab == 0)              */
    const ms_layer_ptrs *layers;   /* host array of n_layers entries                 */
    void *final_norm_g, *final_norm_b;
} ms_section_ptrs;

typedef struct {
    int32_t n_tokens;                 /* N = cu_seqlens[n_seqs]                      */
    int32_t n_seqs;
    const int32_t *cu_seqlens_dev;    /* device [n_seqs + 1]                         */
    const int32_t *cu_seqlens_host;   /* host copy of the same, validated:           */
                                      /* cu[0]=0, non-decreasing, cu[n_seqs]=N;      */
                                      /* zero-length entries are legal and skipped   */
} ms_batch;

typedef struct {
    int32_t vocab, h_teacher, h_student;
    int32_t chunk;                 /* vocabulary rows per chunk (multiple of 8)      */
    int32_t dtype;                 /* ms_dtype of hidden states and lm_heads         */
    float temperature;
    float loss_scale;              /* loss = loss_scale * sum_tokens KL_token        */
    const void *w_teacher_dev;     /* [vocab, h_teacher]                             */
    const void *w_student_dev;     /* [vocab, h_student]                             */
    int32_t token_block;           /* 0: chunk + recompute, at most [N, chunk] logits per model.  > 0 (multiple of */
                                   /* 8): variant for large HBM: tokens go in blocks of this many and a block's     */
                                   /* teacher logits ([token_block, vocab] fp32, independent of N) stay in the      */
                                   /* workspace between the two passes instead of being recomputed                  */
} ms_kd_config;

/* Bytes of device workspace the calls below need for up to max_tokens packed tokens
 * with sequences up to max_seqlen.  0 on invalid config. */
size_t ms_section_workspace_bytes(const ms_section_config *cfg, int32_t max_tokens,
                                  int32_t max_seqlen, int32_t need_backward);
size_t ms_kd_workspace_bytes(const ms_kd_config *kd, int32_t max_tokens);

/* Forward-only section (teacher; Sec. 2.2): h_out[N, d] = final_norm(layers(x_in)).
 * x_in: device, int32 ids [N] (cfg->vocab > 0) or embeddings [N, d].  h_out: device.
 * n_tokens == 0 is the "section skipped" case (Sec. 2.1): returns MS_OK, launches nothing. */
ms_status ms_section_forward(const ms_section_config *cfg, const ms_section_ptrs *weights,
                             const ms_batch *batch, const void *x_in, void *h_out,
                             void *workspace_dev, size_t workspace_bytes, void *stream);

/* Forward + backward section (student, or vision encoder; Sec. 2.2, Sec. 2.1).
 * Exactly one source of the output gradient:
 *   - d_h_out != NULL: upstream gradient [N, d] from a downstream section; kd must be NULL.
 *   - kd != NULL: the KL distillation loss against h_teacher[N, kd->h_teacher] is
 *     evaluated on h_out (kd->h_student must equal d_model); loss_dev (device float),
 *     kl_per_token_dev (device [N] or NULL) and d_w_student (device fp32 [vocab, d], +=)
 *     are produced as by ms_kd_loss_forward_backward.  The workspace must then cover
 *     ms_section_workspace_bytes(..., 1) + ms_kd_workspace_bytes(...).
 * grads: fp32, accumulated.  d_x_in: device [N, d] or NULL; ignored for token-id input
 * (the input gradient then is grads->embedding). */
ms_status ms_section_forward_backward(const ms_section_config *cfg, const ms_section_ptrs *weights,
                                      const ms_section_ptrs *grads, const ms_batch *batch,
                                      const void *x_in, void *h_out, const void *d_h_out,
                                      const ms_kd_config *kd, const void *h_teacher,
                                      void *d_w_student, float *loss_dev, float *kl_per_token_dev,
                                      void *d_x_in, void *workspace_dev, size_t workspace_bytes,
                                      void *stream);

/* Vocabulary-chunked lm_head + temperature softmax + KL(teacher || student) (Sec. 3.1,
 * Sec. 4.2).  Never holds more than [n_tokens, chunk] logits per model.
 *   p = softmax(h_teacher Wt^T / T), q = softmax(h_student Ws^T / T)
 *   kl_per_token = sum_v p (ln p - ln q);  *loss_dev = loss_scale * sum_tokens kl
 *   d_h_student = (loss_scale / T) (q - p) Ws           (overwritten; NULL: forward only)
 *   d_w_student += ((loss_scale / T) (q - p))^T h_student  (fp32; NULL: skipped)
 * No gradient is produced for the teacher. */
ms_status ms_kd_loss_forward_backward(const ms_kd_config *kd, int32_t n_tokens,
                                      const void *h_teacher, const void *h_student,
                                      float *loss_dev, float *kl_per_token_dev,
                                      void *d_h_student, void *d_w_student,
                                      void *workspace_dev, size_t workspace_bytes, void *stream);

/* The same computation for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving / evaluation loops, harnesses that forbid hipMalloc.  The scratch that the call above takes
 * from the caller's workspace (chunk logits, per-token statistics, the logit gradient, the fp32 d_h_student
 * accumulator) lives in a fixed device array inside the library instead: MS_KD_STATIC_SCRATCH_BYTES per GPU, held from
 * the library's first use on that GPU until the process ends.  The call allocates and frees nothing (with
 * ms_profile_enable(1) the launchers create HIP events: leave profiling off here).  A call whose
 * ms_kd_workspace_bytes(kd, n_tokens) exceeds MS_KD_STATIC_SCRATCH_BYTES is rejected with MS_ERR_WORKSPACE before
 * anything is launched (examples that fit: 1024 tokens with chunk 4096 and h_student 2048; 4096 tokens with chunk 1024).
 * All calls on one GPU share the one array: calls that overlap in time on a GPU (different streams or threads) race;
 * calls on one stream are ordered and each clears what it needs.  Results are those of ms_kd_loss_forward_backward. */
#define MS_KD_STATIC_SCRATCH_BYTES (64u << 20)
ms_status ms_kd_loss_forward_backward_static(const ms_kd_config *kd, int32_t n_tokens, const void *h_teacher,
                                             const void *h_student, float *loss_dev, float *kl_per_token_dev,
                                             void *d_h_student, void *d_w_student, void *stream);

/* Vision -> language hand-off (Sec. 2.1 and Sec. 4.1: the encoder's visual tokens are down-sampled 4:1 along the
 * sequence and joined with the text tokens to form the LLM's input; the operator itself is a reading: patch
 * merger + MLP projector).  Group g = visual tokens merge*g .. merge*g + merge-1 of the packed encoder output
 * (each sample's visual length must be a multiple of `merge`, so groups never straddle samples):
 *   cat[g]  = concat of the group's rows                      [merge * d_vit]   (no copy: adjacent rows)
 *   out[g]  = W2 gelu(W1 cat[g] + b1) + b2                    [d_llm]           (exact-erf GELU)
 *   x_llm[positions[g], :] = out[g]                           the LLM's packed embedding stream [n_llm_tokens, d_llm]
 * Text rows of x_llm are the caller's (embedding gather).  positions_dev: device int32 [n_groups], distinct;
 * a position outside [0, n_llm_tokens) is skipped (forward) and contributes a zero gradient (backward).
 * ms_merger_backward: d_x_llm [n_llm_tokens, d_llm] -> d_h_vit [merge * n_groups, d_vit] (overwritten) and
 * grads (fp32, same shapes as the weights, accumulated).  It reads the activations that ms_merger_forward left
 * in the workspace for the same n_groups: the workspace must not be touched in between.
 * w1 [d_hidden, merge * d_vit], b1 [d_hidden], w2 [d_llm, d_hidden], b2 [d_llm] in the storage type; all
 * widths multiples of 8.  n_groups == 0 (text-only batch) returns MS_OK and launches nothing. */
typedef struct {
    int32_t dtype;      /* ms_dtype */
    int32_t d_vit, merge, d_hidden, d_llm;
} ms_merger_config;
typedef struct {
    const void *w1, *b1, *w2, *b2;
} ms_merger_ptrs;
size_t ms_merger_workspace_bytes(const ms_merger_config *cfg, int32_t max_groups);
ms_status ms_merger_forward(const ms_merger_config *cfg, const ms_merger_ptrs *weights, int32_t n_groups,
                            const void *h_vit, const int32_t *positions_dev, int32_t n_llm_tokens,
                            void *x_llm, void *workspace_dev, size_t workspace_bytes, void *stream);
ms_status ms_merger_backward(const ms_merger_config *cfg, const ms_merger_ptrs *weights,
                             const ms_merger_ptrs *grads, int32_t n_groups, const void *h_vit,
                             const int32_t *positions_dev, int32_t n_llm_tokens, const void *d_x_llm,
                             void *d_h_vit, void *workspace_dev, size_t workspace_bytes, void *stream);

/* The student's parameter update (Sec. 2.2: only the student runs optimizer-driven parameter updates; the
 * paper names no optimizer, AdamW is the reading taken).  One fused pass over n elements, all device memory:
 *   g = grad_scale * grad;  m = beta1 m + (1 - beta1) g;  v = beta2 v + (1 - beta2) g^2
 *   master = master (1 - lr wd) - lr (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps)
 *   weight = round(master) in the section's storage type (MS_BF16 or MS_F32)
 * grad, master, m, v: fp32 [n], 16-byte aligned, updated in place (grad is read only unless zero_grad != 0,
 * which clears it for the next accumulation); weight: [n] of `dtype` (may be NULL).  step counts from 1.
 * Arithmetic in fp32. */
typedef struct {
    float lr, beta1, beta2, eps, weight_decay, grad_scale;
    int32_t step;
    int32_t zero_grad;
} ms_adamw_config;
ms_status ms_adamw_step(const ms_adamw_config *cfg, int32_t dtype, int64_t n, float *grad, float *master,
                        float *m, float *v, void *weight, void *stream);

/* Wavefront sample scheduling (Sec. 3.4, Algorithm 1); host code, all pointers are host memory.
 * tuples[n_samples][6] = (t_f_bc, t_f_c, t_f_ac, t_b_bc, t_b_c, t_b_ac): forward time before / within /
 * after the critical section, then backward time before (sections behind the critical one in forward
 * order) / within / after (sections in front of it) the critical section; non-negative, any unit.
 * ms_schedule_samples: stable sort by t_f_bc, then each remaining sample is inserted at the position
 * (lowest on ties; makespans within 1e-9 relative are ties) that gives the least simulated makespan; order_out[n_samples] receives sample indices
 * in execution order, *makespan_out (optional) the simulated makespan.  O(n^2) time for interleave != 0
 * (insertions are evaluated through (max, +) prefix states and suffix products), O(n^3) otherwise.
 * ms_schedule_makespan: makespan of a given order (a permutation of 0..n-1, else MS_ERR_INVALID_ARG) and
 * (optional) the time the critical section spends idle before its last job ends.
 * Timeline model: three serial servers (sections in front of the critical one, the critical section, the
 * sections behind it); a job starts when its server is free and the previous job on the sample's path
 * forward-in-front -> critical forward -> behind (forward + backward) -> critical backward ->
 * backward-in-front is done; the front server runs its forward jobs first; interleave != 0: the critical
 * section runs forward and backward sample by sample, else all forwards then all backwards. */
ms_status ms_schedule_samples(int32_t n_samples, const double *tuples, int32_t interleave,
                              int32_t *order_out, double *makespan_out);
ms_status ms_schedule_makespan(int32_t n_samples, const double *tuples, const int32_t *order,
                               int32_t interleave, double *makespan_out, double *critical_idle_out);

/* Host step that orders samples into packed micro-batches (Sec. 3.4 for the ordering
 * role; a sample of length 0 does not activate the section and is dropped, Sec. 2.1).
 * policy 0 keeps the input order, 1 sorts longest first (stable).  Greedy fill: a sample
 * that does not fit closes the open micro-batch; a sample above the budget stands alone.
 * All arrays are host memory sized for the worst case: order_out[n_samples],
 * mb_offsets_out[n_samples + 1], cu_seqlens_out[2 * n_samples] (per micro-batch a prefix
 * sum starting at 0, concatenated; micro-batch m with k samples occupies k + 1 entries). */
ms_status ms_pack_microbatches(const int32_t *lengths, int32_t n_samples, int32_t token_budget,
                               int32_t policy, int32_t *order_out, int32_t *mb_offsets_out,
                               int32_t *n_mb_out, int32_t *cu_seqlens_out);

const char *ms_last_error(void);

#ifdef __cplusplus
}
#endif
#endif
