// Internal launch helpers shared between the translation units of the library.
#pragma once
#include "common.h"

ms_status launch_fill_f32(float *p, long n, float v, hipStream_t s);
ms_status launch_convert_from_f32(int dtype, const float *src, void *dst, long n, hipStream_t s);
ms_status launch_convert_bf16_to_f32(const void *src, float *dst, long n, hipStream_t s);

// Student-logits GEMM whose epilogue consumes the logits instead of storing them (gemm.hip); mode 1: dz, mode 2:
// per-strip partial statistics [M][nparts][8] = (m_t, s_t, m_s, s_s, A, -, -, -) over 64-column strips.
bool gemm_kd_epilogue_supported(int M, int N, int K, const void *A, long lda, const void *B, long ldb, const float *zt,
                                long ldz, const void *dz, long lddz, int dz_fp32);
ms_status gemm_kd_epilogue(int mode, int M, int N, int K, const void *A, long lda, const void *B, long ldb, const float *zt,
                           long ldz, float *stats, float *part, int nparts, float inv_t, float coef, void *dz, long lddz,
                           int dz_fp32, hipStream_t s);

// Fused gate/up GEMM + SwiGLU (gemm.hip): act[M,F] = silu(A Wg^T) * (A Wu^T), W = [Wg | Wu] rows; gate_up (may be
// null) receives the rounded pre-activations [M, 2F].
bool gemm_swiglu_supported(int M, int F, int K, const void *A, long lda, const void *W, long ldw, const void *act, long ldact,
                           const void *gate_up, long ldgu);
ms_status gemm_swiglu(int M, int F, int K, const void *A, long lda, const void *W, long ldw, void *act, long ldact,
                      void *gate_up, long ldgu, hipStream_t s);

// KD-loss pieces (kd.hip)
ms_status kd_forward_backward(const ms_kd_config *kd, int n_tokens, const void *h_teacher, const void *h_student,
                              float *loss_dev, float *kl_tok_dev, void *d_h_student, void *d_w_student,
                              void *workspace, size_t workspace_bytes, hipStream_t s);
ms_status validate_kd(const ms_kd_config *kd, int n_tokens);

// Optional per-launch timing (api.cpp).  Usage: { ProfScope ps(cls, work, stream); kernel<<<...>>>(...); }
void prof_begin(int cls, double work, hipStream_t s, int *slot);
void prof_end(int slot, hipStream_t s);
struct ProfScope {
    int slot;
    hipStream_t s;
    ProfScope(int cls, double work, hipStream_t stream) : slot(-1), s(stream) { prof_begin(cls, work, stream, &slot); }
    ~ProfScope() { if (slot >= 0) prof_end(slot, s); }
};
