// Internal launch helpers shared between the translation units of the library.
#pragma once
#include "common.h"

ms_status launch_fill_f32(float *p, long n, float v, hipStream_t s);
ms_status launch_convert_from_f32(int dtype, const float *src, void *dst, long n, hipStream_t s);
ms_status launch_convert_bf16_to_f32(const void *src, float *dst, long n, hipStream_t s);

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
