// Matrix-core attention kernels (attention_mfma.hip); bf16 only.
#pragma once
#include "common.h"

bool attn_mfma_forward_supported(int head_dim);
bool attn_mfma_backward_supported(int head_dim);
ms_status attn_mfma_forward(int causal, int nq, int nkv, int hd, int n, int n_seqs, int max_seqlen, const int *cu,
                            const void *qkv, void *o, float *lse, hipStream_t s);
size_t attn_mfma_backward_scratch_bytes(int nq, int nkv, int hd, int n);
ms_status attn_mfma_backward(int causal, int nq, int nkv, int hd, int n, int n_seqs, int max_seqlen, const int *cu,
                             const void *qkv, const void *o, const float *lse, const void *d_o, void *dqkv,
                             void *scratch, hipStream_t s);
