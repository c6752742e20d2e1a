// Host-side plan of the KD step: how its workspace is carved and which configurations it accepts.  No device code:
// this part also builds for the host alone (sanitizer runs of the argument and workspace logic).
#pragma once
#include "common.h"

constexpr int kKdStat = 8;  // floats per token: m_t, s_t, m_s, s_s, A, KL, lse_t, lse_s

struct KdPlan {
    float *zt, *zs, *stats, *dhs;
    void *dz;
    size_t bytes;
    int tb;            // tokens per block
    bool keep;         // teacher logits of a block are kept across the two passes (one [tb, chunk] slab per chunk)
};

// token_block > 0: the tokens are processed in blocks of that many, and the teacher logits of the current block
// stay in the workspace between the statistics pass and the gradient pass (no teacher recompute); the cache
// is [n_chunks][token_block][chunk] fp32, independent of the number of tokens.
KdPlan kd_plan(const ms_kd_config *kd, int n, void *ws);
ms_status validate_kd(const ms_kd_config *kd, int n_tokens);
