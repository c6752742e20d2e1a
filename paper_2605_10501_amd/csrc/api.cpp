// Host-only parts of the C ABI: error reporting and the micro-batch packing step (no HIP runtime calls).
#include <stdarg.h>
#include <stdio.h>

#include <algorithm>
#include <numeric>
#include <vector>

#include "common.h"

static thread_local char g_last_error[512] = "";

ms_status ms_fail(ms_status code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_last_error, sizeof(g_last_error), fmt, ap);
    va_end(ap);
    return code;
}

extern "C" const char *ms_last_error(void) { return g_last_error; }

// Samples of length 0 do not activate the section and are dropped; the rest are taken in
// input order or longest first and packed greedily under the token budget.
extern "C" ms_status ms_pack_microbatches(const int32_t *lengths, int32_t n_samples, int32_t token_budget,
                                          int32_t policy, int32_t *order_out, int32_t *mb_offsets_out,
                                          int32_t *n_mb_out, int32_t *cu_seqlens_out) {
    if (n_samples < 0 || token_budget <= 0 || (policy != 0 && policy != 1))
        return ms_fail(MS_ERR_INVALID_ARG, "pack: n_samples=%d token_budget=%d policy=%d", n_samples, token_budget, policy);
    if (!n_mb_out || !mb_offsets_out || (n_samples > 0 && (!lengths || !order_out || !cu_seqlens_out)))
        return ms_fail(MS_ERR_INVALID_ARG, "pack: null pointer");
    std::vector<int32_t> kept;
    for (int32_t i = 0; i < n_samples; ++i) {
        if (lengths[i] < 0) return ms_fail(MS_ERR_INVALID_ARG, "pack: lengths[%d] is negative", i);
        if (lengths[i] > 0) kept.push_back(i);
    }
    if (policy == 1)
        std::stable_sort(kept.begin(), kept.end(), [&](int32_t a, int32_t b) { return lengths[a] > lengths[b]; });
    int32_t n_order = 0, n_mb = 0, n_cu = 0;
    int64_t tokens = 0;
    mb_offsets_out[0] = 0;
    for (int32_t i : kept) {
        if (tokens > 0 && tokens + lengths[i] > token_budget) {
            mb_offsets_out[++n_mb] = n_order;
            tokens = 0;
        }
        if (tokens == 0) cu_seqlens_out[n_cu++] = 0;
        order_out[n_order++] = i;
        tokens += lengths[i];
        if (tokens > INT32_MAX) return ms_fail(MS_ERR_INVALID_ARG, "pack: micro-batch exceeds 2^31 tokens");
        cu_seqlens_out[n_cu++] = (int32_t)tokens;
    }
    if (tokens > 0) mb_offsets_out[++n_mb] = n_order;
    *n_mb_out = n_mb;
    return MS_OK;
}
