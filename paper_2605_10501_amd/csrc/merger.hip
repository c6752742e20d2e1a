// Vision -> language hand-off (Sec. 2.1, Sec. 4.1): 4:1 patch merger, MLP projector, scatter of the visual
// embeddings into the LLM's packed embedding stream, and the way back.  The merge itself costs nothing: the
// `merge` neighbouring tokens of a group are adjacent rows of the packed encoder output, so [merge * G, d_vit]
// IS [G, merge * d_vit].  The projector runs on the library's GEMM (bias in the epilogue) and GELU kernels;
// only the indexed row copies are new.
#include "common.h"
#include "launch.h"

namespace {

// SCATTER: dst[idx[r], :] = src[r, :];  else (gather): dst[r, :] = src[idx[r], :].  16 bytes per lane.
// A row whose index falls outside [0, n_indexed) is skipped (scatter) or zero-filled (gather).
template <bool SCATTER>
__global__ __launch_bounds__(256) void rows_indexed_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst,
                                                            const int *__restrict__ idx, long n_rows, int vec_per_row,
                                                            int n_indexed) {
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= n_rows * vec_per_row) return;
    const long r = i / vec_per_row;
    const int c = (int)(i % vec_per_row);
    const int k = idx[r];
    const bool ok = (unsigned)k < (unsigned)n_indexed;
    if (SCATTER) {
        if (ok) dst[(long)k * vec_per_row + c] = src[i];
    } else {
        dst[i] = ok ? src[(long)k * vec_per_row + c] : make_uint4(0, 0, 0, 0);
    }
}

struct MergerPlan {
    void *a1, *act, *out, *d_out, *d_act, *d_a1, *colsum;
    size_t bytes;
};

MergerPlan merger_plan(const ms_merger_config *c, int groups, void *ws) {
    Arena a(ws);
    MergerPlan p;
    const size_t es = ms_dtype_size(c->dtype), g = (size_t)groups;
    p.a1 = a.take<void>(g * c->d_hidden * es);
    p.act = a.take<void>(g * c->d_hidden * es);
    p.out = a.take<void>(g * c->d_llm * es);
    p.d_out = a.take<void>(g * c->d_llm * es);
    p.d_act = a.take<void>(g * c->d_hidden * es);
    p.d_a1 = a.take<void>(g * c->d_hidden * es);
    const int widest = c->d_hidden > c->d_llm ? c->d_hidden : c->d_llm;
    p.colsum = a.take<void>(ms_k_norm_backward_scratch_bytes(widest));
    p.bytes = a.off;
    return p;
}

ms_status validate(const ms_merger_config *c, const ms_merger_ptrs *w, int groups, int n_llm) {
    if (!c || !w) return ms_fail(MS_ERR_INVALID_ARG, "merger: null config or weights");
    if (c->dtype != MS_BF16 && c->dtype != MS_F32) return ms_fail(MS_ERR_INVALID_ARG, "merger: bad dtype");
    if (c->d_vit <= 0 || c->merge <= 0 || c->d_hidden <= 0 || c->d_llm <= 0) return ms_fail(MS_ERR_SHAPE, "merger: sizes must be positive");
    if (c->d_vit % 8 || c->d_hidden % 8 || c->d_llm % 8) return ms_fail(MS_ERR_UNSUPPORTED, "merger: widths must be multiples of 8");
    if (groups < 0 || n_llm < 0) return ms_fail(MS_ERR_INVALID_ARG, "merger: negative count");
    if (!w->w1 || !w->b1 || !w->w2 || !w->b2) return ms_fail(MS_ERR_INVALID_ARG, "merger: null weight pointer");
    return MS_OK;
}

}  // namespace

extern "C" size_t ms_merger_workspace_bytes(const ms_merger_config *cfg, int32_t max_groups) {
    if (!cfg || max_groups < 0 || cfg->d_hidden <= 0 || cfg->d_llm <= 0) return 0;
    return merger_plan(cfg, max_groups, nullptr).bytes;
}

extern "C" ms_status ms_merger_forward(const ms_merger_config *cfg, const ms_merger_ptrs *w, int32_t n_groups, const void *h_vit,
                                       const int32_t *positions_dev, int32_t n_llm_tokens, void *x_llm, void *workspace_dev,
                                       size_t workspace_bytes, void *stream) {
    MS_TRY(validate(cfg, w, n_groups, n_llm_tokens));
    if (n_groups == 0) return MS_OK;                              // a text-only batch: the encoder section was skipped
    if (!h_vit || !positions_dev || !x_llm || !workspace_dev) return ms_fail(MS_ERR_INVALID_ARG, "merger_forward: null pointer");
    const MergerPlan p = merger_plan(cfg, n_groups, workspace_dev);
    if (workspace_bytes < p.bytes) return ms_fail(MS_ERR_WORKSPACE, "merger: workspace %zu < %zu bytes", workspace_bytes, p.bytes);
    hipStream_t s = (hipStream_t)stream;
    const int dt = cfg->dtype, din = cfg->merge * cfg->d_vit, dh = cfg->d_hidden, dl = cfg->d_llm;
    MS_TRY(ms_k_gemm(dt, 0, 0, n_groups, dh, din, 1.f, h_vit, din, w->w1, din, p.a1, dh, 0, 0, w->b1, nullptr, 0, 0, 1, s));
    MS_TRY(ms_k_act_forward(1, dt, n_groups, dh, p.a1, p.act, s));
    MS_TRY(ms_k_gemm(dt, 0, 0, n_groups, dl, dh, 1.f, p.act, dh, w->w2, dh, p.out, dl, 0, 0, w->b2, nullptr, 0, 0, 1, s));
    const int vpr = (int)(dl * ms_dtype_size(dt) / 16);
    rows_indexed_kernel<true><<<ms_cdiv((long)n_groups * vpr, 256), 256, 0, s>>>((const uint4 *)p.out, (uint4 *)x_llm, positions_dev,
                                                                                 n_groups, vpr, n_llm_tokens);
    MS_LAUNCH_CHECK();
    return MS_OK;
}

extern "C" ms_status ms_merger_backward(const ms_merger_config *cfg, const ms_merger_ptrs *w, const ms_merger_ptrs *grads,
                                        int32_t n_groups, const void *h_vit, const int32_t *positions_dev, int32_t n_llm_tokens,
                                        const void *d_x_llm, void *d_h_vit, void *workspace_dev, size_t workspace_bytes,
                                        void *stream) {
    MS_TRY(validate(cfg, w, n_groups, n_llm_tokens));
    if (n_groups == 0) return MS_OK;
    if (!grads || !grads->w1 || !grads->b1 || !grads->w2 || !grads->b2) return ms_fail(MS_ERR_INVALID_ARG, "merger_backward: null gradient pointer");
    if (!h_vit || !positions_dev || !d_x_llm || !d_h_vit || !workspace_dev) return ms_fail(MS_ERR_INVALID_ARG, "merger_backward: null pointer");
    const MergerPlan p = merger_plan(cfg, n_groups, workspace_dev);
    if (workspace_bytes < p.bytes) return ms_fail(MS_ERR_WORKSPACE, "merger: workspace %zu < %zu bytes", workspace_bytes, p.bytes);
    hipStream_t s = (hipStream_t)stream;
    const int dt = cfg->dtype, din = cfg->merge * cfg->d_vit, dh = cfg->d_hidden, dl = cfg->d_llm;
    const int vpr = (int)(dl * ms_dtype_size(dt) / 16);
    rows_indexed_kernel<false><<<ms_cdiv((long)n_groups * vpr, 256), 256, 0, s>>>((const uint4 *)d_x_llm, (uint4 *)p.d_out, positions_dev,
                                                                                  n_groups, vpr, n_llm_tokens);
    MS_LAUNCH_CHECK();
    // second linear: d_act = d_out W2;  dW2 += d_out^T act;  db2 += colsum(d_out)
    MS_TRY(ms_k_gemm(dt, 0, 1, n_groups, dh, dl, 1.f, p.d_out, dl, w->w2, dh, p.d_act, dh, 0, 0, nullptr, nullptr, 0, 0, 1, s));
    MS_TRY(ms_k_gemm(dt, 1, 1, dl, dh, n_groups, 1.f, p.d_out, dl, p.act, dh, (void *)grads->w2, dh, 1, 1, nullptr, nullptr, 0, 0, 0, s));
    MS_TRY(ms_k_colsum(dt, n_groups, dl, p.d_out, (float *)grads->b2, p.colsum, s));
    MS_TRY(ms_k_act_backward(1, dt, n_groups, dh, p.d_act, p.a1, p.d_a1, s));
    // first linear: d_cat = d_a1 W1, written as the encoder's output gradient [merge * G, d_vit]
    MS_TRY(ms_k_gemm(dt, 0, 1, n_groups, din, dh, 1.f, p.d_a1, dh, w->w1, din, d_h_vit, din, 0, 0, nullptr, nullptr, 0, 0, 1, s));
    MS_TRY(ms_k_gemm(dt, 1, 1, dh, din, n_groups, 1.f, p.d_a1, dh, h_vit, din, (void *)grads->w1, din, 1, 1, nullptr, nullptr, 0, 0, 0, s));
    MS_TRY(ms_k_colsum(dt, n_groups, dh, p.d_a1, (float *)grads->b1, p.colsum, s));
    return MS_OK;
}
