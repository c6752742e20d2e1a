// Section executor: validates a call, carves the caller's workspace, and sequences the kernels
// of a layer stack forward (teacher) or forward + backward (student / vision encoder).
//
// Tensors that live between kernels are stored in the section dtype, except the forward residual
// stream (layer inputs, post-attention sums, last layer output), which is the running sum of all
// branch outputs and is kept in fp32; norm statistics, log-sum-exps, weight gradients and the loss
// are fp32 too.  In forward+backward mode every layer keeps its
// input, both normed activations, the (rotated) qkv, the attention output and log-sum-exp, the
// post-attention residual, the FFN pre-activation and activation: nothing is recomputed.
#include <vector>

#include "common.h"
#include "launch.h"

namespace {

struct LayerBuf {
    void *x, *h1, *qkv, *o, *x2, *h2, *up, *act;
    float *lse, *rstd1, *mean1, *rstd2, *mean2;
};

struct Plan {
    std::vector<LayerBuf> layers;  // n_layers entries (backward) or 1 shared entry (forward only)
    void *xa, *xb;                 // forward-only residual ping-pong
    void *y_last;
    float *rstd_f, *mean_f;
    int32_t *pos;
    float *rope;
    // backward temporaries
    void *dy0, *dy1, *dx2, *dh, *d_o, *dqkv, *da, *dup, *dhs;
    void *norm_scratch, *attn_scratch;
    size_t bytes;
    bool bwd;                      // layers keep their activations for a backward pass
};

struct Dims {
    int n, d, dqkv, dattn, dup, f, nq, nkv, hd, max_seqlen;
    size_t es;
    bool dec;
};

Dims dims_of(const ms_section_config *c, int n, int max_seqlen) {
    Dims m;
    m.n = n; m.d = c->d_model; m.nq = c->n_q_heads; m.nkv = c->n_kv_heads; m.hd = c->head_dim;
    m.dqkv = (c->n_q_heads + 2 * c->n_kv_heads) * c->head_dim;
    m.dattn = c->n_q_heads * c->head_dim;
    m.dec = c->arch == MS_DECODER;
    m.f = c->d_ffn;
    m.dup = m.dec ? 2 * c->d_ffn : c->d_ffn;
    m.es = ms_dtype_size(c->dtype);
    m.max_seqlen = max_seqlen;
    return m;
}

Plan make_plan(const ms_section_config *c, int n, int max_seqlen, bool bwd, void *ws) {
    const Dims m = dims_of(c, n, max_seqlen);
    Arena a(ws);
    Plan p = {};
    const size_t N = (size_t)n;
    auto act = [&](size_t cols) { return a.take<void>(N * cols * m.es); };
    auto res = [&](size_t cols) { return a.take<void>(N * cols * 4); };   // residual stream: fp32
    auto f32 = [&](size_t cnt) { return a.take<float>(cnt * 4); };
    const int nbuf = bwd ? c->n_layers : 1;
    p.bwd = bwd;
    p.layers.resize(nbuf);
    for (auto &l : p.layers) {
        l.x = bwd ? res(m.d) : nullptr;
        l.h1 = act(m.d); l.qkv = act(m.dqkv); l.o = act(m.dattn); l.x2 = res(m.d); l.h2 = act(m.d);
        l.up = act(m.dup); l.act = act(m.f);
        l.lse = f32(N * m.nq); l.rstd1 = f32(N); l.mean1 = f32(N); l.rstd2 = f32(N); l.mean2 = f32(N);
    }
    if (!bwd) { p.xa = res(m.d); p.xb = res(m.d); }
    p.y_last = res(m.d);
    p.rstd_f = f32(N); p.mean_f = f32(N);
    p.pos = a.take<int32_t>(N * 4);
    p.rope = f32((size_t)max_seqlen * m.hd);  // [max_seqlen, hd/2] (cos, sin)
    if (bwd) {
        p.dy0 = act(m.d); p.dy1 = act(m.d); p.dx2 = act(m.d); p.dh = act(m.d); p.d_o = act(m.dattn);
        p.dqkv = act(m.dqkv); p.da = act(m.f); p.dup = act(m.dup); p.dhs = act(m.d);
        const int widest = m.dup > m.dqkv ? (m.dup > m.d ? m.dup : m.d) : (m.dqkv > m.d ? m.dqkv : m.d);
        p.norm_scratch = a.take<void>(ms_k_norm_backward_scratch_bytes(widest));
        p.attn_scratch = a.take<void>(ms_k_attention_backward_scratch_bytes(c->dtype, m.nq, m.nkv, m.hd, n));
    }
    p.bytes = a.off;
    return p;
}

ms_status validate_config(const ms_section_config *c) {
    if (!c) return ms_fail(MS_ERR_INVALID_ARG, "section: null config");
    if (c->arch != MS_DECODER && c->arch != MS_ENCODER) return ms_fail(MS_ERR_INVALID_ARG, "section: bad arch %d", c->arch);
    if (c->dtype != MS_BF16 && c->dtype != MS_F32) return ms_fail(MS_ERR_INVALID_ARG, "section: bad dtype %d", c->dtype);
    if (c->n_layers <= 0 || c->d_model <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0 || c->head_dim <= 0 ||
        c->d_ffn <= 0 || c->vocab < 0)
        return ms_fail(MS_ERR_SHAPE, "section: sizes must be positive");
    if (c->n_q_heads % c->n_kv_heads)
        return ms_fail(MS_ERR_SHAPE, "section: n_q_heads=%d is not a multiple of n_kv_heads=%d", c->n_q_heads, c->n_kv_heads);
    if (c->head_dim != 64 && c->head_dim != 80 && c->head_dim != 128)
        return ms_fail(MS_ERR_UNSUPPORTED, "section: head_dim=%d (supported: 64, 80, 128)", c->head_dim);
    if (c->d_model % 8 || c->d_ffn % 8)
        return ms_fail(MS_ERR_UNSUPPORTED, "section: d_model=%d and d_ffn=%d must be multiples of 8", c->d_model, c->d_ffn);
    if (!(c->norm_eps >= 0.f) || (c->arch == MS_DECODER && !(c->rope_base > 1.f)))
        return ms_fail(MS_ERR_INVALID_ARG, "section: norm_eps / rope_base out of range");
    return MS_OK;
}

// Limits of the kernels this call will launch, so that nothing fails after the first launch.
ms_status validate_limits(const ms_section_config *c, int n_tokens, bool backward) {
    if (backward && c->d_model > ms_norm_backward_max_d(c->dtype))
        return ms_fail(MS_ERR_UNSUPPORTED, "section: d_model=%d above %d, the widest row the norm backward kernel holds",
                       c->d_model, ms_norm_backward_max_d(c->dtype));
    if (c->dtype == MS_BF16 && !ms_attn_offsets_fit(n_tokens, c->n_q_heads, c->n_kv_heads, c->head_dim))
        return ms_fail(MS_ERR_UNSUPPORTED, "section: %d tokens x %d qkv columns exceed the 4 GiB the attention kernels address",
                       n_tokens, (c->n_q_heads + 2 * c->n_kv_heads) * c->head_dim);
    return MS_OK;
}

ms_status validate_batch(const ms_batch *b, int *max_seqlen) {
    if (!b) return ms_fail(MS_ERR_INVALID_ARG, "section: null batch");
    if (b->n_tokens < 0 || b->n_seqs < 0) return ms_fail(MS_ERR_INVALID_ARG, "section: negative batch size");
    *max_seqlen = 0;
    if (b->n_tokens == 0) return MS_OK;
    if (!b->cu_seqlens_host || !b->cu_seqlens_dev || b->n_seqs == 0)
        return ms_fail(MS_ERR_INVALID_ARG, "section: tokens without cu_seqlens");
    const int32_t *cu = b->cu_seqlens_host;
    if (cu[0] != 0 || cu[b->n_seqs] != b->n_tokens)
        return ms_fail(MS_ERR_INVALID_ARG, "section: cu_seqlens must start at 0 and end at n_tokens=%d", b->n_tokens);
    for (int i = 0; i < b->n_seqs; ++i) {
        if (cu[i + 1] < cu[i]) return ms_fail(MS_ERR_INVALID_ARG, "section: cu_seqlens decreases at %d", i);
        if (cu[i + 1] - cu[i] > *max_seqlen) *max_seqlen = cu[i + 1] - cu[i];
    }
    return MS_OK;
}

ms_status validate_ptrs(const ms_section_config *c, const ms_section_ptrs *w, const char *what) {
    if (!w || !w->layers) return ms_fail(MS_ERR_INVALID_ARG, "section: null %s", what);
    const bool enc = c->arch == MS_ENCODER;
    if ((c->vocab > 0 && !w->embedding) || !w->final_norm_g || (enc && !w->final_norm_b))
        return ms_fail(MS_ERR_INVALID_ARG, "section: %s: null embedding / final norm pointer", what);
    for (int i = 0; i < c->n_layers; ++i) {
        const ms_layer_ptrs &l = w->layers[i];
        if (!l.norm1_g || !l.w_qkv || !l.w_o || !l.norm2_g || !l.w_up || !l.w_down)
            return ms_fail(MS_ERR_INVALID_ARG, "section: %s: null pointer in layer %d", what, i);
        if (enc && (!l.norm1_b || !l.b_qkv || !l.b_o || !l.norm2_b || !l.b_up || !l.b_down))
            return ms_fail(MS_ERR_INVALID_ARG, "section: %s: null bias pointer in encoder layer %d", what, i);
    }
    return MS_OK;
}

struct Exec {
    const ms_section_config *c;
    Dims m;
    const ms_batch *b;
    Plan *p;
    hipStream_t s;
    int dt, kind;

    ms_status gemm(int ta, int tb, int M, int N, int K, const void *A, long lda, const void *B, long ldb, void *C,
                   long ldc, bool c_fp32, bool acc, const void *bias, const void *res, long ldr) {
        return ms_k_gemm(dt, ta, tb, M, N, K, 1.f, A, lda, B, ldb, C, ldc, c_fp32, acc, bias, res, ldr, res != nullptr,
                         acc ? 0 : 1, s);
    }
    // y[n, out] = x[n, in] W[out, in]^T (+ bias) (+ res); with a residual, res and y are the fp32 stream
    ms_status linear(const void *x, int in, const void *W, const void *bias, int out, void *y, const void *res) {
        return gemm(0, 0, m.n, out, in, x, in, W, in, y, out, res != nullptr, false, bias, res, out);
    }
    // dx[n, in] = dy[n, out] W[out, in]
    ms_status dgrad(const void *dy, int out, const void *W, int in, void *dx) {
        return gemm(0, 1, m.n, in, out, dy, out, W, in, dx, in, false, false, nullptr, nullptr, 0);
    }
    // dW[out, in] += dy[n, out]^T x[n, in];  db[out] += colsum(dy)
    ms_status wgrad(const void *dy, int out, const void *x, int in, void *dW, void *db) {
        MS_TRY(gemm(1, 1, out, in, m.n, dy, out, x, in, dW, in, true, true, nullptr, nullptr, 0));
        if (db && !m.dec) MS_TRY(ms_k_colsum(dt, m.n, out, dy, (float *)db, p->norm_scratch, s));
        return MS_OK;
    }

    ms_status prologue() {
        if (m.dec) {
            MS_TRY(ms_k_positions(m.n, b->n_seqs, b->cu_seqlens_dev, p->pos, s));
            MS_TRY(ms_k_rope_table(m.max_seqlen, m.hd, c->rope_base, p->rope, s));
        }
        return MS_OK;
    }

    ms_status layer_forward(const ms_layer_ptrs &w, const void *x, LayerBuf &l, void *y) {
        MS_TRY(ms_k_norm_forward(kind, dt, 1, m.n, m.d, c->norm_eps, x, w.norm1_g, w.norm1_b, l.h1, l.mean1, l.rstd1, s));
        MS_TRY(linear(l.h1, m.d, w.w_qkv, m.dec ? nullptr : w.b_qkv, m.dqkv, l.qkv, nullptr));
        if (m.dec) MS_TRY(ms_k_rope(dt, m.n, m.nq + m.nkv, m.hd, m.dqkv, l.qkv, p->pos, p->rope, 0, s));
        MS_TRY(ms_k_attention_forward(dt, m.dec, m.nq, m.nkv, m.hd, m.n, b->n_seqs, m.max_seqlen, b->cu_seqlens_dev,
                                      l.qkv, l.o, l.lse, s));
        MS_TRY(linear(l.o, m.dattn, w.w_o, m.dec ? nullptr : w.b_o, m.d, l.x2, x));
        MS_TRY(ms_k_norm_forward(kind, dt, 1, m.n, m.d, c->norm_eps, l.x2, w.norm2_g, w.norm2_b, l.h2, l.mean2, l.rstd2, s));
        // decoder, bf16: SwiGLU runs in the epilogue of the gate/up GEMM (the pre-activations are only written
        // when a backward pass will read them)
        void *gu = p->bwd ? l.up : nullptr;
        if (m.dec && dt == MS_BF16 && gemm_swiglu_supported(m.n, m.f, m.d, l.h2, m.d, w.w_up, m.d, l.act, m.f, gu, m.dup)) {
            MS_TRY(gemm_swiglu(m.n, m.f, m.d, l.h2, m.d, w.w_up, m.d, l.act, m.f, gu, m.dup, s));
        } else {
            MS_TRY(linear(l.h2, m.d, w.w_up, m.dec ? nullptr : w.b_up, m.dup, l.up, nullptr));
            MS_TRY(ms_k_act_forward(m.dec ? 0 : 1, dt, m.n, m.f, l.up, l.act, s));
        }
        MS_TRY(linear(l.act, m.f, w.w_down, m.dec ? nullptr : w.b_down, m.d, y, l.x2));
        return MS_OK;
    }

    // dy: gradient of the layer output; dx: gradient of the layer input (distinct buffers)
    ms_status layer_backward(const ms_layer_ptrs &w, const ms_layer_ptrs &g, const LayerBuf &l, const void *dy, void *dx) {
        MS_TRY(dgrad(dy, m.d, w.w_down, m.f, p->da));
        MS_TRY(wgrad(dy, m.d, l.act, m.f, g.w_down, g.b_down));
        MS_TRY(ms_k_act_backward(m.dec ? 0 : 1, dt, m.n, m.f, p->da, l.up, p->dup, s));
        MS_TRY(dgrad(p->dup, m.dup, w.w_up, m.d, p->dh));
        MS_TRY(wgrad(p->dup, m.dup, l.h2, m.d, g.w_up, g.b_up));
        MS_TRY(ms_k_norm_backward(kind, dt, 1, m.n, m.d, p->dh, l.x2, w.norm2_g, l.mean2, l.rstd2, dy, p->dx2,
                                  (float *)g.norm2_g, (float *)g.norm2_b, p->norm_scratch, s));
        MS_TRY(dgrad(p->dx2, m.d, w.w_o, m.dattn, p->d_o));
        MS_TRY(wgrad(p->dx2, m.d, l.o, m.dattn, g.w_o, g.b_o));
        MS_TRY(ms_k_attention_backward(dt, m.dec, m.nq, m.nkv, m.hd, m.n, b->n_seqs, m.max_seqlen, b->cu_seqlens_dev,
                                       l.qkv, l.o, l.lse, p->d_o, p->dqkv, p->attn_scratch, s));
        if (m.dec) MS_TRY(ms_k_rope(dt, m.n, m.nq + m.nkv, m.hd, m.dqkv, p->dqkv, p->pos, p->rope, 1, s));
        MS_TRY(dgrad(p->dqkv, m.dqkv, w.w_qkv, m.d, p->dh));
        MS_TRY(wgrad(p->dqkv, m.dqkv, l.h1, m.d, g.w_qkv, g.b_qkv));
        MS_TRY(ms_k_norm_backward(kind, dt, 1, m.n, m.d, p->dh, l.x, w.norm1_g, l.mean1, l.rstd1, p->dx2, dx,
                                  (float *)g.norm1_g, (float *)g.norm1_b, p->norm_scratch, s));
        return MS_OK;
    }
};

}  // namespace

extern "C" size_t ms_section_workspace_bytes(const ms_section_config *cfg, int32_t max_tokens, int32_t max_seqlen,
                                             int32_t need_backward) {
    if (validate_config(cfg) != MS_OK || max_tokens < 0 || max_seqlen < 0) return 0;
    return make_plan(cfg, max_tokens, max_seqlen, need_backward != 0, nullptr).bytes;
}

extern "C" ms_status ms_section_forward(const ms_section_config *cfg, const ms_section_ptrs *weights,
                                        const ms_batch *batch, const void *x_in, void *h_out, void *workspace_dev,
                                        size_t workspace_bytes, void *stream) {
    MS_TRY(validate_config(cfg));
    int max_seqlen = 0;
    MS_TRY(validate_batch(batch, &max_seqlen));
    if (batch->n_tokens == 0) return MS_OK;
    MS_TRY(validate_limits(cfg, batch->n_tokens, false));
    MS_TRY(validate_ptrs(cfg, weights, "weights"));
    if (!x_in || !h_out || !workspace_dev) return ms_fail(MS_ERR_INVALID_ARG, "section_forward: null pointer");
    Plan p = make_plan(cfg, batch->n_tokens, max_seqlen, false, workspace_dev);
    if (workspace_bytes < p.bytes)
        return ms_fail(MS_ERR_WORKSPACE, "section_forward: workspace %zu < %zu bytes", workspace_bytes, p.bytes);
    Exec e{cfg, dims_of(cfg, batch->n_tokens, max_seqlen), batch, &p, (hipStream_t)stream, cfg->dtype,
           cfg->arch == MS_ENCODER ? 1 : 0};
    MS_TRY(e.prologue());
    const void *x = x_in;
    if (cfg->vocab > 0) {
        MS_TRY(ms_k_embedding_forward(e.dt, 1, e.m.n, e.m.d, cfg->vocab, (const int32_t *)x_in, weights->embedding, p.xa, e.s));
        x = p.xa;
    } else if (e.dt == MS_BF16) {
        MS_TRY(launch_convert_bf16_to_f32(x_in, (float *)p.xa, (long)e.m.n * e.m.d, e.s));
        x = p.xa;
    }
    for (int li = 0; li < cfg->n_layers; ++li) {
        void *y = li + 1 == cfg->n_layers ? p.y_last : (x == p.xa ? p.xb : p.xa);
        MS_TRY(e.layer_forward(weights->layers[li], x, p.layers[0], y));
        x = y;
    }
    return ms_k_norm_forward(e.kind, e.dt, 1, e.m.n, e.m.d, cfg->norm_eps, x, weights->final_norm_g, weights->final_norm_b,
                             h_out, p.mean_f, p.rstd_f, e.s);
}

extern "C" ms_status ms_section_forward_backward(const ms_section_config *cfg, const ms_section_ptrs *weights,
                                                 const ms_section_ptrs *grads, const ms_batch *batch, const void *x_in,
                                                 void *h_out, const void *d_h_out, const ms_kd_config *kd,
                                                 const void *h_teacher, void *d_w_student, float *loss_dev,
                                                 float *kl_per_token_dev, void *d_x_in, void *workspace_dev,
                                                 size_t workspace_bytes, void *stream) {
    MS_TRY(validate_config(cfg));
    int max_seqlen = 0;
    MS_TRY(validate_batch(batch, &max_seqlen));
    hipStream_t s = (hipStream_t)stream;
    if (batch->n_tokens == 0) return (kd && loss_dev) ? launch_fill_f32(loss_dev, 1, 0.f, s) : MS_OK;
    if ((d_h_out != nullptr) == (kd != nullptr))
        return ms_fail(MS_ERR_INVALID_ARG, "section_forward_backward: give exactly one of d_h_out and kd");
    if (kd) {
        MS_TRY(validate_kd(kd, batch->n_tokens));
        if (kd->h_student != cfg->d_model || kd->dtype != cfg->dtype)
            return ms_fail(MS_ERR_SHAPE, "section_forward_backward: kd->h_student / dtype do not match the section");
        if (!loss_dev) return ms_fail(MS_ERR_INVALID_ARG, "section_forward_backward: loss_dev is null");
    }
    MS_TRY(validate_limits(cfg, batch->n_tokens, true));
    MS_TRY(validate_ptrs(cfg, weights, "weights"));
    MS_TRY(validate_ptrs(cfg, grads, "grads"));
    if (!x_in || !h_out || !workspace_dev || (kd && !h_teacher))
        return ms_fail(MS_ERR_INVALID_ARG, "section_forward_backward: null pointer");
    Plan p = make_plan(cfg, batch->n_tokens, max_seqlen, true, workspace_dev);
    const size_t kd_bytes = kd ? ms_kd_workspace_bytes(kd, batch->n_tokens) : 0;
    if (workspace_bytes < p.bytes + kd_bytes)
        return ms_fail(MS_ERR_WORKSPACE, "section_forward_backward: workspace %zu < %zu bytes", workspace_bytes, p.bytes + kd_bytes);
    Exec e{cfg, dims_of(cfg, batch->n_tokens, max_seqlen), batch, &p, s, cfg->dtype, cfg->arch == MS_ENCODER ? 1 : 0};
    MS_TRY(e.prologue());
    const int L = cfg->n_layers;
    const void *x = x_in;
    if (cfg->vocab > 0) {
        MS_TRY(ms_k_embedding_forward(e.dt, 1, e.m.n, e.m.d, cfg->vocab, (const int32_t *)x_in, weights->embedding, p.layers[0].x, s));
        x = p.layers[0].x;
    } else if (e.dt == MS_BF16) {
        MS_TRY(launch_convert_bf16_to_f32(x_in, (float *)p.layers[0].x, (long)e.m.n * e.m.d, s));
        x = p.layers[0].x;
    }
    for (int li = 0; li < L; ++li) {
        void *y = li + 1 == L ? p.y_last : p.layers[li + 1].x;
        p.layers[li].x = const_cast<void *>(x);
        MS_TRY(e.layer_forward(weights->layers[li], x, p.layers[li], y));
        x = y;
    }
    MS_TRY(ms_k_norm_forward(e.kind, e.dt, 1, e.m.n, e.m.d, cfg->norm_eps, p.y_last, weights->final_norm_g,
                             weights->final_norm_b, h_out, p.mean_f, p.rstd_f, s));
    const void *dh = d_h_out;
    if (kd) {
        MS_TRY(kd_forward_backward(kd, e.m.n, h_teacher, h_out, loss_dev, kl_per_token_dev, p.dhs, d_w_student,
                                   (char *)workspace_dev + p.bytes, workspace_bytes - p.bytes, s));
        dh = p.dhs;
    }
    void *dy = p.dy0;
    MS_TRY(ms_k_norm_backward(e.kind, e.dt, 1, e.m.n, e.m.d, dh, p.y_last, weights->final_norm_g, p.mean_f, p.rstd_f, nullptr,
                              dy, (float *)grads->final_norm_g, (float *)grads->final_norm_b, p.norm_scratch, s));
    for (int li = L - 1; li >= 0; --li) {
        void *dx = (li == 0 && cfg->vocab == 0 && d_x_in) ? d_x_in : (dy == p.dy0 ? p.dy1 : p.dy0);
        MS_TRY(e.layer_backward(weights->layers[li], grads->layers[li], p.layers[li], dy, dx));
        dy = dx;
    }
    if (cfg->vocab > 0)
        MS_TRY(ms_k_embedding_backward(e.dt, e.m.n, e.m.d, cfg->vocab, (const int32_t *)x_in, dy, (float *)grads->embedding, s));
    return MS_OK;
}
