// Stand-in for the device kernels, for host-only sanitizer runs of the library's argument, plan and workspace logic.
//
// Every kernel-level entry point that the section executor calls is replaced by a function that touches each of
// its buffers over the full extent the real kernel reads or writes (host memory here): inputs are read byte by byte,
// outputs are filled.  With every buffer allocated at exactly its documented size, AddressSanitizer then reports any
// call whose pointers or sizes do not fit -- an arena carve-out beyond ms_*_workspace_bytes, a mis-sized temporary, a
// wrong leading dimension.  Nothing here computes anything.
#include <stdint.h>
#include <string.h>

#include <map>
#include <string>

#include "maestro_kernels.h"
#include "maestro_section.h"

struct ihipStream_t;
typedef ihipStream_t *hipStream_t;
ms_status ms_fail(ms_status code, const char *fmt, ...);
struct KdPlanView { float *zt, *zs, *stats, *dhs; void *dz; size_t bytes; int tb; bool keep; };

std::map<std::string, long> g_calls;          // how often each stand-in ran (read by the driver)
volatile unsigned g_sink;

static size_t es_of(int dtype) { return dtype == MS_BF16 ? 2 : 4; }
static size_t up256(size_t x) { return (x + 255) / 256 * 256; }
static void rd(const void *p, size_t bytes) {
    if (!p || !bytes) return;
    unsigned acc = 0;
    const unsigned char *b = (const unsigned char *)p;
    for (size_t i = 0; i < bytes; ++i) acc += b[i];
    g_sink = g_sink + acc;
}
static void wr(void *p, size_t bytes) {
    if (p && bytes) memset(p, 0x5a, bytes);
}
static size_t mat(long rows, long cols, long ld, size_t es) { return rows > 0 ? ((size_t)(rows - 1) * ld + cols) * es : 0; }

extern "C" {

size_t ms_k_norm_backward_scratch_bytes(int32_t d) { return d > 0 ? 2 * up256((size_t)1024 * d * 4) : 0; }

ms_status ms_k_norm_forward(int32_t kind, int32_t dtype, int32_t x_fp32, int32_t n, int32_t d, float, const void *x, const void *g,
                            const void *b, void *y, float *mean, float *rstd, void *) {
    ++g_calls["norm_forward"];
    const size_t es = es_of(dtype);
    rd(x, (size_t)n * d * (x_fp32 ? 4 : es)); rd(g, d * es);
    if (kind == 1) { rd(b, d * es); wr(mean, (size_t)n * 4); }
    wr(y, (size_t)n * d * es); wr(rstd, (size_t)n * 4);
    return MS_OK;
}

ms_status ms_k_norm_backward(int32_t kind, int32_t dtype, int32_t x_fp32, int32_t n, int32_t d, const void *dy, const void *x,
                             const void *g, const float *mean, const float *rstd, const void *add, void *dx, float *dg, float *db,
                             void *scratch, void *) {
    ++g_calls["norm_backward"];
    const size_t es = es_of(dtype);
    rd(dy, (size_t)n * d * es); rd(x, (size_t)n * d * (x_fp32 ? 4 : es)); rd(g, d * es); rd(rstd, (size_t)n * 4);
    rd(add, (size_t)n * d * es);
    if (kind == 1) { rd(mean, (size_t)n * 4); rd(db, (size_t)d * 4); wr(db, (size_t)d * 4); }
    wr(scratch, ms_k_norm_backward_scratch_bytes(d));
    wr(dx, (size_t)n * d * es); rd(dg, (size_t)d * 4); wr(dg, (size_t)d * 4);
    return MS_OK;
}

ms_status ms_k_gemm(int32_t dtype, int32_t ta, int32_t tb, int32_t M, int32_t N, int32_t K, float, const void *A, int64_t lda,
                    const void *B, int64_t ldb, void *C, int64_t ldc, int32_t c_fp32, int32_t accumulate, const void *bias,
                    const void *residual, int64_t ldr, int32_t residual_fp32, int32_t, void *) {
    ++g_calls["gemm"];
    const size_t es = es_of(dtype), ec = c_fp32 ? 4 : es;
    rd(A, ta ? mat(K, M, lda, es) : mat(M, K, lda, es));
    rd(B, tb ? mat(K, N, ldb, es) : mat(N, K, ldb, es));
    rd(bias, (size_t)N * es);
    rd(residual, mat(M, N, ldr, residual_fp32 ? 4 : es));
    if (accumulate) rd(C, mat(M, N, ldc, ec));
    // row by row: the gaps between rows (ldc > N) belong to somebody else
    for (int m = 0; m < M; ++m) wr((char *)C + (size_t)m * ldc * ec, (size_t)N * ec);
    return MS_OK;
}

ms_status ms_k_positions(int32_t n, int32_t n_seqs, const int32_t *cu, int32_t *pos, void *) {
    ++g_calls["positions"];
    rd(cu, (size_t)(n_seqs + 1) * 4); wr(pos, (size_t)n * 4);
    return MS_OK;
}

ms_status ms_k_rope_table(int32_t max_pos, int32_t hd, float, float *table, void *) {
    ++g_calls["rope_table"];
    wr(table, (size_t)max_pos * hd * 4);
    return MS_OK;
}

ms_status ms_k_rope(int32_t dtype, int32_t n, int32_t n_heads, int32_t hd, int64_t row_stride, void *x, const int32_t *pos,
                    const float *table, int32_t, void *) {
    ++g_calls["rope"];
    const size_t es = es_of(dtype);
    rd(pos, (size_t)n * 4); rd(table, (size_t)hd * 4);
    for (int t = 0; t < n; ++t) { rd((char *)x + (size_t)t * row_stride * es, (size_t)n_heads * hd * es); wr((char *)x + (size_t)t * row_stride * es, (size_t)n_heads * hd * es); }
    return MS_OK;
}

ms_status ms_k_act_forward(int32_t kind, int32_t dtype, int32_t n, int32_t f, const void *up, void *a, void *) {
    ++g_calls["act_forward"];
    rd(up, (size_t)n * (kind == 0 ? 2 * f : f) * es_of(dtype)); wr(a, (size_t)n * f * es_of(dtype));
    return MS_OK;
}

ms_status ms_k_act_backward(int32_t kind, int32_t dtype, int32_t n, int32_t f, const void *da, const void *up, void *dup, void *) {
    ++g_calls["act_backward"];
    const size_t w = (size_t)n * (kind == 0 ? 2 * f : f) * es_of(dtype);
    rd(da, (size_t)n * f * es_of(dtype)); rd(up, w); wr(dup, w);
    return MS_OK;
}

ms_status ms_k_embedding_forward(int32_t dtype, int32_t out_fp32, int32_t n, int32_t d, int32_t vocab, const int32_t *ids,
                                 const void *table, void *x, void *) {
    ++g_calls["embedding_forward"];
    rd(ids, (size_t)n * 4); rd(table, (size_t)vocab * d * es_of(dtype)); wr(x, (size_t)n * d * (out_fp32 ? 4 : es_of(dtype)));
    return MS_OK;
}

ms_status ms_k_embedding_backward(int32_t dtype, int32_t n, int32_t d, int32_t vocab, const int32_t *ids, const void *dx,
                                  float *d_table, void *) {
    ++g_calls["embedding_backward"];
    rd(ids, (size_t)n * 4); rd(dx, (size_t)n * d * es_of(dtype)); rd(d_table, (size_t)vocab * d * 4); wr(d_table, (size_t)vocab * d * 4);
    return MS_OK;
}

ms_status ms_k_colsum(int32_t dtype, int32_t n, int32_t c, const void *x, float *out, void *scratch, void *) {
    ++g_calls["colsum"];
    rd(x, (size_t)n * c * es_of(dtype)); rd(out, (size_t)c * 4); wr(out, (size_t)c * 4); wr(scratch, ms_k_norm_backward_scratch_bytes(c));
    return MS_OK;
}

size_t ms_k_attention_backward_scratch_bytes(int32_t, int32_t nq, int32_t nkv, int32_t hd, int32_t n) {
    return up256((size_t)nq * n * 4) + up256((size_t)n * 2 * nkv * hd * 4);
}

ms_status ms_k_attention_forward(int32_t dtype, int32_t, int32_t nq, int32_t nkv, int32_t hd, int32_t n, int32_t n_seqs, int32_t,
                                 const int32_t *cu, const void *qkv, void *o, float *lse, void *) {
    ++g_calls["attention_forward"];
    const size_t es = es_of(dtype);
    rd(cu, (size_t)(n_seqs + 1) * 4); rd(qkv, (size_t)n * (nq + 2 * nkv) * hd * es);
    wr(o, (size_t)n * nq * hd * es); wr(lse, (size_t)nq * n * 4);
    return MS_OK;
}

ms_status ms_k_attention_backward(int32_t dtype, int32_t, int32_t nq, int32_t nkv, int32_t hd, int32_t n, int32_t n_seqs, int32_t,
                                  const int32_t *cu, const void *qkv, const void *o, const float *lse, const void *d_o,
                                  void *dqkv, void *scratch, void *) {
    ++g_calls["attention_backward"];
    const size_t es = es_of(dtype);
    rd(cu, (size_t)(n_seqs + 1) * 4); rd(qkv, (size_t)n * (nq + 2 * nkv) * hd * es); rd(o, (size_t)n * nq * hd * es);
    rd(lse, (size_t)nq * n * 4); rd(d_o, (size_t)n * nq * hd * es);
    wr(scratch, ms_k_attention_backward_scratch_bytes(dtype, nq, nkv, hd, n));
    wr(dqkv, (size_t)n * (nq + 2 * nkv) * hd * es);
    return MS_OK;
}

}  // extern "C"

bool gemm_swiglu_supported(int, int F, int K, const void *, long, const void *, long, const void *, long, const void *, long) {
    return K % 64 == 0 && F % 4 == 0;
}

ms_status gemm_swiglu(int M, int F, int K, const void *A, long lda, const void *W, long ldw, void *act, long ldact, void *gate_up,
                      long ldgu, hipStream_t) {
    ++g_calls["gemm_swiglu"];
    rd(A, mat(M, K, lda, 2)); rd(W, mat(2L * F, K, ldw, 2));
    wr(act, mat(M, F, ldact, 2)); wr(gate_up, mat(M, 2L * F, ldgu, 2));
    return MS_OK;
}

ms_status launch_fill_f32(float *p, long n, float, hipStream_t) { ++g_calls["fill"]; wr(p, (size_t)n * 4); return MS_OK; }
ms_status launch_convert_bf16_to_f32(const void *src, float *dst, long n, hipStream_t) {
    ++g_calls["convert"];
    rd(src, (size_t)n * 2); wr(dst, (size_t)n * 4);
    return MS_OK;
}

ms_status validate_kd(const ms_kd_config *kd, int n_tokens);
ms_status kd_forward_backward(const ms_kd_config *kd, int n, const void *h_t, const void *h_s, float *loss, float *kl, void *d_h_s,
                              void *d_w_s, void *ws, size_t ws_bytes, hipStream_t) {
    ++g_calls["kd"];
    ms_status st = validate_kd(kd, n);
    if (st != MS_OK) return st;
    const size_t es = es_of(kd->dtype), need = ms_kd_workspace_bytes(kd, n);
    if (ws_bytes < need) return ms_fail(MS_ERR_WORKSPACE, "kd (stand-in): workspace %zu < %zu", ws_bytes, need);
    rd(h_t, (size_t)n * kd->h_teacher * es); rd(h_s, (size_t)n * kd->h_student * es);
    wr(ws, need); wr(loss, 4); wr(kl, (size_t)n * 4); wr(d_h_s, (size_t)n * kd->h_student * es);
    rd(d_w_s, (size_t)kd->vocab * kd->h_student * 4); wr(d_w_s, (size_t)kd->vocab * kd->h_student * 4);
    return MS_OK;
}
