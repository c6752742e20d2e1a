// Vocabulary-chunked lm_head + temperature softmax + KL(teacher || student).
//
// Pass 1 walks the vocabulary in chunks: two GEMMs give the chunk's teacher and student
// logits (fp32, [N, chunk], the only logits that ever exist), and a row kernel folds them into
// five running numbers per token: max and sum-of-exponentials of both models and the cross
// term sum_v e^{zt/T - m_t} (zt - zs)/T.  From those, KL_tok = A/s_t - lse_t + lse_s.
// Pass 2 recomputes each chunk's logits, forms dz = (scale/T)(q - p) in the storage dtype and
// feeds it to the two gradient GEMMs (dHs accumulated in fp32 over chunks, dWs chunk rows +=).
// On the bf16 fast path the student logits are never stored: the epilogue of their GEMM reads the
// teacher logits of the same tile and emits per-strip partial statistics (pass 1, merged per token
// by a small kernel) or dz itself (pass 2).
#include <mutex>

#include "common.h"
#include "launch.h"
#include "kd_host.h"

// Scratch of ms_kd_loss_forward_backward_static: one copy per GPU, held until the process ends.  In host code this
// name is only a handle for hipGetSymbolAddress; the device address it yields is what kernels and fills receive.
static __device__ __align__(256) unsigned char scratch[MS_KD_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kStat = kKdStat;  // floats per token: m_t, s_t, m_s, s_s, A, KL, lse_t, lse_s

__device__ __forceinline__ float block_max(float v, float *sm) {
    v = wave_max(v);
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = sm[0];
    for (int i = 1; i < (int)(blockDim.x >> 6); ++i) r = fmaxf(r, sm[i]);
    __syncthreads();
    return r;
}
__device__ __forceinline__ float block_sum(float v, float *sm) {
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = 0.f;
    for (int i = 0; i < (int)(blockDim.x >> 6); ++i) r += sm[i];
    __syncthreads();
    return r;
}

// one workgroup per token; zt / zs rows have leading dimension ld, cw valid columns (cw % 4 == 0)
__global__ __launch_bounds__(256) void kd_stats_kernel(const float *__restrict__ zt, const float *__restrict__ zs,
                                                        long ld, int cw, float inv_t, int first,
                                                        float *__restrict__ stats) {
    __shared__ float sm[4];
    const long t = blockIdx.x;
    const float4 *rt = (const float4 *)(zt + t * ld), *rs = (const float4 *)(zs + t * ld);
    const int nv = cw >> 2;
    float mt = -INFINITY, msv = -INFINITY;
    for (int i = threadIdx.x; i < nv; i += 256) {
        const float4 a = rt[i], b = rs[i];
        mt = fmaxf(mt, fmaxf(fmaxf(a.x, a.y), fmaxf(a.z, a.w)));
        msv = fmaxf(msv, fmaxf(fmaxf(b.x, b.y), fmaxf(b.z, b.w)));
    }
    mt = block_max(mt, sm) * inv_t;
    msv = block_max(msv, sm) * inv_t;
    float *st = stats + t * kStat;
    float m_t = mt, m_s = msv, f_t = 0.f, f_s = 0.f, o_st = 0.f, o_ss = 0.f, o_a = 0.f;
    if (!first) {
        const float omt = st[0], oms = st[2];
        o_st = st[1]; o_ss = st[3]; o_a = st[4];
        m_t = fmaxf(mt, omt);
        m_s = fmaxf(msv, oms);
        f_t = __expf(omt - m_t);
        f_s = __expf(oms - m_s);
    }
    float s_t = 0.f, s_s = 0.f, a_c = 0.f;
    for (int i = threadIdx.x; i < nv; i += 256) {
        const float4 a = rt[i], b = rs[i];
        const float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float et = __expf(av[e] * inv_t - m_t);
            s_t += et;
            a_c += et * (av[e] - bv[e]) * inv_t;
            s_s += __expf(bv[e] * inv_t - m_s);
        }
    }
    s_t = block_sum(s_t, sm);
    s_s = block_sum(s_s, sm);
    a_c = block_sum(a_c, sm);
    if (threadIdx.x == 0) {
        st[0] = m_t;
        st[1] = o_st * f_t + s_t;
        st[2] = m_s;
        st[3] = o_ss * f_s + s_s;
        st[4] = o_a * f_t + a_c;
    }
}

// per token: log-sum-exps for pass 2 (slots 6, 7 of its statistics) and its KL term (slot 5)
__global__ __launch_bounds__(256) void kd_token_kernel(float *__restrict__ stats, int n, float *__restrict__ kl_tok) {
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= n) return;
    float *st = stats + (long)t * kStat;
    const float lse_t = st[0] + __logf(st[1]);
    const float lse_s = st[2] + __logf(st[3]);
    const float kl = st[4] / st[1] - lse_t + lse_s;
    st[5] = kl;
    st[6] = lse_t;
    st[7] = lse_s;
    if (kl_tok) kl_tok[t] = kl;
}

// single workgroup: the scalar loss from the per-token KL terms (fixed summation order)
__global__ __launch_bounds__(1024) void kd_loss_kernel(const float *__restrict__ stats, int n, float loss_scale,
                                                        float *__restrict__ loss) {
    __shared__ float sm[16];
    float acc = 0.f;
    for (int t = threadIdx.x; t < n; t += 1024) acc += stats[(long)t * kStat + 5];
    acc = block_sum(acc, sm);
    if (threadIdx.x == 0) *loss = loss_scale * acc;
}

template <class T>
__global__ __launch_bounds__(256) void kd_dz_kernel(const float *__restrict__ zt, const float *__restrict__ zs, long ld,
                                                    int cw, float inv_t, float coef, const float *__restrict__ stats,
                                                    T *__restrict__ dz) {
    const long t = blockIdx.y;
    const int c4 = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (c4 >= cw) return;
    const float lse_t = stats[t * kStat + 6], lse_s = stats[t * kStat + 7];
    const float4 a = *(const float4 *)(zt + t * ld + c4), b = *(const float4 *)(zs + t * ld + c4);
    const float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
    T *o = dz + t * ld + c4;
#pragma unroll
    for (int e = 0; e < 4; ++e)
        o[e] = from_f32<T>(coef * (__expf(bv[e] * inv_t - lse_s) - __expf(av[e] * inv_t - lse_t)));
}

// Fused path: merges the per-strip partial statistics that the student-logits GEMM epilogue wrote for one
// chunk ([n][nparts][8]: m_t, s_t, m_s, s_s, A) into the running per-token statistics.  One wave per token.
__global__ __launch_bounds__(256) void kd_combine_kernel(const float *__restrict__ part, int nparts, int n, int first,
                                                          float *__restrict__ stats) {
    const int lane = threadIdx.x & 63;
    const long t = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= n) return;
    float m_t = -INFINITY, s_t = 0.f, m_s = -INFINITY, s_s = 0.f, a = 0.f;
    auto merge = [&](float mt_i, float st_i, float ms_i, float ss_i, float a_i) {
        const float nt = fmaxf(m_t, mt_i), ns = fmaxf(m_s, ms_i);
        const float ut = nt == -INFINITY ? 0.f : nt, us = ns == -INFINITY ? 0.f : ns;
        const float ft0 = __expf(m_t - ut), ft1 = __expf(mt_i - ut), fs0 = __expf(m_s - us), fs1 = __expf(ms_i - us);
        s_t = s_t * ft0 + st_i * ft1;
        a = a * ft0 + a_i * ft1;
        s_s = s_s * fs0 + ss_i * fs1;
        m_t = nt;
        m_s = ns;
    };
    for (int i = lane; i < nparts; i += 64) {
        const float *q = part + (t * nparts + i) * 8;
        const float4 v = *(const float4 *)q;
        merge(v.x, v.y, v.z, v.w, q[4]);
    }
    // across the wave: common maxima, rescaled sums
    const float wt = wave_max(m_t), wsm = wave_max(m_s);
    const float ut = wt == -INFINITY ? 0.f : wt, us = wsm == -INFINITY ? 0.f : wsm;
    const float ft = __expf(m_t - ut), fs = __expf(m_s - us);
    s_t = wave_sum(s_t * ft);
    a = wave_sum(a * ft);
    s_s = wave_sum(s_s * fs);
    m_t = wt;
    m_s = wsm;
    if (lane == 0) {
        float *st = stats + t * kStat;
        if (!first) merge(st[0], st[1], st[2], st[3], st[4]);
        st[0] = m_t; st[1] = s_t; st[2] = m_s; st[3] = s_s; st[4] = a;
    }
}

}  // namespace

ms_status kd_forward_backward(const ms_kd_config *kd, int n, const void *h_t, const void *h_s, float *loss_dev,
                              float *kl_tok_dev, void *d_h_s, void *d_w_s, void *workspace, size_t workspace_bytes,
                              hipStream_t s) {
    MS_TRY(validate_kd(kd, n));
    if (!loss_dev) return ms_fail(MS_ERR_INVALID_ARG, "kd: loss_dev is null");
    if (n == 0) return launch_fill_f32(loss_dev, 1, 0.f, s);
    if (!h_t || !h_s || !workspace) return ms_fail(MS_ERR_INVALID_ARG, "kd: null pointer");
    const KdPlan p = kd_plan(kd, n, workspace);
    if (workspace_bytes < p.bytes) return ms_fail(MS_ERR_WORKSPACE, "kd: workspace %zu < %zu bytes", workspace_bytes, p.bytes);
    const int V = kd->vocab, Cv = kd->chunk, Ht = kd->h_teacher, Hs = kd->h_student, dt = kd->dtype;
    const size_t es = ms_dtype_size(dt);
    const float inv_t = 1.f / kd->temperature;
    const char *wt = (const char *)kd->w_teacher_dev, *wsd = (const char *)kd->w_student_dev;
    const int passes = (d_h_s || d_w_s) ? 2 : 1;
    const bool keep = p.keep && passes == 2;
    if (d_h_s) MS_TRY(launch_fill_f32(p.dhs, (long)n * Hs, 0.f, s));
    for (int t0 = 0; t0 < n; t0 += p.tb) {
        const int nb = n - t0 < p.tb ? n - t0 : p.tb;
        const char *ht_b = (const char *)h_t + (size_t)t0 * Ht * es, *hs_b = (const char *)h_s + (size_t)t0 * Hs * es;
        float *stats_b = p.stats + (size_t)t0 * kStat, *dhs_b = p.dhs + (size_t)t0 * Hs;
        // bf16 fast path: the student-logits GEMM consumes its own output (statistics in pass 1, dz in pass 2)
        // together with the stored teacher logits; the zs buffer then only holds the per-strip partials
        bool fused = dt == MS_BF16;
        for (int v0 = 0; v0 < V && fused; v0 += Cv) {
            const int cw = V - v0 < Cv ? V - v0 : Cv;
            fused = gemm_kd_epilogue_supported(nb, cw, Hs, hs_b, Hs, wsd + (size_t)v0 * Hs * es, Hs, p.zt, Cv, p.dz, Cv, 0);
        }
        for (int pass = 0; pass < passes; ++pass) {
            for (int v0 = 0, ci = 0; v0 < V; v0 += Cv, ++ci) {
                const int cw = V - v0 < Cv ? V - v0 : Cv;
                float *zt = keep ? p.zt + (size_t)ci * p.tb * Cv : p.zt;
                if (pass == 0 || !keep)
                    MS_TRY(ms_k_gemm(dt, 0, 0, nb, cw, Ht, 1.f, ht_b, Ht, wt + (size_t)v0 * Ht * es, Ht, zt, Cv, 1, 0, nullptr, nullptr, 0, 0, 1, s));
                if (fused) {
                    const int nparts = ms_cdiv(cw, 64);
                    if (pass == 0) {
                        MS_TRY(gemm_kd_epilogue(2, nb, cw, Hs, hs_b, Hs, wsd + (size_t)v0 * Hs * es, Hs, zt, Cv, nullptr, p.zs, nparts,
                                                inv_t, 0.f, nullptr, 0, 0, s));
                        ProfScope ps(9, 32.0 * nb * nparts, s);
                        kd_combine_kernel<<<ms_cdiv(nb, 4), 256, 0, s>>>(p.zs, nparts, nb, v0 == 0, stats_b);
                        MS_LAUNCH_CHECK();
                        continue;
                    }
                    MS_TRY(gemm_kd_epilogue(1, nb, cw, Hs, hs_b, Hs, wsd + (size_t)v0 * Hs * es, Hs, zt, Cv, stats_b, nullptr, 0, inv_t,
                                            kd->loss_scale * inv_t, p.dz, Cv, 0, s));
                } else {
                    MS_TRY(ms_k_gemm(dt, 0, 0, nb, cw, Hs, 1.f, hs_b, Hs, wsd + (size_t)v0 * Hs * es, Hs, p.zs, Cv, 1, 0, nullptr, nullptr, 0, 0, 1, s));
                    if (pass == 0) {
                        ProfScope ps(9, 8.0 * nb * cw, s);
                        kd_stats_kernel<<<nb, 256, 0, s>>>(zt, p.zs, Cv, cw, inv_t, v0 == 0, stats_b);
                        MS_LAUNCH_CHECK();
                        continue;
                    }
                    const float coef = kd->loss_scale * inv_t;
                    dim3 grid(ms_cdiv(cw, 1024), nb);
                    {
                        ProfScope ps(10, (8.0 + es) * nb * cw, s);
                        if (dt == MS_BF16) kd_dz_kernel<bf16_t><<<grid, 256, 0, s>>>(zt, p.zs, Cv, cw, inv_t, coef, stats_b, (bf16_t *)p.dz);
                        else kd_dz_kernel<float><<<grid, 256, 0, s>>>(zt, p.zs, Cv, cw, inv_t, coef, stats_b, (float *)p.dz);
                    }
                    MS_LAUNCH_CHECK();
                }
                if (d_h_s)  // dHs[N, Hs] += dz[N, cw] Ws_c[cw, Hs]
                    MS_TRY(ms_k_gemm(dt, 0, 1, nb, Hs, cw, 1.f, p.dz, Cv, wsd + (size_t)v0 * Hs * es, Hs, dhs_b, Hs, 1, 1, nullptr, nullptr, 0, 0, 1, s));
                if (d_w_s)  // dWs_c[cw, Hs] += dz^T[cw, N] Hs[N, Hs]
                    MS_TRY(ms_k_gemm(dt, 1, 1, cw, Hs, nb, 1.f, p.dz, Cv, hs_b, Hs, (float *)d_w_s + (size_t)v0 * Hs, Hs, 1, 1, nullptr, nullptr, 0, 0, 0, s));
            }
            if (pass == 0) {
                kd_token_kernel<<<ms_cdiv(nb, 256), 256, 0, s>>>(stats_b, nb, kl_tok_dev ? kl_tok_dev + t0 : nullptr);
                MS_LAUNCH_CHECK();
            }
        }
    }
    kd_loss_kernel<<<1, 1024, 0, s>>>(p.stats, n, kd->loss_scale, loss_dev);
    MS_LAUNCH_CHECK();
    if (d_h_s) MS_TRY(launch_convert_from_f32(dt, p.dhs, d_h_s, (long)n * Hs, s));
    return MS_OK;
}

extern "C" ms_status ms_kd_loss_forward_backward(const ms_kd_config *kd, int32_t n_tokens, const void *h_teacher,
                                                 const void *h_student, float *loss_dev, float *kl_per_token_dev,
                                                 void *d_h_student, void *d_w_student, void *workspace_dev,
                                                 size_t workspace_bytes, void *stream) {
    return kd_forward_backward(kd, n_tokens, h_teacher, h_student, loss_dev, kl_per_token_dev, d_h_student, d_w_student,
                               workspace_dev, workspace_bytes, (hipStream_t)stream);
}

// ------------------------------------------------------------------ allocation-free variant
namespace {
constexpr int kMaxDevices = 64;
void *g_scratch_dev[kMaxDevices];       // device address of `scratch` on each GPU, resolved on first use
std::mutex g_scratch_mutex;

ms_status static_scratch(void **out) {
    int dev = -1;
    MS_CHECK_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return ms_fail(MS_ERR_UNSUPPORTED, "kd_static: device index %d out of range", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_dev[dev]) {
        void *p = nullptr;
        MS_CHECK_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return ms_fail(MS_ERR_HIP, "kd_static: no device address for the scratch array");
        g_scratch_dev[dev] = p;
    }
    *out = g_scratch_dev[dev];
    return MS_OK;
}
}  // namespace

extern "C" ms_status ms_kd_loss_forward_backward_static(const ms_kd_config *kd, int32_t n_tokens, const void *h_teacher,
                                                        const void *h_student, float *loss_dev, float *kl_per_token_dev,
                                                        void *d_h_student, void *d_w_student, void *stream) {
    MS_TRY(validate_kd(kd, n_tokens));
    const size_t need = kd_plan(kd, n_tokens, nullptr).bytes;
    if (need > (size_t)MS_KD_STATIC_SCRATCH_BYTES)
        return ms_fail(MS_ERR_WORKSPACE, "kd_static: %d tokens x chunk %d need %zu bytes of scratch, the built-in buffer holds %zu",
                       n_tokens, kd->chunk, need, (size_t)MS_KD_STATIC_SCRATCH_BYTES);
    void *ws = nullptr;
    MS_TRY(static_scratch(&ws));
    return kd_forward_backward(kd, n_tokens, h_teacher, h_student, loss_dev, kl_per_token_dev, d_h_student, d_w_student, ws,
                               (size_t)MS_KD_STATIC_SCRATCH_BYTES, (hipStream_t)stream);
}
