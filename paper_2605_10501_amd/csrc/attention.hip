// Variable-length softmax attention on packed tokens: host entry points and the scalar
// (one wave per query row) kernels used for fp32 data and for shapes the matrix-core kernels
// do not cover.  The matrix-core kernels live in attention_mfma.hip.
#include "common.h"
#include "launch.h"
#include "attention.h"

namespace {

__device__ __forceinline__ int find_seq(const int *cu, int n_seqs, int t) {
    int lo = 0, hi = n_seqs;  // largest b with cu[b] <= t (skips zero-length sequences)
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (cu[mid] <= t) lo = mid; else hi = mid;
    }
    return lo;
}

// grid (token, ceil(nq / 4)); wave = one query head.  Keys are visited 64 at a time: lanes first
// hold one key each (scores), then one or two output columns each (P V).
template <class T>
__global__ __launch_bounds__(256) void attn_fwd_scalar_kernel(const T *__restrict__ qkv, T *__restrict__ o,
                                                               float *__restrict__ lse, const int *__restrict__ cu,
                                                               int n_seqs, int n, int nq, int nkv, int hd, int causal,
                                                               float scale) {
    __shared__ float qs[4][128], ps[4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t = blockIdx.x;
    const int h = blockIdx.y * 4 + wave;
    const bool active = h < nq;
    const int hh = active ? h : nq - 1;
    const int b = find_seq(cu, n_seqs, t);
    const int s0 = cu[b], s1 = causal ? t + 1 : cu[b + 1];
    const long ld = (long)(nq + 2 * nkv) * hd;
    const int g = hh / (nq / nkv);
    const T *qp = qkv + (long)t * ld + (long)hh * hd;
    const T *kb = qkv + (long)nq * hd + (long)g * hd;
    const T *vb = qkv + (long)(nq + nkv) * hd + (long)g * hd;
    for (int d = lane; d < hd; d += 64) qs[wave][d] = to_f32(qp[d]);
    __syncthreads();
    float m = -INFINITY, l = 0.f, acc0 = 0.f, acc1 = 0.f;
    for (int j0 = s0; j0 < s1; j0 += 64) {
        const int j = j0 + lane;
        float sc = -INFINITY;
        if (j < s1) {
            const T *kp = kb + (long)j * ld;
            float dot = 0.f;
            for (int d = 0; d < hd; ++d) dot += qs[wave][d] * to_f32(kp[d]);
            sc = dot * scale;
        }
        const float mnew = fmaxf(m, wave_max(sc));
        const float pj = j < s1 ? __expf(sc - mnew) : 0.f;
        const float corr = m == -INFINITY ? 0.f : __expf(m - mnew);
        l = l * corr + wave_sum(pj);
        acc0 *= corr;
        acc1 *= corr;
        m = mnew;
        ps[wave][lane] = pj;
        __syncthreads();
        const int cnt = s1 - j0 < 64 ? s1 - j0 : 64;
        for (int jj = 0; jj < cnt; ++jj) {
            const T *vp = vb + (long)(j0 + jj) * ld;
            const float w = ps[wave][jj];
            if (lane < hd) acc0 += w * to_f32(vp[lane]);
            if (lane + 64 < hd) acc1 += w * to_f32(vp[lane + 64]);
        }
        __syncthreads();
    }
    if (!active) return;
    T *op = o + (long)t * nq * hd + (long)h * hd;
    if (lane < hd) op[lane] = from_f32<T>(acc0 / l);
    if (lane + 64 < hd) op[lane + 64] = from_f32<T>(acc1 / l);
    if (lane == 0) lse[(long)h * n + t] = m + __logf(l);
}

// Backward, same decomposition.  dQ is produced directly; dK and dV are accumulated with fp32
// atomics into dkv[n, 2 * nkv * hd] (K heads then V heads), converted afterwards.
template <class T>
__global__ __launch_bounds__(256) void attn_bwd_scalar_kernel(const T *__restrict__ qkv, const T *__restrict__ o,
                                                               const float *__restrict__ lse, const T *__restrict__ d_o,
                                                               T *__restrict__ dqkv, float *__restrict__ dkv,
                                                               const int *__restrict__ cu, int n_seqs, int n, int nq,
                                                               int nkv, int hd, int causal, float scale) {
    __shared__ float qs[4][128], dos[4][128], ps[4][64], dss[4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t = blockIdx.x;
    const int h = blockIdx.y * 4 + wave;
    const bool active = h < nq;
    const int hh = active ? h : nq - 1;
    const int b = find_seq(cu, n_seqs, t);
    const int s0 = cu[b], s1 = causal ? t + 1 : cu[b + 1];
    const long ld = (long)(nq + 2 * nkv) * hd;
    const long ldkv = (long)2 * nkv * hd;
    const int g = hh / (nq / nkv);
    const T *qp = qkv + (long)t * ld + (long)hh * hd;
    const T *kb = qkv + (long)nq * hd + (long)g * hd;
    const T *vb = qkv + (long)(nq + nkv) * hd + (long)g * hd;
    const T *dop = d_o + (long)t * nq * hd + (long)hh * hd;
    const T *op = o + (long)t * nq * hd + (long)hh * hd;
    float delta = 0.f;
    for (int d = lane; d < hd; d += 64) {
        qs[wave][d] = to_f32(qp[d]);
        const float dv = to_f32(dop[d]);
        dos[wave][d] = dv;
        delta += dv * to_f32(op[d]);
    }
    delta = wave_sum(delta);
    const float L = lse[(long)hh * n + t];
    __syncthreads();
    float dq0 = 0.f, dq1 = 0.f;
    for (int j0 = s0; j0 < s1; j0 += 64) {
        const int j = j0 + lane;
        float pj = 0.f, ds = 0.f;
        if (j < s1) {
            const T *kp = kb + (long)j * ld, *vp = vb + (long)j * ld;
            float dot = 0.f, dp = 0.f;
            for (int d = 0; d < hd; ++d) {
                dot += qs[wave][d] * to_f32(kp[d]);
                dp += dos[wave][d] * to_f32(vp[d]);
            }
            pj = __expf(dot * scale - L);
            ds = pj * (dp - delta) * scale;
        }
        ps[wave][lane] = pj;
        dss[wave][lane] = ds;
        __syncthreads();
        const int cnt = s1 - j0 < 64 ? s1 - j0 : 64;
        if (active)
            for (int jj = 0; jj < cnt; ++jj) {
                const long row = j0 + jj;
                const T *kp = kb + row * ld;
                const float w = ps[wave][jj], e = dss[wave][jj];
                float *dkp = dkv + row * ldkv + (long)g * hd;
                float *dvp = dkv + row * ldkv + (long)(nkv + g) * hd;
                if (lane < hd) {
                    dq0 += e * to_f32(kp[lane]);
                    unsafeAtomicAdd(dkp + lane, e * qs[wave][lane]);
                    unsafeAtomicAdd(dvp + lane, w * dos[wave][lane]);
                }
                if (lane + 64 < hd) {
                    dq1 += e * to_f32(kp[lane + 64]);
                    unsafeAtomicAdd(dkp + lane + 64, e * qs[wave][lane + 64]);
                    unsafeAtomicAdd(dvp + lane + 64, w * dos[wave][lane + 64]);
                }
            }
        __syncthreads();
    }
    if (!active) return;
    T *dqp = dqkv + (long)t * ld + (long)h * hd;
    if (lane < hd) dqp[lane] = from_f32<T>(dq0);
    if (lane + 64 < hd) dqp[lane + 64] = from_f32<T>(dq1);
}

// dqkv[t, nq*hd + c] = (T) dkv[t, c]
template <class T>
__global__ void dkv_convert_kernel(const float *__restrict__ dkv, T *__restrict__ dqkv, long total, int ckv, long ld,
                                   int qcols) {
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    long t = i / ckv;
    int c = i % ckv;
    dqkv[t * ld + qcols + c] = from_f32<T>(dkv[i]);
}

}  // namespace

static ms_status check_attn(const char *who, int dtype, int nq, int nkv, int hd, int n, int n_seqs, int max_seqlen,
                            const void *cu) {
    if (n < 0 || n_seqs < 0 || !cu) return ms_fail(MS_ERR_INVALID_ARG, "%s: bad batch", who);
    if (nq <= 0 || nkv <= 0 || nq % nkv) return ms_fail(MS_ERR_SHAPE, "%s: n_q_heads=%d must be a multiple of n_kv_heads=%d", who, nq, nkv);
    if (hd <= 0 || hd > 128) return ms_fail(MS_ERR_UNSUPPORTED, "%s: head_dim=%d above 128", who, hd);
    if (dtype != MS_BF16 && dtype != MS_F32) return ms_fail(MS_ERR_INVALID_ARG, "%s: bad dtype", who);
    if (max_seqlen < 0) return ms_fail(MS_ERR_INVALID_ARG, "%s: negative max_seqlen", who);
    return MS_OK;
}

extern "C" ms_status ms_k_attention_forward(int32_t dtype, int32_t causal, int32_t nq, int32_t nkv, int32_t hd,
                                            int32_t n, int32_t n_seqs, int32_t max_seqlen, const int32_t *cu,
                                            const void *qkv, void *o, float *lse, void *stream) {
    MS_TRY(check_attn("attention_forward", dtype, nq, nkv, hd, n, n_seqs, max_seqlen, cu));
    if (n == 0 || n_seqs == 0) return MS_OK;
    if (!qkv || !o || !lse) return ms_fail(MS_ERR_INVALID_ARG, "attention_forward: null pointer");
    hipStream_t s = (hipStream_t)stream;
    const float scale = 1.f / sqrtf((float)hd);
    ProfScope ps(2, 0.0, s);  // work (flops) depends on the sequence lengths: computed by the caller
    if (dtype == MS_BF16 && attn_mfma_forward_supported(hd))
        return attn_mfma_forward(causal, nq, nkv, hd, n, n_seqs, max_seqlen, cu, qkv, o, lse, s);
    dim3 grid(n, ms_cdiv(nq, 4));
    if (dtype == MS_BF16)
        attn_fwd_scalar_kernel<bf16_t><<<grid, 256, 0, s>>>((const bf16_t *)qkv, (bf16_t *)o, lse, cu, n_seqs, n, nq, nkv, hd, causal, scale);
    else
        attn_fwd_scalar_kernel<float><<<grid, 256, 0, s>>>((const float *)qkv, (float *)o, lse, cu, n_seqs, n, nq, nkv, hd, causal, scale);
    MS_LAUNCH_CHECK();
    return MS_OK;
}

extern "C" size_t ms_k_attention_backward_scratch_bytes(int32_t dtype, int32_t nq, int32_t nkv, int32_t hd, int32_t n) {
    if (nq <= 0 || nkv <= 0 || hd <= 0 || n < 0) return 0;
    if (dtype == MS_BF16 && attn_mfma_backward_supported(hd)) return attn_mfma_backward_scratch_bytes(nq, nkv, hd, n);
    return ms_align_up((size_t)n * 2 * nkv * hd * sizeof(float));
}

extern "C" ms_status ms_k_attention_backward(int32_t dtype, int32_t causal, int32_t nq, int32_t nkv, int32_t hd,
                                             int32_t n, int32_t n_seqs, int32_t max_seqlen, const int32_t *cu,
                                             const void *qkv, const void *o, const float *lse, const void *d_o,
                                             void *dqkv, void *scratch, void *stream) {
    MS_TRY(check_attn("attention_backward", dtype, nq, nkv, hd, n, n_seqs, max_seqlen, cu));
    if (n == 0 || n_seqs == 0) return MS_OK;
    if (!qkv || !o || !lse || !d_o || !dqkv || !scratch) return ms_fail(MS_ERR_INVALID_ARG, "attention_backward: null pointer");
    hipStream_t s = (hipStream_t)stream;
    const float scale = 1.f / sqrtf((float)hd);
    ProfScope ps(3, 0.0, s);
    if (dtype == MS_BF16 && attn_mfma_backward_supported(hd))
        return attn_mfma_backward(causal, nq, nkv, hd, n, n_seqs, max_seqlen, cu, qkv, o, lse, d_o, dqkv, scratch, s);
    float *dkv = (float *)scratch;
    const long total = (long)n * 2 * nkv * hd;
    MS_TRY(launch_fill_f32(dkv, total, 0.f, s));
    dim3 grid(n, ms_cdiv(nq, 4));
    const long ld = (long)(nq + 2 * nkv) * hd;
    if (dtype == MS_BF16) {
        attn_bwd_scalar_kernel<bf16_t><<<grid, 256, 0, s>>>((const bf16_t *)qkv, (const bf16_t *)o, lse, (const bf16_t *)d_o, (bf16_t *)dqkv, dkv, cu, n_seqs, n, nq, nkv, hd, causal, scale);
        MS_LAUNCH_CHECK();
        dkv_convert_kernel<bf16_t><<<ms_cdiv(total, 256), 256, 0, s>>>(dkv, (bf16_t *)dqkv, total, 2 * nkv * hd, ld, nq * hd);
    } else {
        attn_bwd_scalar_kernel<float><<<grid, 256, 0, s>>>((const float *)qkv, (const float *)o, lse, (const float *)d_o, (float *)dqkv, dkv, cu, n_seqs, n, nq, nkv, hd, causal, scale);
        MS_LAUNCH_CHECK();
        dkv_convert_kernel<float><<<ms_cdiv(total, 256), 256, 0, s>>>(dkv, (float *)dqkv, total, 2 * nkv * hd, ld, nq * hd);
    }
    MS_LAUNCH_CHECK();
    return MS_OK;
}
