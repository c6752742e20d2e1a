// Matrix-core variable-length attention for bf16 (head_dim 64, 80, 128), forward.
//
// One workgroup (4 waves) owns 128 consecutive queries of one sequence and one query head; each
// wave owns 32 of them and keeps its Q fragments in registers.  Keys / values are visited 64 at a
// time through two LDS buffers (global -> registers -> LDS, one barrier per tile):
//   * K tile row-major [64 keys][head_dim] as 64-wide sub-tiles;
//   * V tile transposed while staged, Vt[head_dim][64 keys], so that the P V product can contract
//     over keys with 8-byte LDS reads.
// Scores are computed transposed, S^T = K Q^T (v_mfma_f32_32x32x16_bf16): in the accumulator
// layout a lane then holds 32 keys of ONE query, so the online-softmax row maximum and sum are
// register reductions plus a single cross-half shuffle, the rescale factor is a per-lane scalar,
// and the probabilities are already laid out as the B operand of O^T += Vt P^T.
#include "attention.h"
#include "launch.h"
#include "mfma_tiles.h"

namespace {

template <int HD> struct AttnDims {
    static constexpr int NKS = (HD + 63) / 64;   // 64-wide sub-tiles of a K (or Q) tile
    static constexpr int DB = (HD + 31) / 32;    // 32-row blocks of the transposed output
    static constexpr int KST = HD / 16;          // MFMA k-steps over head_dim
};

__device__ __forceinline__ bf16x8 pack8(const float *v) {
    bf16x8 r;
#pragma unroll
    for (int i = 0; i < 8; ++i) r[i] = (bf16_t)v[i];
    return r;
}

template <int HD, bool CAUSAL>
__global__ __launch_bounds__(256) void attn_fwd_mfma_kernel(const bf16_t *__restrict__ qkv, bf16_t *__restrict__ o,
                                                             float *__restrict__ lse, const int *__restrict__ cu, int n,
                                                             int nq, int nkv, float scale_log2e) {
    using D = AttnDims<HD>;
    constexpr int BQ = 128, BKV = 64;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    bf16_t *Ks = (bf16_t *)smem_raw;                          // [2][NKS][64 * 64]
    bf16_t *Vt = Ks + 2 * D::NKS * 64 * 64;                   // [2][DB * 32 * 64]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lrow = lane & 31, half = lane >> 5;
    const int b = blockIdx.z, h = blockIdx.y;
    const int s0 = cu[b], s1 = cu[b + 1];
    const int ntile = (s1 - s0 + BQ - 1) / BQ;
    const int qt = ntile - 1 - (int)blockIdx.x;               // long (late) tiles first
    if (qt < 0) return;
    const int g = h / (nq / nkv);
    const long ld = (long)(nq + 2 * nkv) * HD;
    const int q0 = s0 + qt * BQ + wave * 32;                  // first query of this wave (token index)
    const int kv_end = CAUSAL ? (s0 + (qt + 1) * BQ < s1 ? s0 + (qt + 1) * BQ : s1) : s1;
    const int nkt = (kv_end - s0 + BKV - 1) / BKV;
    const bf16_t *Kb = qkv + (long)(nq + g) * HD;
    const bf16_t *Vb = qkv + (long)(nq + nkv + g) * HD;

    // Q fragments (B operand): lane = query column, 8 consecutive d per k-step half
    bf16x8 qf[D::KST];
    {
        const int q = q0 + lrow;
        const bf16_t *qp = qkv + (long)q * ld + (long)h * HD + half * 8;
#pragma unroll
        for (int ks = 0; ks < D::KST; ++ks) {
            if (q < s1) qf[ks] = *(const bf16x8 *)(qp + ks * 16);
            else
#pragma unroll
                for (int i = 0; i < 8; ++i) qf[ks][i] = (bf16_t)0.f;
        }
    }

    Stager<64, false> sk[D::NKS];
    Stager<D::DB * 32, true> sv;
    auto load_tile = [&](int j) {
#pragma unroll
        for (int i = 0; i < D::NKS; ++i) sk[i].load(Kb, ld, s0 + j * BKV, kv_end, i * 64, HD, tid);
        sv.load(Vb, ld, 0, HD, s0 + j * BKV, kv_end, tid);
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int i = 0; i < D::NKS; ++i) sk[i].store(Ks + (buf * D::NKS + i) * 64 * 64, tid);
        sv.store(Vt + buf * D::DB * 32 * 64, tid);
    };

    f32x16 oacc[D::DB];
#pragma unroll
    for (int i = 0; i < D::DB; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[i][r] = 0.f;
    float m = -INFINITY, l = 0.f;

    load_tile(0);
    store_tile(0);
    __syncthreads();

    for (int j = 0; j < nkt; ++j) {
        const int cur = j & 1;
        if (j + 1 < nkt) load_tile(j + 1);
        const bf16_t *kt = Ks + cur * D::NKS * 64 * 64;
        const bf16_t *vt = Vt + cur * D::DB * 32 * 64;

        // S^T[key][q] for the 64 keys of the tile: two 32-key blocks
        f32x16 st[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) st[kb][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < D::KST; ++ks) {
                const bf16x8 kf = *(const bf16x8 *)(kt + (ks / 4) * 64 * 64 + lds_off(kb * 32 + lrow, (ks % 4) * 2 + half));
                st[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], st[kb], 0, 0, 0);
            }
        }
        // scale, mask, row maximum (one query per lane; the other half-wave holds the other keys)
        const int q = q0 + lrow;
        const int key0 = s0 + j * BKV + 4 * half;
        float p[2][16];
        float mx = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = key0 + kb * 32 + 8 * (r >> 2) + (r & 3);
                const bool ok = key < kv_end && (!CAUSAL || key <= q);
                const float s = ok ? st[kb][r] * scale_log2e : -INFINITY;
                p[kb][r] = s;
                mx = fmaxf(mx, s);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m, mx);
        const float m_use = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m - m_use);          // m = -inf on the first tile -> 0
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                p[kb][r] = __builtin_amdgcn_exp2f(p[kb][r] - m_use);
                psum += p[kb][r];
            }
        l = l * alpha + psum;
        m = m_new;
#pragma unroll
        for (int i = 0; i < D::DB; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[i][r] *= alpha;

        // O^T[d][q] += Vt[d][key] P^T[key][q]; k-slot s of half h is key 16t + 4h + s (s < 4),
        // 16t + 8 + 4h + (s - 4) (s >= 4): exactly accumulator registers 8t .. 8t+7
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const bf16x8 pf = pack8(&p[kb][8 * t]);
#pragma unroll
                for (int db = 0; db < D::DB; ++db) {
                    const int row = db * 32 + lrow;
                    const uint2 lo = *(const uint2 *)(vt + lds_off(row, kb * 4 + 2 * t) + 4 * half);
                    const uint2 hi = *(const uint2 *)(vt + lds_off(row, kb * 4 + 2 * t + 1) + 4 * half);
                    union { uint4 u; bf16x8 v; } vf;
                    vf.u = make_uint4(lo.x, lo.y, hi.x, hi.y);
                    oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.v, pf, oacc[db], 0, 0, 0);
                }
            }
        if (j + 1 < nkt) store_tile(cur ^ 1);
        __syncthreads();
    }

    l += __shfl_xor(l, 32, 64);
    const int q = q0 + lrow;
    if (q >= s1) return;
    const float inv = 1.f / l;
    bf16_t *op = o + (long)q * nq * HD + (long)h * HD;
#pragma unroll
    for (int db = 0; db < D::DB; ++db)
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
            const int d = db * 32 + 8 * rg + 4 * half;
            if (d < HD) {
                union { uint2 u; bf16_t v[4]; } w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w.v[e] = (bf16_t)(oacc[db][rg * 4 + e] * inv);
                *(uint2 *)(op + d) = w.u;
            }
        }
    if (half == 0) lse[(long)h * n + q] = (m + log2f(l)) * 0.6931471805599453f;
}

template <int HD>
ms_status launch_fwd(int causal, int nq, int nkv, int n, int n_seqs, int max_seqlen, const int *cu, const void *qkv,
                     void *o, float *lse, hipStream_t s) {
    using D = AttnDims<HD>;
    const size_t smem = (size_t)2 * (D::NKS * 64 * 64 + D::DB * 32 * 64) * sizeof(bf16_t);
    dim3 grid(ms_cdiv(max_seqlen, 128), nq, n_seqs);
    const float sc = 1.4426950408889634f / sqrtf((float)HD);
#define GO(C)                                                                                                   \
    do {                                                                                                        \
        static bool attr_set = false;                                                                           \
        if (!attr_set && smem > 48 * 1024) {                                                                    \
            MS_CHECK_HIP(hipFuncSetAttribute((const void *)attn_fwd_mfma_kernel<HD, C>,                         \
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));           \
            attr_set = true;                                                                                    \
        }                                                                                                       \
        attn_fwd_mfma_kernel<HD, C><<<grid, 256, smem, s>>>((const bf16_t *)qkv, (bf16_t *)o, lse, cu, n, nq, nkv, sc); \
    } while (0)
    if (causal) GO(true); else GO(false);
#undef GO
    MS_LAUNCH_CHECK();
    return MS_OK;
}

}  // namespace

bool attn_mfma_forward_supported(int hd) { return hd == 64 || hd == 80 || hd == 128; }
bool attn_mfma_backward_supported(int) { return false; }

ms_status attn_mfma_forward(int causal, int nq, int nkv, int hd, int n, int n_seqs, int max_seqlen, const int *cu,
                            const void *qkv, void *o, float *lse, hipStream_t s) {
    if (max_seqlen <= 0) return MS_OK;
    if (hd == 64) return launch_fwd<64>(causal, nq, nkv, n, n_seqs, max_seqlen, cu, qkv, o, lse, s);
    if (hd == 80) return launch_fwd<80>(causal, nq, nkv, n, n_seqs, max_seqlen, cu, qkv, o, lse, s);
    if (hd == 128) return launch_fwd<128>(causal, nq, nkv, n, n_seqs, max_seqlen, cu, qkv, o, lse, s);
    return ms_fail(MS_ERR_UNSUPPORTED, "attention: head_dim %d has no matrix-core kernel", hd);
}

size_t attn_mfma_backward_scratch_bytes(int, int, int, int) { return 0; }
ms_status attn_mfma_backward(int, int, int, int, int, int, int, const int *, const void *, const void *, const float *,
                             const void *, void *, void *, hipStream_t) {
    return ms_fail(MS_ERR_UNSUPPORTED, "attention backward: matrix-core path not built");
}
