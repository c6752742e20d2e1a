// Matrix-core variable-length attention for bf16 (head_dim 64, 80, 128), forward and backward.
//
// One workgroup (4 waves) owns 128 consecutive queries of one sequence and one query head; each
// wave owns 32 of them and keeps its Q fragments in registers.  Keys / values are visited 64 at a
// time through two LDS buffers filled by direct global -> LDS loads (no staging registers), both
// row-major [64 keys][head_dim] as 64-wide swizzled sub-tiles; the P V product, which contracts
// over keys, reads V through the transposing LDS load (ds_read_b64_tr_b16).
// Scores are computed transposed, S^T = K Q^T (v_mfma_f32_32x32x16_bf16): in the accumulator
// layout a lane then holds 32 keys of ONE query, so the online-softmax row maximum and sum are
// register reductions plus a single cross-half shuffle, the rescale factor is a per-lane scalar,
// and the probabilities are already laid out as the B operand of O^T += Vt P^T.
#include <type_traits>

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

// Workgroup -> (sequence, head, tile level).  Workgroups reach the 8 XCDs round-robin by blockIdx, and each XCD has an
// L2 of its own: XCD k runs the blocks with blockIdx % 8 == k, in blockIdx order.  The heads are divided into
// G = gcd(heads, 8) classes of hpc neighbouring heads (one GQA group or a part of one); a class belongs to S = 8 / G
// XCDs, which stripe its tile levels between them in serpentine order, so that under a causal mask every stripe weighs
// the same whatever the sequence lengths are.  Level 0 is the heaviest tile (the last query tile, the first key
// block).  Within an XCD the order is chunks of kAttnChunk levels, heaviest chunk first, and within a chunk sequence,
// head of the class, level: the workgroups that run at one time are neighbouring levels of a few (sequence, head)
// pairs and read the same K/V (or Q/dO) rows, which then come from L2.
constexpr int kAttnChunk = 8;
struct AttnGrid { int S, hpc, M; long blocks; };
__host__ __device__ inline AttnGrid attn_grid(int heads, int n_seqs, int nlevel_max) {
    const int low = heads & -heads, G = low < 8 ? low : 8;          // gcd(heads, 8)
    AttnGrid a;
    a.S = 8 / G; a.hpc = heads / G;
    a.M = ((nlevel_max + a.S - 1) / a.S + kAttnChunk - 1) / kAttnChunk * kAttnChunk;   // levels per stripe, whole chunks
    a.blocks = 8L * a.M * a.hpc * n_seqs;
    return a;
}
struct AttnSlot { int b, h, level; };
__device__ inline AttnSlot attn_slot(unsigned bid, int heads, int n_seqs, int nlevel_max) {
    const AttnGrid a = attn_grid(heads, n_seqs, nlevel_max);
    const int k = bid & 7, j = bid >> 3;
    const int cls = k / a.S, r = k % a.S;
    const int li = j % kAttnChunk, hc = (j / kAttnChunk) % a.hpc;
    const int b = (j / (kAttnChunk * a.hpc)) % n_seqs, chunk = j / (kAttnChunk * a.hpc * n_seqs);
    const int m = chunk * kAttnChunk + li, rr = (r + b + hc) % a.S;
    return {b, cls * a.hpc + hc, m * a.S + ((m & 1) ? a.S - 1 - rr : rr)};
}

template <int HD, bool CAUSAL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_fwd_mfma_kernel(const bf16_t *__restrict__ qkv, bf16_t *__restrict__ o,
                                                             float *__restrict__ lse, const int *__restrict__ cu, int n,
                                                             int nq, int nkv, int n_seqs, int ntile_max, float scale_log2e) {
    using D = AttnDims<HD>;
    constexpr int BQ = 128, BKV = 64, TS = D::NKS * 4096;
    // separate LDS objects per buffer: lets the compiler tell in-flight direct-to-LDS loads from reads
    __shared__ __align__(16) bf16_t K0[TS], K1[TS], V0[TS], V1[TS];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lrow = lane & 31, half = lane >> 5;
    const AttnSlot slot = attn_slot(blockIdx.x, nq, n_seqs, ntile_max);
    const int qt = ntile_max - 1 - slot.level, h = slot.h, b = slot.b;
    if (qt < 0) return;
    const int s0 = cu[b], s1 = cu[b + 1];
    if (qt * BQ >= s1 - s0) return;
    const int g = h / (nq / nkv);
    const long ld = (long)(nq + 2 * nkv) * HD;
    const int q0 = s0 + qt * BQ + wave * 32;
    const int kv_end = CAUSAL ? (s0 + (qt + 1) * BQ < s1 ? s0 + (qt + 1) * BQ : s1) : s1;
    const int nkt = (kv_end - s0 + BKV - 1) / BKV;
    const int kcol = (nq + g) * HD, vcol = (nq + nkv + g) * HD;
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(qkv, (long)n * ld * 2);

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
    // each wave issues a quarter of the 2 * 8 * NKS instructions that fill one K tile and one V tile
    // (waves 0 and 1 fill the K tile, waves 2 and 3 the V tile; the lane's part of the addresses is computed once)
    constexpr int PER = 4 * D::NKS;
    RowTileLane dl;
    dl.init(lane, (unsigned)(ld * 2));
    const bool fill_v = wave >= 2;
    const unsigned dcol = (unsigned)(fill_v ? vcol : kcol) * 2;
    auto issue = [&](int j, bf16_t *kt, bf16_t *vt) {
        const unsigned base = (unsigned)((long)(s0 + j * BKV) * ld * 2) + dcol;
        bf16_t *t = fill_v ? vt : kt;
#pragma unroll
        for (int i = 0; i < PER; ++i) rowtile_dma_lane<HD, 64>(rs, t, base, (unsigned)(ld * 2), (wave & 1) * PER + i, dl);
    };
    // The same loads in KST portions, placed between the MFMAs of the S product of the tile before: a direct-to-LDS
    // load occupies the wave's issue slot for tens of cycles, which the MFMAs already queued cover.  A tile past the
    // end is requested out of range (zeros that nobody reads), so the loop body has no branch.
    auto issue_part = [&](int ks, int j, bf16_t *kt, bf16_t *vt) __attribute__((always_inline)) {
        const unsigned base = (unsigned)((long)(s0 + j * BKV) * ld * 2) + dcol;
        const unsigned inv = j < nkt ? 0u : kOob;
        bf16_t *t = fill_v ? vt : kt;
#pragma unroll
        for (int i = ks * PER / D::KST; i < (ks + 1) * PER / D::KST; ++i)
            rowtile_dma_lane<HD, 64>(rs, t, base, (unsigned)(ld * 2), (wave & 1) * PER + i, dl, inv);
    };

    f32x16 oacc[D::DB];
#pragma unroll
    for (int i = 0; i < D::DB; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[i][r] = 0.f;
    float m = -INFINITY, l = 0.f;
    const int q = q0 + lrow;

    auto compute = [&](int j, const bf16_t *kt, const bf16_t *vt, bf16_t *kn, bf16_t *vn) {
        // S^T[key][q] for the 64 keys of the tile: two 32-key blocks (two independent accumulation chains); the
        // K fragments of k-step ks + 1 are read while the MFMAs of k-step ks run
        f32x16 st[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) st[kb][r] = 0.f;
        auto kfrag = [&](int ks, int kb) {
            return *(const bf16x8 *)(kt + (ks / 4) * 4096 + lds_off(kb * 32 + lrow, (ks % 4) * 2 + half));
        };
        bf16x8 kf[2][2];
        kf[0][0] = kfrag(0, 0);
        kf[0][1] = kfrag(0, 1);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
#pragma unroll
        for (int ks = 0; ks < D::KST; ++ks) {
            if (ks + 1 < D::KST) {
                kf[(ks + 1) & 1][0] = kfrag(ks + 1, 0);
                kf[(ks + 1) & 1][1] = kfrag(ks + 1, 1);
            }
            st[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks & 1][0], qf[ks], st[0], 0, 0, 0);
            st[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks & 1][1], qf[ks], st[1], 0, 0, 0);
            issue_part(ks, j + 1, kn, vn);
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x020, (PER + D::KST - 1) / D::KST, 0);
        }
        // mask (only tiles that touch the diagonal or the end of the sequence: wave-uniform test), row
        // maximum on the raw scores (one query per lane; the other half-wave holds the other keys),
        // then p = exp2(s * scale - m) with the scale folded into one fused multiply-add
        const int key0 = s0 + j * BKV + 4 * half;
        const bool need_mask = s0 + j * BKV + BKV > kv_end || (CAUSAL && s0 + j * BKV + BKV - 1 > q0);
        if (need_mask) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = key0 + kb * 32 + 8 * (r >> 2) + (r & 3);
                    const bool ok = key < kv_end && (!CAUSAL || key <= q);
                    st[kb][r] = ok ? st[kb][r] : -INFINITY;
                }
        }
        float mx = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, st[kb][r]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * scale_log2e;
        const float m_new = fmaxf(m, mx);
        const float m_use = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m - m_use);          // m = -inf on the first tile -> 0
        float p[2][16];
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                p[kb][r] = __builtin_amdgcn_exp2f(__builtin_fmaf(st[kb][r], scale_log2e, -m_use));
                psum += p[kb][r];
            }
        l = l * alpha + psum;
        m = m_new;
        if (__builtin_amdgcn_ballot_w64(alpha != 1.f)) {    // wave-uniform: skip the rescale once the maxima settle
#pragma unroll
            for (int i = 0; i < D::DB; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[i][r] *= alpha;
        }
        // O^T[d][q] += V^T[d][key] P^T[key][q]; k-slot s of half h is key 16t + 4h + s (s < 4),
        // 16t + 8 + 4h + (s - 4) (s >= 4): exactly accumulator registers 8t .. 8t+7.  V stays
        // row-major in LDS and is read through the transposing LDS load.
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const bf16x8 pf = pack8(&p[kb][8 * t]);
#pragma unroll
                for (int db = 0; db < D::DB; ++db)
                    oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rowtile_tr_frag(vt, kb * 32 + 16 * t, db * 32, lane), pf,
                                                                         oacc[db], 0, 0, 0);
            }
    };

    issue(0, K0, V0);
    dma_publish_barrier();
    for (int j = 0; j < nkt; j += 2) {
        compute(j, K0, V0, K1, V1);
        dma_publish_barrier();
        if (j + 1 < nkt) compute(j + 1, K1, V1, K0, V0);
        dma_publish_barrier();
    }

    l += __shfl_xor(l, 32, 64);
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

// ===================================================================== backward
// Row terms of the softmax backward, one pair per (head, token): ld[h, t] = (lse[h, t] * log2(e), delta[h, t]) with
// delta = sum_d dO[t, h, d] O[t, h, d] (the row term of the softmax Jacobian).  Interleaved so that the 32 pairs of a
// 32-query tile are 256 contiguous bytes (one direct-to-LDS load in the dK/dV kernel).
__global__ __launch_bounds__(256) void attn_delta_kernel(const bf16_t *__restrict__ o, const bf16_t *__restrict__ d_o,
                                                          const float *__restrict__ lse, float2 *__restrict__ ld, int n, int nq,
                                                          int hd) {
    // 8 lanes per (token, head): consecutive lanes read consecutive 16-byte pieces, so a wave's load is one
    // contiguous run; the 8 partial sums meet through xor-shuffles
    const long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const long idx = gid >> 3;
    const int sub = (int)(gid & 7);
    const bool live = idx < (long)n * nq;
    float acc = 0.f;
    if (live) {
        const bf16_t *a = o + idx * hd, *b = d_o + idx * hd;
        for (int d = sub * 8; d < hd; d += 64) {
            const Vec16<bf16_t> x = ldv(a + d), y = ldv(b + d);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc += (float)x.v[e] * (float)y.v[e];
        }
    }
    acc += __shfl_xor(acc, 1, 64);
    acc += __shfl_xor(acc, 2, 64);
    acc += __shfl_xor(acc, 4, 64);
    if (live && sub == 0) {
        const long at = (long)(idx % nq) * n + idx / nq;
        ld[at] = make_float2(lse[at] * 1.4426950408889634f, acc);
    }
}

// dQ: same decomposition as the forward kernel (workgroup = 128 queries of one head, keys visited
// 64 at a time, K and V tiles loaded directly into LDS).  S^T = K Q^T and dP^T = V dO^T are
// accumulator tiles with one query per lane, so P = exp2(S^T c - lse[q]) and
// dS^T = P (dP^T - delta[q]) use per-lane scalars, and dS^T is the B operand of dQ^T += K^T dS^T
// with K^T read from the row-major K tile through the transposing LDS load.
template <int HD, bool CAUSAL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_bwd_dq_mfma_kernel(const bf16_t *__restrict__ qkv, const bf16_t *__restrict__ d_o,
                                                                const float2 *__restrict__ ld2,
                                                                bf16_t *__restrict__ dqkv, const int *__restrict__ cu, int n,
                                                                int nq, int nkv, int n_seqs, int ntile_max, float scale) {
    using D = AttnDims<HD>;
    constexpr int BQ = 128, BKV = 64, TS = D::NKS * 4096;
    __shared__ __align__(16) bf16_t K0[TS], K1[TS], V0[TS], V1[TS];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lrow = lane & 31, half = lane >> 5;
    const AttnSlot slot = attn_slot(blockIdx.x, nq, n_seqs, ntile_max);
    const int qt = ntile_max - 1 - slot.level, h = slot.h, b = slot.b;
    if (qt < 0) return;
    const int s0 = cu[b], s1 = cu[b + 1];
    if (qt * BQ >= s1 - s0) return;
    const int g = h / (nq / nkv);
    const long ld = (long)(nq + 2 * nkv) * HD;
    const int q0 = s0 + qt * BQ + wave * 32;
    const int kv_end = CAUSAL ? (s0 + (qt + 1) * BQ < s1 ? s0 + (qt + 1) * BQ : s1) : s1;
    const int nkt = (kv_end - s0 + BKV - 1) / BKV;
    const int kcol = (nq + g) * HD, vcol = (nq + nkv + g) * HD;
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(qkv, (long)n * ld * 2);
    const float c = scale * 1.4426950408889634f;

    const int q = q0 + lrow;
    const bool qok = q < s1;
    bf16x8 qf[D::KST], dof[D::KST];
    {
        const bf16_t *qp = qkv + (long)q * ld + (long)h * HD + half * 8;
        const bf16_t *dp = d_o + (long)q * nq * HD + (long)h * HD + half * 8;
#pragma unroll
        for (int ks = 0; ks < D::KST; ++ks) {
            if (qok) {
                qf[ks] = *(const bf16x8 *)(qp + ks * 16);
                dof[ks] = *(const bf16x8 *)(dp + ks * 16);
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) { qf[ks][i] = (bf16_t)0.f; dof[ks][i] = (bf16_t)0.f; }
            }
        }
    }
    const float2 row = qok ? ld2[(long)h * n + q] : make_float2(0.f, 0.f);   // (lse * log2(e), delta)
    const float lse2 = row.x, dlt = row.y;

    // (waves 0 and 1 fill the K tile, waves 2 and 3 the V tile; the lane's part of the addresses is computed once)
    constexpr int PER = 4 * D::NKS;
    RowTileLane dl;
    dl.init(lane, (unsigned)(ld * 2));
    const bool fill_v = wave >= 2;
    const unsigned dcol = (unsigned)(fill_v ? vcol : kcol) * 2;
    auto issue = [&](int j, bf16_t *kt, bf16_t *vt) {
        const unsigned base = (unsigned)((long)(s0 + j * BKV) * ld * 2) + dcol;
        bf16_t *t = fill_v ? vt : kt;
#pragma unroll
        for (int i = 0; i < PER; ++i) rowtile_dma_lane<HD, 64>(rs, t, base, (unsigned)(ld * 2), (wave & 1) * PER + i, dl);
    };
    // The same loads in KST portions, placed between the MFMAs of the S product of the tile before: a direct-to-LDS
    // load occupies the wave's issue slot for tens of cycles, which the MFMAs already queued cover.  A tile past the
    // end is requested out of range (zeros that nobody reads), so the loop body has no branch.
    auto issue_part = [&](int ks, int j, bf16_t *kt, bf16_t *vt) __attribute__((always_inline)) {
        const unsigned base = (unsigned)((long)(s0 + j * BKV) * ld * 2) + dcol;
        const unsigned inv = j < nkt ? 0u : kOob;
        bf16_t *t = fill_v ? vt : kt;
#pragma unroll
        for (int i = ks * PER / D::KST; i < (ks + 1) * PER / D::KST; ++i)
            rowtile_dma_lane<HD, 64>(rs, t, base, (unsigned)(ld * 2), (wave & 1) * PER + i, dl, inv);
    };

    f32x16 dq[D::DB];
#pragma unroll
    for (int i = 0; i < D::DB; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) dq[i][r] = 0.f;

    auto compute = [&](int j, const bf16_t *kt, const bf16_t *vt, bf16_t *kn, bf16_t *vn) {
        const int key0 = s0 + j * BKV + 4 * half;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            f32x16 st, dp;
#pragma unroll
            for (int r = 0; r < 16; ++r) { st[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
            for (int ks = 0; ks < D::KST; ++ks) {
                const int off = (ks / 4) * 4096 + lds_off(kb * 32 + lrow, (ks % 4) * 2 + half);
                st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8 *)(kt + off), qf[ks], st, 0, 0, 0);
                dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8 *)(vt + off), dof[ks], dp, 0, 0, 0);
                if (kb == 0) issue_part(ks, j + 1, kn, vn);
            }
            // rows past the end of the sequence have zero Q, dO, lse and delta (dS = 0 there without a mask)
            const int kfirst = s0 + j * BKV + kb * 32;
            const bool need_mask = kfirst + 32 > kv_end || (CAUSAL && kfirst + 31 > q0);
            float ds[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float p = __builtin_amdgcn_exp2f(__builtin_fmaf(st[r], c, -lse2));
                if (need_mask) {
                    const int key = key0 + kb * 32 + 8 * (r >> 2) + (r & 3);
                    p = (key < kv_end && (!CAUSAL || key <= q)) ? p : 0.f;
                }
                ds[r] = p * (dp[r] - dlt);
            }
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const bf16x8 dsf = pack8(&ds[8 * t]);
#pragma unroll
                for (int db = 0; db < D::DB; ++db)
                    dq[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rowtile_tr_frag(kt, kb * 32 + 16 * t, db * 32, lane), dsf,
                                                                       dq[db], 0, 0, 0);
            }
        }
    };

    issue(0, K0, V0);
    dma_publish_barrier();
    for (int j = 0; j < nkt; j += 2) {
        compute(j, K0, V0, K1, V1);
        dma_publish_barrier();
        if (j + 1 < nkt) compute(j + 1, K1, V1, K0, V0);
        dma_publish_barrier();
    }
    if (!qok) return;
    bf16_t *op = dqkv + (long)q * ld + (long)h * HD;
#pragma unroll
    for (int db = 0; db < D::DB; ++db)
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
            const int d = db * 32 + 8 * rg + 4 * half;
            if (d < HD) {
                union { uint2 u; bf16_t v[4]; } w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w.v[e] = (bf16_t)(dq[db][rg * 4 + e] * scale);
                *(uint2 *)(op + d) = w.u;
            }
        }
}

// dK, dV: workgroup = NW waves with 32 keys each of one KV head (K fragments in registers; V fragments in registers
// as well or as a tile in LDS); it walks the query heads of the group and their query tiles, 32 rows at a time.  S = Q K^T and dP = dO V^T
// are accumulator tiles with one KEY per lane and queries down the registers, which is the A-operand layout of
// dV += P^T dO and dK += dS^T Q; their B operands (dO and Q with queries as the contraction index) come from the
// row-major tiles through the transposing LDS load.  256 registers per wave: two waves per SIMD (two 4-wave workgroups
// per CU, which drift apart so that one's exponentials overlap the other's MFMAs, or one 8-wave workgroup).
//
// The query tiles (Q rows, dO rows and the 32 (lse, delta) pairs, everything by direct-to-LDS loads: no load of the
// loop goes through registers, so no wave waits on a load in the middle of a tile) go through a ring of NST LDS stages,
// requested NST - 1 tiles ahead.  One barrier per tile does both jobs: before it each wave waits until ITS loads of
// the tile have landed (s_waitcnt vmcnt(k): loads complete in order and exactly k younger ones, those of the next
// NST - 2 tiles, may still be in flight; tiles past the end are requested as out-of-range loads so that the count is
// the same in every iteration), after it all waves have finished the previous tile, whose stage is then handed to the
// tile NST - 1 ahead.  Measured on MI355X (c5 student / c4 encoder shapes, in the step): NW = 4, NST = 2 (two
// independent workgroups per CU, 66 KB of LDS each) 28.0 / 57.2 ms per step; NW = 8 with NST = 3 or 4 (one workgroup
// per CU, all eight waves in lockstep) 28.8 / 58.0 and 29.1 / 67.5: deeper prefetch buys nothing, the kernel is not
// waiting for memory but for its own MFMA -> exponentials -> MFMA chain, which two independent workgroups overlap
// better than one.  (NW = 4 with NST = 3 needs 80.75 KB of LDS for head_dim 128, 768 bytes too many for two per CU.)
// !SPLIT: the sums over the query group stay in registers, no atomics.
// SPLIT: one workgroup per query head of the group instead of one per K/V head (4x the workgroups and a 4x
// shorter longest one under grouped-query attention); partial dK/dV are then summed with fp32 atomics
// into dkv_acc [n][2][nkv * HD], which attn_dkv_store_kernel rounds into dqkv afterwards.
template <int N> __device__ __forceinline__ void wait_vmcnt_lgkm0() {
    // gfx9 encoding: vmcnt = bits 3:0 and 15:14, expcnt = bits 6:4 (7: no wait), lgkmcnt = bits 11:8 (0)
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4));
}
// barrier between waves that exchange data through LDS, without the full memory fence of __syncthreads (which would
// wait for every outstanding load): the wavefront-scope fences only keep the compiler from moving LDS accesses across
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int HD, bool CAUSAL, bool SPLIT, int NW, int NST>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_bwd_dkv_mfma_kernel(
    const bf16_t *__restrict__ qkv, const bf16_t *__restrict__ d_o, const float2 *__restrict__ ld2,
    bf16_t *__restrict__ dqkv, float *__restrict__ dkv_acc, const int *__restrict__ cu, int n, int nq, int nkv, int n_seqs,
    int nblk_max, float scale) {
    using D = AttnDims<HD>;
    static_assert(NST >= 2 && NST <= 4 && (NW == 4 || NW == 8), "ring of 2..4 stages, 4 or 8 waves");
    constexpr int BK_ = 32 * NW, BQ = 32, QS = D::NKS * 2048, VS = D::NKS * 4096;
    constexpr int Q2 = NST > 2 ? QS : 8, Q3 = NST > 3 ? QS : 8;        // stages beyond NST are not used
    // separate LDS objects per stage: lets the compiler tell the stage being filled from the stage being read
    __shared__ __align__(16) bf16_t Qa[QS], Qb[QS], Qc[Q2], Qd[Q3], Oa[QS], Ob[QS], Oc[Q2], Od[Q3];
    __shared__ __align__(16) bf16_t Vs[(BK_ / 64) * VS];
    __shared__ __align__(16) float Fa[64], Fb[64], Fc[64], Fd[64];     // per query row of the tile: (lse * log2(e), delta)
    bf16_t *const Qst[4] = {Qa, Qb, Qc, Qd}, *const Ost[4] = {Oa, Ob, Oc, Od};
    float *const Fst[4] = {Fa, Fb, Fc, Fd};

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lrow = lane & 31, half = lane >> 5;
    // level = key block: the earliest key blocks meet the most query tiles under a causal mask
    const int grp = nq / nkv;
    const AttnSlot slot = attn_slot(blockIdx.x, SPLIT ? nq : nkv, n_seqs, nblk_max);
    const int hsub = SPLIT ? slot.h % grp : 0, g = SPLIT ? slot.h / grp : slot.h, b = slot.b;
    if (slot.level >= nblk_max) return;
    const int s0 = cu[b], s1 = cu[b + 1];
    const int kblk = slot.level * BK_;                      // first key of the workgroup, relative to s0
    if (kblk >= s1 - s0) return;
    const long ld = (long)(nq + 2 * nkv) * HD, ldo = (long)nq * HD;
    const int kw0 = s0 + kblk + wave * 32;                  // first key of the wave
    const int key = kw0 + lrow;                             // this lane's key (token index)
    const bool kok = key < s1;
    const float c = scale * 1.4426950408889634f;
    const __amdgpu_buffer_rsrc_t rq = make_rsrc(qkv, (long)n * ld * 2), ro = make_rsrc(d_o, (long)n * ldo * 2);
    const __amdgpu_buffer_rsrc_t rf = make_rsrc(ld2, (long)nq * n * 8);

    // the V tile (64-key row tiles): keys past the end of the sequence hold the next sequence's rows or zeros, which
    // only ever meet p = 0.  (Each wave only reads the rows of its own 32 keys; keeping them in registers like the K
    // fragments was measured: it spills.)
    {
        constexpr int PER = (BK_ / 64) * 8 * D::NKS / NW;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int idx = wave * PER + i, t = idx / (8 * D::NKS);
            rowtile_dma<HD>(rq, Vs + t * VS, s0 + kblk + t * 64, ld, (nq + nkv + g) * HD, idx % (8 * D::NKS), lane);
        }
    }
    bf16x8 kf[D::KST];
    {
        const bf16_t *kp = qkv + (long)key * ld + (long)(nq + g) * HD + half * 8;
#pragma unroll
        for (int ks = 0; ks < D::KST; ++ks) {
            if (kok) kf[ks] = *(const bf16x8 *)(kp + ks * 16);
            else
#pragma unroll
                for (int i = 0; i < 8; ++i) kf[ks][i] = (bf16_t)0.f;
        }
    }
    // query tiles that see this key block.  They are walked from the last one down: the workgroups of a (sequence, head)
    // that run at the same time on an XCD (neighbouring key blocks) then read the same Q / dO rows at the same time, one
    // fetch into L2 serving all of them, whereas walks that start at each block's own first tile are staggered.
    const int qt_first = CAUSAL ? kblk / BQ : 0;
    const int nqt = (s1 - s0 + BQ - 1) / BQ - qt_first;
    const int niter = SPLIT ? nqt : nqt * grp;

    // Requests tile `it` (out of range: zeros that nobody reads).  Per wave: NKS loads of Q / dO rows, wave 0 one more
    // for the 32 (lse, delta) pairs = 64 consecutive floats.
    // The first half of the waves fills the Q tile, the second half the dO tile; the lane's part of the addresses
    // is computed once.
    constexpr int PERQ = 8 * D::NKS / NW;
    static_assert((4 * D::NKS) % PERQ == 0, "a wave fills rows of one tile only");
    const bool fill_o = wave * PERQ >= 4 * D::NKS;
    const unsigned ldw2 = (unsigned)((fill_o ? ldo : ld) * 2);
    const __amdgpu_buffer_rsrc_t rw = fill_o ? ro : rq;
    RowTileLane dl;
    dl.init(lane, ldw2);
    auto issue = [&](int it, bf16_t *qt_, bf16_t *ot_, float *f) __attribute__((always_inline)) {
        const unsigned inv = it < niter ? 0u : kOob;
        const int itc = it < niter ? it : 0;
        const int h = g * grp + (SPLIT ? hsub : itc / nqt);
        const int qs = s0 + (qt_first + nqt - 1 - itc % nqt) * BQ;
        const unsigned base = (unsigned)qs * ldw2 + (unsigned)(h * HD) * 2;
        bf16_t *t = fill_o ? ot_ : qt_;
#pragma unroll
        for (int i = 0; i < PERQ; ++i) rowtile_dma_lane<HD, 32>(rw, t, base, ldw2, (wave * PERQ + i) % (4 * D::NKS), dl, inv);
        if (wave == 0)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rf, (lds_void *)f, 4, (unsigned)((((long)h * n + qs) * 2 + lane) * 4) | inv, 0, 0, 0);
    };

    const bf16_t *vrow = Vs + (wave >> 1) * VS;             // the 64-key row tile holding this wave's keys
    const int vr = (wave & 1) * 32 + lrow;
    // One pass over the query tiles accumulates dV (WHICH = 0: needs S only), dK (1: needs S and dP) or both
    // (2).  Both accumulator sets are kept (one pass) for every head_dim.  At head_dim 128 that is 128 accumulator
    // registers and the kernel spills about 22 of its 256 registers, which was measured against the alternative that
    // fits: two passes (0 then 1) with one accumulator set, one extra S product and a second round of exponentials per
    // tile.  One pass is 11-13 % faster at the c5 / c2 student shapes (3.62 -> 3.21 ms, 0.51 -> 0.465 ms per layer).
    // The two-pass code path stays selectable here.
    constexpr bool ONE_PASS = true;
    f32x16 acc[D::DB], acc2[ONE_PASS ? D::DB : 1];          // acc2: dV when both are accumulated (acc is dK then)
    auto compute = [&](auto which, int it, const bf16_t *qt_, const bf16_t *ot_, const float *f) __attribute__((always_inline)) {
        constexpr int WHICH = decltype(which)::value;
        constexpr bool DK = WHICH >= 1, BOTH = WHICH == 2;
        const int qs = s0 + (qt_first + nqt - 1 - it % nqt) * BQ;
        if (CAUSAL && qs + BQ - 1 < kw0) return;            // every query of the tile precedes every key of the wave
        f32x16 st, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) { st[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < D::KST; ++ks) {
            const int off = lds_off(lrow, (ks % 4) * 2 + half);
            st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8 *)(qt_ + (ks / 4) * 2048 + off), kf[ks], st, 0, 0, 0);
            if constexpr (DK) {
                const bf16x8 vfr = *(const bf16x8 *)(vrow + (ks / 4) * 4096 + lds_off(vr, (ks % 4) * 2 + half));
                dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8 *)(ot_ + (ks / 4) * 2048 + off), vfr, dp, 0, 0, 0);
            }
        }
        // accumulator rows are queries 8*(r/4) + 4*half + r%4, the column is this lane's key; keys and queries past
        // the end of the sequence are masked (their rows hold the next sequence's data or zeros)
        const bool need_mask = kw0 + 31 >= s1 || qs + BQ > s1 || (CAUSAL && kw0 + 31 > qs);
        // 16 queries (one MFMA k-step of the second product) at a time, to keep few values live
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            float w[8], w2[BOTH ? 8 : 1];
#pragma unroll
            for (int rg = 0; rg < 2; ++rg) {
                const int qr = 16 * t + 8 * rg + 4 * half;
                const float4 fa = *(const float4 *)(f + 2 * qr), fb = *(const float4 *)(f + 2 * qr + 4);
                const float lv[4] = {fa.x, fa.z, fb.x, fb.z}, dvv[4] = {fa.y, fa.w, fb.y, fb.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int r = rg * 4 + e;
                    float pe = __builtin_amdgcn_exp2f(__builtin_fmaf(st[8 * t + r], c, -lv[e]));
                    if (need_mask) {
                        const int qq = qs + qr + e;
                        pe = (kok && qq < s1 && (!CAUSAL || key <= qq)) ? pe : 0.f;
                    }
                    w[r] = DK ? pe * (dp[8 * t + r] - dvv[e]) : pe;
                    if constexpr (BOTH) w2[r] = pe;
                }
            }
            const bf16x8 wf = pack8(w);
            const bf16_t *bt = DK ? qt_ : ot_;              // dK += dS^T Q, dV += P^T dO
#pragma unroll
            for (int db = 0; db < D::DB; ++db)
                acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, rowtile_tr_frag<2048>(bt, 16 * t, db * 32, lane), acc[db], 0, 0, 0);
            if constexpr (BOTH) {
                const bf16x8 pf = pack8(w2);
#pragma unroll
                for (int db = 0; db < D::DB; ++db)
                    acc2[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pf, rowtile_tr_frag<2048>(ot_, 16 * t, db * 32, lane), acc2[db], 0, 0, 0);
            }
        }
    };
    // accumulators: row = key wave*32 + 8*(r/4) + 4*half + r%4, column d = db*32 + lrow
    auto store = [&](const f32x16 *acc, int col0, float mul) __attribute__((always_inline)) {
#pragma unroll
        for (int db = 0; db < D::DB; ++db) {
            const int d = db * 32 + lrow;
            if (d >= HD) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int kk = s0 + kblk + wave * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
                if (kk >= s1) continue;
                if constexpr (SPLIT) unsafeAtomicAdd(dkv_acc + (long)kk * (2 * nkv * HD) + col0 - nq * HD + d, acc[db][r] * mul);
                else dqkv[(long)kk * ld + col0 + d] = (bf16_t)(acc[db][r] * mul);
            }
        }
    };
    // one tile of the ring: stage S holds tile `it`; the stage of tile it - 1 receives tile it + NST - 1
    auto ring_step = [&](auto which, int it, const bf16_t *q_cur, const bf16_t *o_cur, const float *f_cur, bf16_t *q_nxt,
                         bf16_t *o_nxt, float *f_nxt) __attribute__((always_inline)) {
        if (it >= niter) return;                            // workgroup-uniform
        // own loads of tile `it` have landed; the younger ones (tiles it+1 .. it+NST-2) may still be in flight
        if (wave == 0) wait_vmcnt_lgkm0<(NST - 2) * (PERQ + 1)>();
        else wait_vmcnt_lgkm0<(NST - 2) * PERQ>();
        lds_barrier();
        issue(it + NST - 1, q_nxt, o_nxt, f_nxt);
        compute(which, it, q_cur, o_cur, f_cur);
    };
    auto pass = [&](auto which) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < D::DB; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                acc[i][r] = 0.f;
                if constexpr (ONE_PASS) acc2[i][r] = 0.f;
            }
#pragma unroll
        for (int k = 0; k < NST - 1; ++k) issue(k, Qst[k], Ost[k], Fst[k]);
        for (int it = 0; it < niter; it += NST) {
#pragma unroll
            for (int k = 0; k < NST; ++k) {
                constexpr int P = NST - 1;                  // stage k holds tile it + k; stage k - 1 (mod NST) is free
                ring_step(which, it + k, Qst[k], Ost[k], Fst[k], Qst[(k + P) % NST], Ost[(k + P) % NST], Fst[(k + P) % NST]);
            }
        }
        // everything still in flight (tiles past the end: zeros) lands, and every wave is done reading, before the
        // stages are reused by the next pass or the workgroup's LDS is released
        __syncthreads();
    };
    if constexpr (ONE_PASS) {
        pass(std::integral_constant<int, 2>{});
        store(acc2, (nq + nkv + g) * HD, 1.f);
        store(acc, (nq + g) * HD, scale);
    } else {
        pass(std::integral_constant<int, 0>{});
        store(acc, (nq + nkv + g) * HD, 1.f);
        pass(std::integral_constant<int, 1>{});
        store(acc, (nq + g) * HD, scale);
    }
}

// dqkv[:, K and V columns] = bf16(dkv_acc); w = 2 * nkv * HD fp32 per token, 4 per thread
__global__ __launch_bounds__(256) void attn_dkv_store_kernel(const float *__restrict__ acc, bf16_t *__restrict__ dqkv, long n, int w,
                                                             long ld, int col0) {
    const long i = ((long)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i >= n * w) return;
    const long t = i / w;
    const int c = (int)(i % w);
    const float4 v = *(const float4 *)(acc + i);
    bf16_t *dst = dqkv + t * ld + col0 + c;
    union { bf16_t h[4]; uint2 u; } o;
    o.h[0] = (bf16_t)v.x; o.h[1] = (bf16_t)v.y; o.h[2] = (bf16_t)v.z; o.h[3] = (bf16_t)v.w;
    *(uint2 *)dst = o.u;
}

template <int HD>
ms_status launch_fwd(int causal, int nq, int nkv, int n, int n_seqs, int max_seqlen, const int *cu, const void *qkv,
                     void *o, float *lse, hipStream_t s) {
    const int ntile_max = ms_cdiv(max_seqlen, 128);
    const long blocks = attn_grid(nq, n_seqs, ntile_max).blocks;
    if (blocks > 0x7fffffffL || !ms_attn_offsets_fit(n, nq, nkv, HD))
        return ms_fail(MS_ERR_UNSUPPORTED, "attention: batch too large for 32-bit tile offsets");
    const float sc = 1.4426950408889634f / sqrtf((float)HD);
    if (causal) attn_fwd_mfma_kernel<HD, true><<<(unsigned)blocks, 256, 0, s>>>((const bf16_t *)qkv, (bf16_t *)o, lse, cu, n, nq, nkv, n_seqs, ntile_max, sc);
    else attn_fwd_mfma_kernel<HD, false><<<(unsigned)blocks, 256, 0, s>>>((const bf16_t *)qkv, (bf16_t *)o, lse, cu, n, nq, nkv, n_seqs, ntile_max, sc);
    MS_LAUNCH_CHECK();
    return MS_OK;
}

template <int HD>
ms_status launch_bwd(int causal, int nq, int nkv, int n, int n_seqs, int max_seqlen, const int *cu, const void *qkv,
                     const void *o, const float *lse, const void *d_o, void *dqkv, void *scratch, hipStream_t s) {
    const float scale = 1.f / sqrtf((float)HD);
    const int ntile_max = ms_cdiv(max_seqlen, 128);
    const long blocks = attn_grid(nq, n_seqs, ntile_max).blocks;
    // grouped-query attention: split the group's query heads over workgroups (see the kernel)
    const bool split = nq / nkv > 1;
    const long blocks_dkv = attn_grid(split ? nq : nkv, n_seqs, ntile_max).blocks;     // 128 keys each, like the query tiles
    if (blocks > 0x7fffffffL || blocks_dkv > 0x7fffffffL || !ms_attn_offsets_fit(n, nq, nkv, HD))
        return ms_fail(MS_ERR_UNSUPPORTED, "attention: batch too large for 32-bit tile offsets");
    const unsigned grid_dkv = (unsigned)blocks_dkv;
    float2 *ld2 = (float2 *)scratch;                       // [nq][n] pairs (lse * log2(e), delta)
    attn_delta_kernel<<<ms_cdiv((long)n * nq * 8, 256), 256, 0, s>>>((const bf16_t *)o, (const bf16_t *)d_o, lse, ld2, n, nq, HD);
    MS_LAUNCH_CHECK();
    float *dkv_acc = (float *)((char *)scratch + ms_align_up((size_t)nq * n * sizeof(float2)));
    const int w = 2 * nkv * HD;
    if (split) MS_TRY(launch_fill_f32(dkv_acc, (long)n * w, 0.f, s));
#define GO(C)                                                                                                          \
    do {                                                                                                               \
        attn_bwd_dq_mfma_kernel<HD, C><<<(unsigned)blocks, 256, 0, s>>>((const bf16_t *)qkv, (const bf16_t *)d_o, ld2, \
                                                                        (bf16_t *)dqkv, cu, n, nq, nkv, n_seqs,        \
                                                                        ntile_max, scale);                             \
        MS_LAUNCH_CHECK();                                                                                             \
        if (split)                                                                                                     \
            attn_bwd_dkv_mfma_kernel<HD, C, true, 4, 2><<<grid_dkv, 256, 0, s>>>((const bf16_t *)qkv, (const bf16_t *)d_o, \
                                                                                 ld2, (bf16_t *)dqkv, dkv_acc, cu, n,  \
                                                                                 nq, nkv, n_seqs, ntile_max, scale);   \
        else                                                                                                           \
            attn_bwd_dkv_mfma_kernel<HD, C, false, 4, 2><<<grid_dkv, 256, 0, s>>>((const bf16_t *)qkv, (const bf16_t *)d_o, \
                                                                                  ld2, (bf16_t *)dqkv, dkv_acc, cu, n, \
                                                                                  nq, nkv, n_seqs, ntile_max, scale);  \
    } while (0)
    if (causal) GO(true); else GO(false);
#undef GO
    MS_LAUNCH_CHECK();
    if (split) {
        attn_dkv_store_kernel<<<ms_cdiv((long)n * w / 4, 256), 256, 0, s>>>(dkv_acc, (bf16_t *)dqkv, n, w, (long)(nq + 2 * nkv) * HD,
                                                                          nq * HD);
        MS_LAUNCH_CHECK();
    }
    return MS_OK;
}

}  // namespace

bool attn_mfma_forward_supported(int hd) { return hd == 64 || hd == 80 || hd == 128; }
bool attn_mfma_backward_supported(int hd) { return hd == 64 || hd == 80 || hd == 128; }

ms_status attn_mfma_forward(int causal, int nq, int nkv, int hd, int n, int n_seqs, int max_seqlen, const int *cu,
                            const void *qkv, void *o, float *lse, hipStream_t s) {
    if (max_seqlen <= 0) return MS_OK;
    if (hd == 64) return launch_fwd<64>(causal, nq, nkv, n, n_seqs, max_seqlen, cu, qkv, o, lse, s);
    if (hd == 80) return launch_fwd<80>(causal, nq, nkv, n, n_seqs, max_seqlen, cu, qkv, o, lse, s);
    if (hd == 128) return launch_fwd<128>(causal, nq, nkv, n, n_seqs, max_seqlen, cu, qkv, o, lse, s);
    return ms_fail(MS_ERR_UNSUPPORTED, "attention: head_dim %d has no matrix-core kernel", hd);
}

size_t attn_mfma_backward_scratch_bytes(int nq, int nkv, int hd, int n) {
    // (lse, delta) pairs [nq][n], then (grouped-query attention only) the fp32 dK/dV accumulator [n][2][nkv * hd]
    return ms_align_up((size_t)nq * n * 2 * sizeof(float)) + (nq > nkv ? ms_align_up((size_t)n * 2 * nkv * hd * sizeof(float)) : 0);
}

ms_status attn_mfma_backward(int causal, int nq, int nkv, int hd, int n, int n_seqs, int max_seqlen, const int *cu,
                             const void *qkv, const void *o, const float *lse, const void *d_o, void *dqkv,
                             void *scratch, hipStream_t s) {
    if (max_seqlen <= 0) return MS_OK;
    if (hd == 64) return launch_bwd<64>(causal, nq, nkv, n, n_seqs, max_seqlen, cu, qkv, o, lse, d_o, dqkv, scratch, s);
    if (hd == 80) return launch_bwd<80>(causal, nq, nkv, n, n_seqs, max_seqlen, cu, qkv, o, lse, d_o, dqkv, scratch, s);
    if (hd == 128) return launch_bwd<128>(causal, nq, nkv, n, n_seqs, max_seqlen, cu, qkv, o, lse, d_o, dqkv, scratch, s);
    return ms_fail(MS_ERR_UNSUPPORTED, "attention backward: head_dim %d has no matrix-core kernel", hd);
}
