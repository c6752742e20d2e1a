// GEMM kernels of the section path.
//
// bf16: C = alpha * A(m,k) B(n,k) on the CDNA4 matrix cores (v_mfma_f32_32x32x16_bf16).
//   * workgroup = 256 threads = 4 waves in a 2x2 grid, workgroup tile BM x BN x 64;
//   * both operands are staged global -> registers -> LDS with a one-tile register prefetch and
//     two LDS buffers, so one barrier per K tile is enough;
//   * LDS rows are 64 bf16 (128 B) = eight 16-byte chunks; chunk c of row r is stored at chunk
//     c ^ ((r ^ (r >> 3)) & 7), which keeps the fragment reads (32 consecutive rows, one chunk)
//     and the transposed staging writes (rows 8 apart) off each other's banks;
//   * an operand stored K-major ("transposed": weight gradients, input gradients) is
//     transposed in registers while it is staged: a thread loads an 8(k) x 8(m) block as eight
//     16-byte rows and writes eight 16-byte K-contiguous rows, so the MFMA loop is the same for
//     all four layouts;
//   * workgroup ids are remapped so that the ids one XCD receives (id mod 8) are neighbours in
//     tile space and share operand panels in that XCD's L2.
// fp32: a plain LDS-tiled FMA kernel (correctness path of the fp32 workload).
#include "common.h"
#include "launch.h"
#include "mfma_tiles.h"

namespace {

struct GemmParams {
    const void *A, *B;
    void *C;
    const void *bias, *residual;
    long lda, ldb, ldc, ldr;
    int M, N, K;
    int tiles_m, tiles_n;
    int k_tiles_per_split;  // in units of 64
    float alpha;
    int c_fp32, accumulate, atomic, res_fp32;
};

template <int BM, int BN, bool TA, bool TB>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmParams p) {
    constexpr int WTM = BM / 2, WTN = BN / 2, MI = WTM / 32, NI = WTN / 32;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    bf16_t *As = (bf16_t *)smem_raw;         // [2][BM*64]
    bf16_t *Bs = As + 2 * BM * BK;           // [2][BN*64]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // XCD-aware remap of the workgroup id, then grouped (8 tile rows) ordering
    int pid;
    {
        const int nb = gridDim.x, b = blockIdx.x;
        const int per = nb >> 3, rem = nb & 7, x = b & 7, q = b >> 3;
        pid = x * per + (x < rem ? x : rem) + q;
    }
    constexpr int GM = 8;
    const int group = pid / (GM * p.tiles_n);
    const int first_m = group * GM;
    const int gsize = (p.tiles_m - first_m) < GM ? (p.tiles_m - first_m) : GM;
    const int tm = first_m + (pid % (GM * p.tiles_n)) % gsize;
    const int tn = (pid % (GM * p.tiles_n)) / gsize;
    const int m0 = tm * BM, n0 = tn * BN;

    const int kt_begin = blockIdx.y * p.k_tiles_per_split;
    int kt_end = kt_begin + p.k_tiles_per_split;
    const int kt_total = (p.K + BK - 1) / BK;
    if (kt_end > kt_total) kt_end = kt_total;
    const int nk = kt_end - kt_begin;
    if (nk <= 0) return;
    const int k_end = p.K;

    const bf16_t *A = (const bf16_t *)p.A, *B = (const bf16_t *)p.B;
    Stager<BM, TA> sa;
    Stager<BN, TB> sb;

    f32x16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    sa.load(A, p.lda, m0, p.M, kt_begin * BK, k_end, tid);
    sb.load(B, p.ldb, n0, p.N, kt_begin * BK, k_end, tid);
    sa.store(As, tid);
    sb.store(Bs, tid);
    __syncthreads();

    const int frow = lane & 31, fhalf = lane >> 5;
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < nk) {
            sa.load(A, p.lda, m0, p.M, (kt_begin + kt + 1) * BK, k_end, tid);
            sb.load(B, p.ldb, n0, p.N, (kt_begin + kt + 1) * BK, k_end, tid);
        }
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8 af[MI], bfr[NI];
#pragma unroll
            for (int i = 0; i < MI; ++i) {
                const int r = i * 32 + frow;
                // the swizzle uses the row index inside the whole tile
                af[i] = *(const bf16x8 *)(As + cur * BM * BK + lds_off(wm * WTM + r, kk * 2 + fhalf));
            }
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                const int r = j * 32 + frow;
                bfr[j] = *(const bf16x8 *)(Bs + cur * BN * BK + lds_off(wn * WTN + r, kk * 2 + fhalf));
            }
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) {
            sa.store(As + (cur ^ 1) * BM * BK, tid);
            sb.store(Bs + (cur ^ 1) * BN * BK, tid);
        }
        __syncthreads();
    }

    // epilogue: acc[i][j][r] is C(row, col) with row = 8*(r/4) + 4*(lane/32) + r%4, col = lane%32
    const bf16_t *bias = (const bf16_t *)p.bias, *res = (const bf16_t *)p.residual;
    const float *res32 = (const float *)p.residual;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int col = n0 + wn * WTN + j * 32 + frow;
            if (col >= p.N) continue;
            const float bv = bias ? (float)bias[col] : 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm * WTM + i * 32 + 8 * (r >> 2) + 4 * fhalf + (r & 3);
                if (row >= p.M) continue;
                float v = acc[i][j][r] * p.alpha + bv;
                if (res) v += p.res_fp32 ? res32[(long)row * p.ldr + col] : (float)res[(long)row * p.ldr + col];
                if (p.c_fp32) {
                    float *c = (float *)p.C + (long)row * p.ldc + col;
                    if (p.atomic) unsafeAtomicAdd(c, v);
                    else if (p.accumulate) *c += v;
                    else *c = v;
                } else {
                    ((bf16_t *)p.C)[(long)row * p.ldc + col] = (bf16_t)v;
                }
            }
        }
}

// ------------------------------------------------------------------ fp32 reference-speed kernel
struct GemmF32Params {
    const float *A, *B;
    float *C;
    const float *bias, *residual;
    long sam, sak, sbn, sbk, ldc, ldr;
    int M, N, K;
    float alpha;
    int accumulate;
};

__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmF32Params p) {
    __shared__ float As[16][65], Bs[16][65];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < p.K; k0 += 16) {
        for (int i = threadIdx.x; i < 64 * 16; i += 256) {
            const int r = i >> 4, k = i & 15;
            As[k][r] = (m0 + r < p.M && k0 + k < p.K) ? p.A[(long)(m0 + r) * p.sam + (long)(k0 + k) * p.sak] : 0.f;
            Bs[k][r] = (n0 + r < p.N && k0 + k < p.K) ? p.B[(long)(n0 + r) * p.sbn + (long)(k0 + k) * p.sbk] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[k][ty + 16 * i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Bs[k][tx + 16 * j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int row = m0 + ty + 16 * i, col = n0 + tx + 16 * j;
            if (row >= p.M || col >= p.N) continue;
            float v = acc[i][j] * p.alpha;
            if (p.bias) v += p.bias[col];
            if (p.residual) v += p.residual[(long)row * p.ldr + col];
            float *c = p.C + (long)row * p.ldc + col;
            *c = p.accumulate ? *c + v : v;
        }
}

template <int BM, int BN>
ms_status launch_bf16(const GemmParams &p, int ta, int tb, int splits, hipStream_t s) {
    const size_t smem = (size_t)2 * (BM + BN) * BK * sizeof(bf16_t);
    dim3 grid(p.tiles_m * p.tiles_n, splits);
    ProfScope ps((ta || tb) ? 1 : 0, 2.0 * p.M * p.N * p.K, s);
#define GO(TA, TB)                                                                                        \
    do {                                                                                                  \
        static bool attr_set = false;                                                                     \
        if (!attr_set && smem > 48 * 1024) {                                                              \
            MS_CHECK_HIP(hipFuncSetAttribute((const void *)gemm_bf16_kernel<BM, BN, TA, TB>,              \
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));     \
            attr_set = true;                                                                              \
        }                                                                                                 \
        gemm_bf16_kernel<BM, BN, TA, TB><<<grid, 256, smem, s>>>(p);                                      \
    } while (0)
    if (!ta && !tb) GO(false, false);
    else if (!ta && tb) GO(false, true);
    else if (ta && !tb) GO(true, false);
    else GO(true, true);
#undef GO
    MS_LAUNCH_CHECK();
    return MS_OK;
}

}  // namespace

extern "C" ms_status ms_k_gemm(int32_t dtype, int32_t trans_a, int32_t trans_b, int32_t M, int32_t N, int32_t K,
                               float alpha, const void *A, int64_t lda, const void *B, int64_t ldb, void *C,
                               int64_t ldc, int32_t c_fp32, int32_t accumulate, const void *bias,
                               const void *residual, int64_t ldr, int32_t residual_fp32, int32_t split_k,
                               void *stream) {
    if (M == 0 || N == 0) return MS_OK;
    if (!A || !B || !C || M < 0 || N < 0 || K < 0) return ms_fail(MS_ERR_INVALID_ARG, "gemm: null pointer or negative size");
    if (accumulate && !c_fp32 && dtype == MS_BF16) return ms_fail(MS_ERR_INVALID_ARG, "gemm: accumulate needs an fp32 C");
    hipStream_t s = (hipStream_t)stream;
    if (dtype == MS_F32) {
        GemmF32Params p;
        p.A = (const float *)A; p.B = (const float *)B; p.C = (float *)C;
        p.bias = (const float *)bias; p.residual = (const float *)residual;
        p.sam = trans_a ? 1 : lda; p.sak = trans_a ? lda : 1;
        p.sbn = trans_b ? 1 : ldb; p.sbk = trans_b ? ldb : 1;
        p.ldc = ldc; p.ldr = ldr; p.M = M; p.N = N; p.K = K; p.alpha = alpha; p.accumulate = accumulate;
        gemm_f32_kernel<<<dim3(ms_cdiv(N, 64), ms_cdiv(M, 64)), 256, 0, s>>>(p);
        MS_LAUNCH_CHECK();
        return MS_OK;
    }
    auto al = [](const void *q) { return ((uintptr_t)q & 15) == 0; };
    if (!al(A) || !al(B) || lda % 8 || ldb % 8 || (trans_a ? M % 8 : K % 8) || (trans_b ? N % 8 : K % 8))
        return ms_fail(MS_ERR_UNSUPPORTED,
                       "gemm(bf16): contiguous dimension of each operand must be a multiple of 8 and 16-byte aligned "
                       "(M=%d N=%d K=%d ta=%d tb=%d lda=%ld ldb=%ld)", M, N, K, trans_a, trans_b, (long)lda, (long)ldb);
    GemmParams p;
    p.A = A; p.B = B; p.C = C; p.bias = bias; p.residual = residual;
    p.lda = lda; p.ldb = ldb; p.ldc = ldc; p.ldr = ldr; p.M = M; p.N = N; p.K = K; p.alpha = alpha;
    p.c_fp32 = c_fp32; p.accumulate = accumulate; p.res_fp32 = residual_fp32;
    constexpr int BM = 128, BN = 128;
    p.tiles_m = ms_cdiv(M, BM); p.tiles_n = ms_cdiv(N, BN);
    const int kt_total = ms_cdiv(K, BK) < 1 ? 1 : ms_cdiv(K, BK);
    int splits = split_k;
    if (splits <= 0) {  // automatic: only when accumulating into fp32 and the grid is small
        splits = 1;
        if (accumulate && c_fp32) {
            const int tiles = p.tiles_m * p.tiles_n;
            while (tiles * splits < 512 && kt_total / (splits * 2) >= 8) splits *= 2;
        }
    }
    if (splits > 1 && !(accumulate && c_fp32)) return ms_fail(MS_ERR_INVALID_ARG, "gemm: split_k needs accumulate into fp32");
    if (splits > kt_total) splits = kt_total;
    p.k_tiles_per_split = ms_cdiv(kt_total, splits);
    splits = ms_cdiv(kt_total, p.k_tiles_per_split);
    p.atomic = splits > 1;
    return launch_bf16<BM, BN>(p, trans_a, trans_b, splits, s);
}
