// GEMM kernels of the section path.
//
// bf16: C = alpha * A(m,k) B(n,k) on the CDNA4 matrix cores, all four operand layouts.
//   * gemm_bf16_fast_kernel: workgroup tile 256 x 256 x 64 (8 waves, wave tile 128 x 64, one workgroup per CU) or
//     128 x 128 x 64 (4 waves, two per CU); v_mfma_f32_16x16x32_bf16 by default (v_mfma_f32_32x32x16_bf16 selectable);
//   * every operand tile goes global -> LDS directly (buffer_load ... lds), two LDS buffers per operand, one barrier
//     per K tile; a K-contiguous operand lands as [rows][64] with the 16-byte chunk index XOR-swizzled (applied on the
//     global side of the load; the swizzle makes every fragment read pattern free of LDS bank conflicts), a K-major operand (weight gradients, input gradients) lands as a row tile and is read
//     through the transposing LDS load (ds_read_b64_tr_b16), so no layout needs a transposed copy;
//   * fragments are double-buffered in registers, LDS reads of the next k-step interleaved with the MFMAs;
//   * epilogues (bias, bf16 / fp32 residual, fp32 or bf16 output, accumulate, fused SwiGLU, fused KD statistics / dz)
//     pass the accumulators through the idle LDS buffers so that each lane stores 4 consecutive columns, with
//     non-temporal global accesses; split-K uses fp32 atomics;
//   * workgroup ids are remapped so that each XCD works on a contiguous range of tiles, ordered in groups of M-tiles
//     x all N-tiles, and shares operand panels in its L2;
//   * gemm_bf16_kernel is the register-staged, bounds-checked fallback (K not a multiple of 64 with a K-contiguous
//     operand, matrices of 4 GB and more).
// fp32: a plain LDS-tiled FMA kernel (correctness path of the fp32 workload).
#include <stdlib.h>

#include <atomic>

#include "common.h"
#include "launch.h"
#include "mfma_tiles.h"
#include <type_traits>
#include <utility>

namespace {

// gcc-style vectors: the return types of the buffer load builtins
typedef unsigned int u32x4 __attribute__((vector_size(16)));
typedef unsigned int u32x2 __attribute__((vector_size(8)));

struct GemmParams {
    const void *A, *B;
    void *C;
    const void *bias, *residual;
    long lda, ldb, ldc, ldr;
    int M, N, K;
    int tiles_m, tiles_n;
    int k_tiles_per_split;  // in units of 64
    float alpha;
    int c_fp32, accumulate, atomic, res_fp32, vec_epilogue;
    // KD epilogues (EPI != 0): the tile holds student logits zs; zt = teacher logits of the same chunk
    const float *kd_zt;      // [M, kd_ldz] fp32
    long kd_ldz;
    float *kd_stats;         // EPI_KD_DZ: [M][8] per-token statistics (lse_t at 6, lse_s at 7), read
    float *kd_part;          // EPI_KD_STATS: [M][kd_nparts][8] partial statistics per 64-column strip, written
    int kd_nparts;
    float kd_inv_t, kd_coef;
    // EPI_SWIGLU: B = [gate rows (sg_f) | up rows (sg_f)], N = sg_f output columns; C = silu(gate) * up
    // [M, ldc]; sg_gu (optional) also receives the rounded gate | up pre-activations [M, sg_ldgu]
    int sg_f;
    void *sg_gu;
    long sg_ldgu;
};

enum { EPI_NONE = 0, EPI_KD_DZ = 1, EPI_KD_STATS = 2, EPI_SWIGLU = 3 };

// All-reduce over each aligned group of 16 lanes with DPP moves (one vector-ALU instruction per step, no LDS
// crossbar): swap within pairs, swap pairs within quads, mirror within 8 lanes (reaches the other quad), mirror within
// 16 lanes (reaches the other half).  After the four steps all 16 lanes hold the group's result.
template <int CTRL> __device__ __forceinline__ float dpp_move(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
constexpr int kDppQuadXor1 = 0xB1, kDppQuadXor2 = 0x4E, kDppRowHalfMirror = 0x141, kDppRowMirror = 0x140;
__device__ __forceinline__ float row16_max(float v) {
    v = fmaxf(v, dpp_move<kDppQuadXor1>(v));
    v = fmaxf(v, dpp_move<kDppQuadXor2>(v));
    v = fmaxf(v, dpp_move<kDppRowHalfMirror>(v));
    return fmaxf(v, dpp_move<kDppRowMirror>(v));
}
__device__ __forceinline__ float row16_sum(float v) {
    v += dpp_move<kDppQuadXor1>(v);
    v += dpp_move<kDppQuadXor2>(v);
    v += dpp_move<kDppRowHalfMirror>(v);
    return v + dpp_move<kDppRowMirror>(v);
}

// Cache policy of the vector epilogues' global accesses (auxiliary operand of the buffer instructions): non-temporal.
// The output tile, the residual and the teacher logits stream through once, and the 4 MB L2 of an XCD is what
// keeps the operand panels that its 32 CUs share; left at the default policy the epilogue traffic evicts them
// (measured: fp32-output and fp32-residual GEMMs 7-8 % slower, the c2 step 2.5 %).  The operand loads keep the
// default: made non-temporal they lose that sharing (15 % slower).
constexpr int kStream = 2;

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
        // fragments of k-step kk+1 are fetched from LDS while the MFMAs of k-step kk run
        bf16x8 af[2][MI], bfr[2][NI];
        auto load_frags = [&](int kk, int slot) {
#pragma unroll
            for (int i = 0; i < MI; ++i)
                af[slot][i] = *(const bf16x8 *)(As + cur * BM * BK + lds_off(wm * WTM + i * 32 + frow, kk * 2 + fhalf));
#pragma unroll
            for (int j = 0; j < NI; ++j)
                bfr[slot][j] = *(const bf16x8 *)(Bs + cur * BN * BK + lds_off(wn * WTN + j * 32 + frow, kk * 2 + fhalf));
        };
        load_frags(0, 0);
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            if (kk + 1 < BK / 16) load_frags(kk + 1, (kk + 1) & 1);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk & 1][i], bfr[kk & 1][j], acc[i][j], 0, 0, 0);
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

// ------------------------------------------------------------------ fast path
// Same tiling and MFMA loop, but
//   * an operand stored K-contiguous goes global -> LDS directly (buffer_load ... lds, 16 bytes per
//     lane, one instruction fills 8 tile rows = 1 KB): lane l of the instruction that fills rows
//     8G .. 8G+7 lands at row 8G + l/8, chunk position l%8, so it fetches the chunk that the LDS
//     swizzle assigns to that position.  No staging registers, no LDS store instructions; rows
//     past the end of the matrix read as zero through the buffer descriptor's range check;
//   * the epilogue addresses C (and the residual) through buffer descriptors as well, so rows
//     past M are dropped by the range check and columns past N by one select per column:
//     no per-element branches.
// Needs K % 64 == 0 when an operand is K-contiguous and every matrix below 4 GB.
// The same for an operand stored K-major: the tile is 64 k-rows x COLS columns, kept as COLS/64 sub-tiles
// [64][64]; instruction idx fills 8-row group idx % 8 of sub-tile idx / 8.  Rows past K fall outside the
// descriptor (zeros), so K needs no padding; columns past the matrix edge read the next row (never stored).
template <int COLS, int NWAVES>
struct RowTileStager {
    static constexpr int NI = COLS / 8 / NWAVES;
    unsigned base[NI];                     // byte offset of this lane's 16 bytes at k0 = 0, per instruction
    unsigned ldb;                          // bytes per k-row
    __device__ __forceinline__ void init(long ld, int col0, int wave, int lane) {
        ldb = (unsigned)(ld * 2);
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int idx = wave * NI + i, sub = idx >> 3, g = idx & 7;
            const int r = g * 8 + (lane >> 3);
            const int c = (lane & 7) ^ swz_row(r);
            base[i] = (unsigned)r * ldb + (unsigned)(col0 + sub * 64 + c * 8) * 2;
        }
    }
    __device__ __forceinline__ void issue(__amdgpu_buffer_rsrc_t rs, bf16_t *tile, int k0, int wave, unsigned inv) const {
        const unsigned koff = (unsigned)k0 * ldb;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int idx = wave * NI + i;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void *)(tile + (idx >> 3) * 4096 + (idx & 7) * 512), 16,
                                                     (base[i] + koff) | inv, 0, 0, 0);
        }
    }
};

// B tile of the fused gate/up + SwiGLU GEMM: tile row R = 64 * w + 32 * u + l holds weight row
// u * F + col0 + 32 * w + l (u = 0 gate, 1 up), so that the two 32-column blocks of wave column w are
// the gate and the up pre-activation of the same 32 output columns (same lane, same register).
template <int ROWS, int NWAVES>
struct GateUpStager {
    static constexpr int NI = ROWS / 8 / NWAVES;
    unsigned lanepart;                     // (lane >> 3) rows + swizzle-free part, in bytes
    unsigned ldb;                          // bytes per row
    int x, col0, f;
    __device__ __forceinline__ void init(long ld, int col0_, int f_, int lane) {
        ldb = (unsigned)(ld * 2);
        lanepart = (unsigned)(lane >> 3) * ldb;
        x = (lane & 7) ^ swz_row(lane >> 3);
        col0 = col0_;
        f = f_;
    }
    __device__ __forceinline__ void issue(__amdgpu_buffer_rsrc_t rs, bf16_t *tile, int k0, int wave, unsigned inv) const {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int g = wave * NI + i;                                   // 8-row group of the tile (scalar)
            const int wrow = ((g >> 2) & 1) * f + col0 + (g >> 3) * 32 + (g & 3) * 8;
            const unsigned voff = ((unsigned)wrow * ldb + lanepart + ((x ^ swz_row(8 * g)) << 4)) | inv;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void *)(tile + g * 8 * BK), 16, voff, k0 * 2, 0, 0);
        }
    }
};

template <int ROWS, int NWAVES>
struct DmaStager {
    static constexpr int NI = ROWS / 8 / NWAVES;   // instructions per wave per tile
    unsigned rowoff;                       // byte offset of this lane's row within an 8-row group
    unsigned ld8;                          // bytes between 8-row groups
    int x;                                 // (lane & 7) ^ swz_row(lane >> 3): chunk swizzle without the group term swz_row(8 g)
    __device__ __forceinline__ void init(long ld, int row0, int lane) {
        rowoff = (unsigned)(((long)(row0 + (lane >> 3)) * ld) * 2);
        ld8 = (unsigned)(ld * 16);
        x = (lane & 7) ^ swz_row(lane >> 3);
    }
    // wave (scalar) fills 8-row groups wave*NI .. wave*NI + NI-1 of the tile
    // inv = 0, or kOob to fill the tile with zeros (OR-ing it in puts every lane out of range without a branch)
    __device__ __forceinline__ void issue(__amdgpu_buffer_rsrc_t rs, bf16_t *tile, int k0, int wave, unsigned inv) const {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int g = wave * NI + i;
            const unsigned voff = (rowoff + g * ld8 + ((x ^ swz_row(8 * g)) << 4)) | inv;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void *)(tile + g * 8 * BK), 16, voff, k0 * 2, 0, 0);
        }
    }
};

// Scheduling pattern of one k-step: spread R LDS reads over the first MFMAs (R/M each, at least one),
// then the remaining MFMAs back to back.
template <int N>
__device__ __forceinline__ void sched_reads_then_mfma() {
    __builtin_amdgcn_sched_group_barrier(0x100, N, 0);   // N LDS reads
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
}
template <int R, int PER, int... I>
__device__ __forceinline__ void sched_pairs(std::integer_sequence<int, I...>) {
    (sched_reads_then_mfma<((I + 1) * PER <= R ? PER : R - I * PER)>(), ...);
}
// Scheduling pattern of one k-step with 16-row fragments: per row block, its NB MFMAs and then the reads that
// refill its A fragment (RA reads) and, behind the first NB row blocks, one B fragment (RB reads).
// VM = number of direct-to-LDS loads issued in this k-step (0, or one tile's worth): spread evenly over the row blocks.
template <int NB, int RA, int RB, int VM, int... I>
__device__ __forceinline__ void sched_mfma_then_reads(std::integer_sequence<int, I...>) {
    constexpr int MB = sizeof...(I), PB = (VM + MB - 1) / MB;      // loads per row block
    ((__builtin_amdgcn_sched_group_barrier(0x008, NB, 0), __builtin_amdgcn_sched_group_barrier(0x100, RA + (I < NB ? RB : 0), 0),
      (I * PB < VM ? __builtin_amdgcn_sched_group_barrier(0x020, (VM - I * PB < PB ? VM - I * PB : PB), 0) : (void)0)), ...);
}
template <int R, int M>
__device__ __forceinline__ void interleave_reads_with_mfma() {
    constexpr int PER = R >= M ? (R + M - 1) / M : 1;     // reads in front of each of the first MFMAs
    constexpr int PAIRS = (R + PER - 1) / PER;
    static_assert(PAIRS <= M, "more read groups than MFMAs");
    sched_pairs<R, PER>(std::make_integer_sequence<int, PAIRS>{});
    if constexpr (M > PAIRS) __builtin_amdgcn_sched_group_barrier(0x008, M - PAIRS, 0);
}

// Addresses of the transposing reads of a K-major operand for v_mfma_f32_16x16x32_bf16: the 16 lanes of group g
// (= lane / 16) read k rows 8g .. 8g+7 of the k-step (two reads of four rows) for the 16 columns of a block.
// The LDS swizzle of those rows does not depend on the k-step, and the two 16-column halves of a 32-column
// block differ by one flipped chunk bit: four registers per operand, everything else is a constant offset.
struct TrFragAddr16 {
    int base[2][2];   // [16-column half of the 32-column block][first / second read], element offset within the tile
    __device__ __forceinline__ void init(int w32, int lane) {
        const int g = lane >> 4, r = lane & 15, q = r >> 2;
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
            const int m = w32 * 32 + 16 * hf + 4 * (r & 3);
            const int sub = m >> 6, chunk = (m & 63) >> 3;
#pragma unroll
            for (int rd = 0; rd < 2; ++rd) {
                const int rl = 8 * g + q + 4 * rd;                       // row within the 32-row k-step
                const int sw = swz_row(rl);
                base[hf][rd] = sub * 4096 + rl * 64 + ((chunk ^ sw) << 3) + (m & 7);
            }
        }
    }
    // block16 = index of the wave's 16-column block; off = element offset of its 32-column block's sub-tile pair
    __device__ __forceinline__ bf16x8 frag(const bf16_t *tile, int kk, int block16, int off) const {
        return tr_frag(tile + base[block16 & 1][0] + kk * 2048 + off, tile + base[block16 & 1][1] + kk * 2048 + off);
    }
};

// Addresses of the 16-byte fragment reads of a K-contiguous operand for v_mfma_f32_16x16x32_bf16: lane = (row
// lane % 16 of the 16-row block, k-group lane / 16).  The LDS swizzle makes the chunk position depend on the
// parity of the block and on the k-step; four registers per operand cover all blocks with constant offsets.
struct KFragAddr16 {
    int base[2][2];   // [block parity][k-step], element offset within the tile of block 0 / 1
    __device__ __forceinline__ void init(int row0, int lane) {      // row0 = first tile row of the wave (multiple of 32)
        const int r = lane & 15, g = lane >> 4;
#pragma unroll
        for (int par = 0; par < 2; ++par)
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) base[par][kk] = lds_off(row0 + par * 16 + r, kk * 4 + g) - par * 16 * BK;
    }
    __device__ __forceinline__ bf16x8 frag(const bf16_t *tile, int kk, int block16) const {
        return *(const bf16x8 *)(tile + base[block16 & 1][kk] + block16 * 16 * BK);
    }
};

// M16 selects v_mfma_f32_16x16x32_bf16 (16-row fragments, two k-steps of 32 per K tile) instead of
// v_mfma_f32_32x32x16_bf16 (32-row fragments, four k-steps of 16): the same LDS traffic and the same number of
// accumulator registers, but on operands with realistic bit activity the chip sustains a higher clock on it.
template <int BM, int BN, int WM, int WN, bool TA, bool TB, int EPI = EPI_NONE, bool M16 = false>
__global__ __launch_bounds__(64 * WM * WN) void gemm_bf16_fast_kernel(GemmParams p) {
    constexpr int NT = 64 * WM * WN;
    constexpr int FR = M16 ? 16 : 32;                         // rows of an MFMA fragment / accumulator block
    constexpr int KSTEP = M16 ? 32 : 16, KS = BK / KSTEP;     // contraction depth of an MFMA, k-steps per K tile
    constexpr int WTM = BM / WM, WTN = BN / WN, MI = WTM / FR, NI = WTN / FR;
    constexpr int MI32 = WTM / 32, NI32 = WTN / 32;           // the epilogues work on 32-row blocks
    using acc_t = std::conditional_t<M16, f32x4, f32x16>;
    constexpr int ACC_N = M16 ? 4 : 16;
    // four separate LDS objects (not one carved array): the compiler orders LDS reads against
    // in-flight direct-to-LDS loads by alias analysis, and can only tell the buffer being filled
    // from the buffer being read when they are distinct objects
    __shared__ __align__(16) bf16_t As0[BM * BK], As1[BM * BK], Bs0[BN * BK], Bs1[BN * BK];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keep it in a scalar register
    const int wm = wave / WN, wn = wave % WN;
    int pid;
    {
        const int nb = gridDim.x, b = blockIdx.x;
        const int per = nb >> 3, rem = nb & 7, x = b & 7, q = b >> 3;
        pid = x * per + (x < rem ? x : rem) + q;
    }
    constexpr int GM = BM >= 256 ? 4 : 8;
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

    const bf16_t *A = (const bf16_t *)p.A, *B = (const bf16_t *)p.B;
    std::conditional_t<TA, RowTileStager<BM, WM * WN>, DmaStager<BM, WM * WN>> da;
    std::conditional_t<EPI == EPI_SWIGLU, GateUpStager<BN, WM * WN>,
                       std::conditional_t<TB, RowTileStager<BN, WM * WN>, DmaStager<BN, WM * WN>>> db;
    // descriptor ranges: rows x leading dimension of the matrix as stored ([M or N][K], or [K][M or N])
    const __amdgpu_buffer_rsrc_t ra = make_rsrc(A, TA ? ((long)(p.K - 1) * p.lda + p.M) * 2 : ((long)(p.M - 1) * p.lda + p.K) * 2);
    const __amdgpu_buffer_rsrc_t rb = make_rsrc(B, TB ? ((long)(p.K - 1) * p.ldb + p.N) * 2
                                                      : ((long)((EPI == EPI_SWIGLU ? 2 * p.sg_f : p.N) - 1) * p.ldb + p.K) * 2);
    if constexpr (TA) da.init(p.lda, m0, wave, lane); else da.init(p.lda, m0, lane);
    if constexpr (EPI == EPI_SWIGLU) db.init(p.ldb, n0 / 2, p.sg_f, lane);   // tile tn covers output columns tn * BN/2 ..
    else if constexpr (TB) db.init(p.ldb, n0, wave, lane);
    else db.init(p.ldb, n0, lane);

    acc_t acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < ACC_N; ++r) acc[i][j][r] = 0.f;

    // Start moving K tile kt towards LDS; a tile past the end of this workgroup's K range arrives as zeros.
    // An operand stored K-major ([K][M]) is loaded as a "row tile" (64 k-rows x BM columns) and read back
    // through the transposing LDS load, so every layout goes global -> LDS without staging registers.
    auto fetch = [&](int kt, bf16_t *as, bf16_t *bs) {
        const bool valid = kt < nk;
        const unsigned inv = valid ? 0u : kOob;
        const int k0 = (kt_begin + kt) * BK;
        da.issue(ra, as, k0, wave, inv);
        db.issue(rb, bs, k0, wave, inv);
    };
    // lane -> (fragment row, k-group of 8 consecutive k): 32 rows x 2 groups, or 16 rows x 4 groups
    const int frow = lane & (FR - 1), fhalf = lane / FR;
    // 32-row block i (32-column block j) of this wave within the tile.  For a K-major operand the blocks
    // of a wave are spread one per 64-wide LDS sub-tile pair so that all of them share one LDS address
    // register (constant offsets); for a K-contiguous operand they are adjacent for the same reason.
    auto row_base = [&](int i) { return TA ? i * (32 * WM) + wm * 32 : wm * WTM + i * 32; };
    auto col_base = [&](int j) { return TB ? j * (32 * WN) + wn * 32 : wn * WTN + j * 32; };
    // the same for fragment blocks (16-row blocks are the halves of the 32-row blocks)
    auto frow_base = [&](int i) { return M16 ? row_base(i >> 1) + (i & 1) * 16 : row_base(i); };
    auto fcol_base = [&](int j) { return M16 ? col_base(j >> 1) + (j & 1) * 16 : col_base(j); };
    // Operand fragments are double-buffered in registers: the LDS reads of k-step kk+1 are issued between
    // the MFMAs of k-step kk.
    bf16x8 af[2][MI], bfr[2][NI];
    std::conditional_t<M16, TrFragAddr16, TrFragAddr> tra, trb;
    if constexpr (TA) tra.init(wm, lane);     // block i of the wave: columns i * 32 * WM + wm * 32 of the row tile
    if constexpr (TB) trb.init(wn, lane);
    KFragAddr16 ka, kb;
    if constexpr (M16 && !TA) ka.init(wm * WTM, lane);
    if constexpr (M16 && !TB) kb.init(wn * WTN, lane);
    auto load_a = [&](const bf16_t *as, int kk, int slot, int i) {
        if constexpr (TA && M16) af[slot][i] = tra.frag(as, kk, i, (i >> 1) * (32 * WM / 64) * 4096);
        else if constexpr (TA) af[slot][i] = tra.frag(as, kk, i * (32 * WM / 64) * 4096);
        else if constexpr (M16) af[slot][i] = ka.frag(as, kk, i);
        else af[slot][i] = *(const bf16x8 *)(as + lds_off(frow_base(i) + frow, kk * (KSTEP / 8) + fhalf));
    };
    auto load_b = [&](const bf16_t *bs, int kk, int slot, int j) {
        if constexpr (TB && M16) bfr[slot][j] = trb.frag(bs, kk, j, (j >> 1) * (32 * WN / 64) * 4096);
        else if constexpr (TB) bfr[slot][j] = trb.frag(bs, kk, j * (32 * WN / 64) * 4096);
        else if constexpr (M16) bfr[slot][j] = kb.frag(bs, kk, j);
        else bfr[slot][j] = *(const bf16x8 *)(bs + lds_off(fcol_base(j) + frow, kk * (KSTEP / 8) + fhalf));
    };
    auto load_frags = [&](const bf16_t *as, const bf16_t *bs, int kk, int slot) {
#pragma unroll
        for (int i = 0; i < MI; ++i) load_a(as, kk, slot, i);
#pragma unroll
        for (int j = 0; j < NI; ++j) load_b(bs, kk, slot, j);
    };
    auto mfma_step = [&](int slot) {
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                if constexpr (M16) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[slot][i], bfr[slot][j], acc[i][j], 0, 0, 0);
                else acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[slot][i], bfr[slot][j], acc[i][j], 0, 0, 0);
            }
    };
    constexpr int LDS_READS = (TA ? 2 : 1) * MI + (TB ? 2 : 1) * NI, MFMAS = MI * NI;
    // One k-step: the MFMAs on fragment slot `cur`, with the reads of the next k-step's fragments (tile la / lb,
    // k-step lkk) between them.  With 32-row fragments all reads go in front (one per MFMA).  With 16-row
    // fragments there are twice as many fragment registers per k-step, so the A fragment of row block i is
    // read right after the MFMAs of row block i, into the registers those MFMAs have just released; only the
    // B fragments are held twice.
    auto step = [&](auto cur_c, auto fetch_c, const bf16_t *la, const bf16_t *lb, int lkk) __attribute__((always_inline)) {
        constexpr int cur = decltype(cur_c)::value;          // compile-time: the fragment arrays must stay registers
        constexpr int VM = decltype(fetch_c)::value ? (BM + BN) / 8 / (WM * WN) : 0;   // loads of a fetch issued just before
        if constexpr (M16) {
            static_assert(NI <= MI, "B fragments are read behind the first NI row blocks");
#pragma unroll
            for (int i = 0; i < MI; ++i) {
#pragma unroll
                for (int j = 0; j < NI; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[cur][i], bfr[cur][j], acc[i][j], 0, 0, 0);
                load_a(la, lkk, cur ^ 1, i);
                if (i < NI) load_b(lb, lkk, cur ^ 1, i);
            }
            sched_mfma_then_reads<NI, (TA ? 2 : 1), (TB ? 2 : 1), VM>(std::make_integer_sequence<int, MI>{});
        } else {
            load_frags(la, lb, lkk, cur ^ 1);
            mfma_step(cur);
            interleave_reads_with_mfma<LDS_READS, MFMAS>();
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    // One K tile: steps 0..2 read the next step's fragments from the same tile; before the last step the
    // next tile has landed (own loads: vmcnt(0); the other waves': barrier) and everybody is done reading
    // this one, so its buffers are handed to the tile after next and the last step reads the first
    // fragments of the next tile.  One barrier per tile.
    auto tile = [&](const bf16_t *ca, const bf16_t *cb, const bf16_t *na, const bf16_t *nb, bf16_t *fa, bf16_t *fb,
                    int kt_fetch) __attribute__((always_inline)) {
        using S0 = std::integral_constant<int, 0>;
        using S1 = std::integral_constant<int, 1>;
        static_assert(KS == 2 || KS == 4, "k-steps per K tile");
        step(S0{}, S0{}, ca, cb, 1);
        if constexpr (KS == 4) {
            step(S1{}, S0{}, ca, cb, 2);
            step(S0{}, S0{}, ca, cb, 3);
        }
        dma_publish_barrier();
        fetch(kt_fetch, fa, fb);
        step(S1{}, S1{}, na, nb, 0);
    };

    fetch(0, As0, Bs0);
    dma_publish_barrier();
    fetch(1, As1, Bs1);
    load_frags(As0, Bs0, 0, 0);
    // two K tiles per trip so that each half names its LDS buffers statically; an odd tile count is
    // rounded up with a tile of zeros (a single loop exit keeps the accumulators in place)
    for (int kt = 0; kt < nk; kt += 2) {
        tile(As0, Bs0, As1, Bs1, As0, Bs0, kt + 2);
        tile(As1, Bs1, As0, Bs0, As1, Bs1, kt + 3);
    }
    dma_publish_barrier();   // the (all-zero) tiles still in flight must land before the epilogue reuses LDS

    // ---- epilogue staging: the accumulators of the wave's 32-row block i go to LDS as [32 rows][64 columns]
    // fp32 (v = value transform), from where each lane reads 4 consecutive columns of a row.  The 16-column
    // group index (32x32 MFMA: column bit 5 only) is XOR-ed with row bits so that the lanes of one store
    // instruction, which hold the same columns of rows 4 apart, use different banks.
    auto stg_swz = [](int row) { return M16 ? ((row >> 2) & 3) << 4 : ((row >> 2) & 1) << 5; };
    // The lanes of a wave exchange data through the staging area, and the LDS executes a wave's accesses in
    // program order; what has to be kept is the program order itself: to the compiler a lane's reads and another
    // lane's writes are unrelated addresses that it may reorder.  wave_sync() is a compiler-level fence between the
    // two phases (no instruction).
    auto wave_sync = []() __attribute__((always_inline)) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };
    auto stage_block = [&](float *stg, int i, auto v) __attribute__((always_inline)) {
        wave_sync();     // the reads of the previous block come first
        if constexpr (M16) {
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int j = 0; j < NI; ++j)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int row = h * 16 + 4 * fhalf + r;
                        stg[row * 64 + ((j * 16 + frow) ^ stg_swz(row))] = v(acc[2 * i + h][j][r]);
                    }
        } else {
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = 8 * (r >> 2) + 4 * fhalf + (r & 3);
                    stg[row * 64 + ((j * 32 + frow) ^ stg_swz(row))] = v(acc[i][j][r]);
                }
        }
        wave_sync();     // every lane's values are in LDS before any lane reads
    };
    // ---- epilogue.  C and the residual are addressed through buffer descriptors: rows past M are
    // dropped (stores) or read as zero by the range check, columns past N by one select.
    const int esz = p.c_fp32 ? 4 : 2;
    const __amdgpu_buffer_rsrc_t rc = make_rsrc(p.C, (long)p.M * p.ldc * esz);
    const int rsz = p.res_fp32 ? 4 : 2;
    const __amdgpu_buffer_rsrc_t rr = make_rsrc(p.residual ? p.residual : p.C, p.residual ? (long)p.M * p.ldr * rsz : 0);
    const bf16_t *bias = (const bf16_t *)p.bias;
    if constexpr (EPI == EPI_SWIGLU) {
        // acc[i][0] = gate, acc[i][1] = up of output columns n0/2 + wn*32 + (0..31).  Both are rounded to
        // the storage type first (they are the values a separate activation kernel would read back), staged
        // through LDS as [32 rows][gate 32 | up 32], and each lane then owns 4 consecutive output columns.
        static_assert(WTN == 64 && NI32 == 2 && !TA && !TB, "SwiGLU epilogue is built for the K-contiguous layout");
        constexpr int WPA = BM / 64;
        float *stg = (float *)((wave / WPA) ? As1 : As0) + (wave % WPA) * 2048;
        const int prow = lane >> 3, pcol = (lane & 7) * 4;
        const int colg = n0 / 2 + wn * 32 + pcol;
        const bool cok = colg < p.N;
        const __amdgpu_buffer_rsrc_t rg = make_rsrc(p.sg_gu ? p.sg_gu : p.C, p.sg_gu ? (long)p.M * p.sg_ldgu * 2 : 0);
        auto pack4 = [](const float *v) {
            u32x2 w;
            w[0] = (unsigned)__builtin_bit_cast(unsigned short, (bf16_t)v[0]) | ((unsigned)__builtin_bit_cast(unsigned short, (bf16_t)v[1]) << 16);
            w[1] = (unsigned)__builtin_bit_cast(unsigned short, (bf16_t)v[2]) | ((unsigned)__builtin_bit_cast(unsigned short, (bf16_t)v[3]) << 16);
            return w;
        };
#pragma unroll
        for (int i = 0; i < MI32; ++i) {
            stage_block(stg, i, [&](float a) { return (float)(bf16_t)(a * p.alpha); });
#pragma unroll
            for (int ps = 0; ps < 4; ++ps) {
                const int row = ps * 8 + prow;
                const int flip = stg_swz(row);
                const float4 g4 = *(const float4 *)(stg + row * 64 + (pcol ^ flip));
                const float4 u4 = *(const float4 *)(stg + row * 64 + ((32 + pcol) ^ flip));
                const float gv[4] = {g4.x, g4.y, g4.z, g4.w}, uv[4] = {u4.x, u4.y, u4.z, u4.w};
                float a[4];
#pragma unroll
                for (int e = 0; e < 4; ++e)   // silu(g) u = g u / (1 + e^-g); hardware reciprocal (1 ulp) instead of the division sequence
                    a[e] = gv[e] * uv[e] * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * gv[e]));
                const long rowg = m0 + wm * WTM + i * 32 + row;
                __builtin_amdgcn_raw_buffer_store_b64(pack4(a), rc, cok ? (unsigned)((rowg * p.ldc + colg) * 2) : kOob, 0, kStream);
                if (p.sg_gu) {
                    const unsigned go = cok ? (unsigned)((rowg * p.sg_ldgu + colg) * 2) : kOob;
                    __builtin_amdgcn_raw_buffer_store_b64(pack4(gv), rg, go, 0, kStream);
                    __builtin_amdgcn_raw_buffer_store_b64(pack4(uv), rg, cok ? go + (unsigned)p.sg_f * 2 : kOob, 0, kStream);
                }
            }
        }
        return;
    }
    // ---- vector epilogues.  Each wave passes its accumulators through LDS, 32 rows at a time, to turn the
    // MFMA layout (a lane owns one column) into rows: a lane then handles 4 consecutive columns of a row, so
    // global reads and writes are 8..16 bytes per lane and 128..256 contiguous bytes per row.  What the
    // epilogue reads from memory for a 32-row block (fp32/bf16 residual, C when accumulating, teacher logits)
    // is fetched one block ahead into registers: the loads of block i+1 are issued before the stores of
    // block i, so no pass waits for a store or for its own load's full latency.
    if (EPI != EPI_NONE || p.vec_epilogue) {
        static_assert(WTN == 64, "staging assumes 64-column wave tiles");
        constexpr int WPA = BM / 64;                       // waves sharing one of the (now idle) A buffers
        float *stg = (float *)((wave / WPA) ? As1 : As0) + (wave % WPA) * 2048;
        const int prow = lane >> 4, pcol = (lane & 15) * 4;
        const int colg = n0 + col_base(pcol >> 5) + (pcol & 31);
        const bool cok = colg < p.N;
        // the prefetched stream: KD -> teacher logits (fp32); else residual (fp32 or bf16); else C (accumulate)
        const bool aux_res = EPI == EPI_NONE && p.residual != nullptr;
        const bool aux_c = EPI == EPI_NONE && !aux_res && p.accumulate && p.c_fp32;
        const bool has_aux = EPI != EPI_NONE || aux_res || aux_c;
        const bool aux4 = EPI != EPI_NONE || aux_c || p.res_fp32;                  // 4-byte elements
        const long aux_ld = EPI != EPI_NONE ? p.kd_ldz : (aux_res ? p.ldr : p.ldc);
        const __amdgpu_buffer_rsrc_t ra_ = EPI != EPI_NONE ? make_rsrc(p.kd_zt, (long)p.M * p.kd_ldz * 4) : (aux_res ? rr : rc);
        u32x4 aux[2][8];
        float2 lsev[2][8];                                                         // EPI_KD_DZ: (lse_t, lse_s) of the row
        auto prefetch = [&](int i, u32x4 *dst, float2 *ldst) {
#pragma unroll
            for (int ps = 0; ps < 8; ++ps) {
                const long rowg = m0 + row_base(i) + ps * 4 + prow;
                const unsigned off = cok ? (unsigned)((rowg * aux_ld + colg) * (aux4 ? 4 : 2)) : kOob;
                if (aux4) dst[ps] = __builtin_amdgcn_raw_buffer_load_b128(ra_, off, 0, kStream);
                else {
                    const u32x2 q = __builtin_amdgcn_raw_buffer_load_b64(ra_, off, 0, kStream);
                    dst[ps][0] = q[0]; dst[ps][1] = q[1];
                }
                if constexpr (EPI == EPI_KD_DZ) ldst[ps] = rowg < p.M ? *(const float2 *)(p.kd_stats + rowg * 8 + 6) : make_float2(0.f, 0.f);
            }
        };
        float bv[4] = {0.f, 0.f, 0.f, 0.f};
        if (EPI == EPI_NONE && bias && cok) {
            const uint2 b2 = *(const uint2 *)(bias + colg);
            bv[0] = (float)__builtin_bit_cast(bf16_t, (unsigned short)(b2.x & 0xffff));
            bv[1] = (float)__builtin_bit_cast(bf16_t, (unsigned short)(b2.x >> 16));
            bv[2] = (float)__builtin_bit_cast(bf16_t, (unsigned short)(b2.y & 0xffff));
            bv[3] = (float)__builtin_bit_cast(bf16_t, (unsigned short)(b2.y >> 16));
        }
        auto store4 = [&](const float *v, unsigned co) {
            if (p.c_fp32) {
                u32x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = __builtin_bit_cast(unsigned, v[e]);
                __builtin_amdgcn_raw_buffer_store_b128(w, rc, co, 0, kStream);
            } else {
                u32x2 w;
                w[0] = (unsigned)__builtin_bit_cast(unsigned short, (bf16_t)v[0]) | ((unsigned)__builtin_bit_cast(unsigned short, (bf16_t)v[1]) << 16);
                w[1] = (unsigned)__builtin_bit_cast(unsigned short, (bf16_t)v[2]) | ((unsigned)__builtin_bit_cast(unsigned short, (bf16_t)v[3]) << 16);
                __builtin_amdgcn_raw_buffer_store_b64(w, rc, co, 0, kStream);
            }
        };
        const float it = p.kd_inv_t;
        const float it2 = it * 1.4426950408889634f;      // e^{z/T - m} = 2^{z it2 - m log2(e)}: one fused multiply-add feeds exp2
        if (has_aux) prefetch(0, aux[0], lsev[0]);
#pragma unroll
        for (int i = 0; i < MI32; ++i) {
            if (has_aux && i + 1 < MI32) prefetch(i + 1, aux[(i + 1) & 1], lsev[(i + 1) & 1]);
            stage_block(stg, i, [&](float a) { return a * p.alpha; });
#pragma unroll
            for (int ps = 0; ps < 8; ++ps) {
                const int row = ps * 4 + prow;
                const float4 t = *(const float4 *)(stg + row * 64 + (pcol ^ stg_swz(row)));
                const long rowg = m0 + row_base(i) + row;
                const u32x4 q = aux[i & 1][ps];
                const unsigned co = cok ? (unsigned)((rowg * p.ldc + colg) * esz) : kOob;
                if constexpr (EPI == EPI_NONE) {
                    float v[4] = {t.x + bv[0], t.y + bv[1], t.z + bv[2], t.w + bv[3]};
                    if (aux_res || aux_c) {
                        if (aux4) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) v[e] += __uint_as_float(q[e]);
                        } else {
                            v[0] += (float)__builtin_bit_cast(bf16_t, (unsigned short)(q[0] & 0xffff));
                            v[1] += (float)__builtin_bit_cast(bf16_t, (unsigned short)(q[0] >> 16));
                            v[2] += (float)__builtin_bit_cast(bf16_t, (unsigned short)(q[1] & 0xffff));
                            v[3] += (float)__builtin_bit_cast(bf16_t, (unsigned short)(q[1] >> 16));
                        }
                    }
                    if (aux_res && p.accumulate && p.c_fp32) {        // both a residual and += : C is read in place
                        const u32x4 c4 = __builtin_amdgcn_raw_buffer_load_b128(rc, co, 0, 0);
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] += __uint_as_float(c4[e]);
                    }
                    store4(v, co);
                } else {
                    // the tile holds student logits zs; q = teacher logits zt of the same elements
                    const float zs[4] = {t.x, t.y, t.z, t.w};
                    float zt[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) zt[e] = __uint_as_float(q[e]);
                    if constexpr (EPI == EPI_KD_DZ) {
                        // dz = coef * (exp(zs/T - lse_s) - exp(zt/T - lse_t)) -> C (storage dtype)
                        const float lt2 = lsev[i & 1][ps].x * 1.4426950408889634f, ls2 = lsev[i & 1][ps].y * 1.4426950408889634f;
                        float v[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            v[e] = p.kd_coef * (__builtin_amdgcn_exp2f(__builtin_fmaf(zs[e], it2, -ls2)) -
                                                __builtin_amdgcn_exp2f(__builtin_fmaf(zt[e], it2, -lt2)));
                        store4(v, co);
                    } else {
                        // per row, over this wave's 64 columns: max and sum of exponentials of zt/T and zs/T and
                        // the cross term sum e^{zt/T - m_t} (zt - zs)/T -> kd_part; the 16 lanes that share a
                        // row reduce with data-parallel-primitive moves inside their group (no LDS round trip)
                        float mt = cok ? fmaxf(fmaxf(zt[0], zt[1]), fmaxf(zt[2], zt[3])) : -INFINITY;
                        float ms = cok ? fmaxf(fmaxf(zs[0], zs[1]), fmaxf(zs[2], zs[3])) : -INFINITY;
                        mt = row16_max(mt);
                        ms = row16_max(ms);
                        mt *= it; ms *= it;                                   // T > 0
                        const float mt2 = mt == -INFINITY ? 0.f : mt * 1.4426950408889634f;
                        const float ms2 = ms == -INFINITY ? 0.f : ms * 1.4426950408889634f;
                        float st = 0.f, ss = 0.f, ac = 0.f;
                        if (cok) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const float et = __builtin_amdgcn_exp2f(__builtin_fmaf(zt[e], it2, -mt2));
                                st += et;
                                ac = __builtin_fmaf(et, zt[e] - zs[e], ac);
                                ss += __builtin_amdgcn_exp2f(__builtin_fmaf(zs[e], it2, -ms2));
                            }
                            ac *= it;
                        }
                        st = row16_sum(st);
                        ss = row16_sum(ss);
                        ac = row16_sum(ac);
                        if ((lane & 15) == 0 && rowg < p.M && n0 + wn * WTN < p.N) {
                            float *o = p.kd_part + ((long)rowg * p.kd_nparts + (n0 + wn * WTN) / 64) * 8;
                            *(float4 *)o = make_float4(mt, st, ms, ss);
                            o[4] = ac;
                        }
                    }
                }
            }
        }
        return;
    }
    // scalar epilogue: split-K atomics and shapes whose rows are not 4-element aligned
#pragma unroll
    for (int j = 0; j < NI; ++j) {
        const int col = n0 + fcol_base(j) + frow;
        const bool cok = col < p.N;
        const float bv = (bias && cok) ? (float)bias[col] : 0.f;
#pragma unroll
        for (int i = 0; i < MI; ++i) {
#pragma unroll
            for (int r = 0; r < ACC_N; ++r) {
                const int row = m0 + frow_base(i) + (M16 ? 4 * fhalf + r : 8 * (r >> 2) + 4 * fhalf + (r & 3));
                float v = acc[i][j][r] * p.alpha + bv;
                if (p.residual) {
                    const unsigned ro = cok ? (unsigned)(((long)row * p.ldr + col) * rsz) : kOob;
                    if (p.res_fp32) v += __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rr, ro, 0, 0));
                    else v += (float)__builtin_bit_cast(bf16_t, __builtin_amdgcn_raw_buffer_load_b16(rr, ro, 0, 0));
                }
                const unsigned co = cok ? (unsigned)(((long)row * p.ldc + col) * esz) : kOob;
                if (p.c_fp32) {
                    if (p.atomic) {
                        if (cok && row < p.M) unsafeAtomicAdd((float *)p.C + (long)row * p.ldc + col, v);
                    } else {
                        if (p.accumulate) v += __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rc, co, 0, 0));
                        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), rc, co, 0, 0);
                    }
                } else {
                    __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(unsigned short, (bf16_t)v), rc, co, 0, 0);
                }
            }
            // keep the scheduler from pulling every accumulator out of the AGPRs at once
            __builtin_amdgcn_sched_barrier(0);
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

// Explicit instantiations: the host pass has been seen to reference the launch stubs of some of these
// without defining them when they are only instantiated implicitly from the launcher below.
#define MS_INST(BM, WN, TA, TB)                                                                          \
    template __global__ void gemm_bf16_fast_kernel<BM, BM, 2, WN, TA, TB, EPI_NONE, false>(GemmParams); \
    template __global__ void gemm_bf16_fast_kernel<BM, BM, 2, WN, TA, TB, EPI_NONE, true>(GemmParams)
MS_INST(256, 4, false, false); MS_INST(256, 4, false, true); MS_INST(256, 4, true, false); MS_INST(256, 4, true, true);
MS_INST(128, 2, false, false); MS_INST(128, 2, false, true); MS_INST(128, 2, true, false); MS_INST(128, 2, true, true);
#undef MS_INST
#define MS_INST_EPI(EPI)                                                                                      \
    template __global__ void gemm_bf16_fast_kernel<256, 256, 2, 4, false, false, EPI, false>(GemmParams);    \
    template __global__ void gemm_bf16_fast_kernel<256, 256, 2, 4, false, false, EPI, true>(GemmParams);     \
    template __global__ void gemm_bf16_fast_kernel<128, 128, 2, 2, false, false, EPI, false>(GemmParams);    \
    template __global__ void gemm_bf16_fast_kernel<128, 128, 2, 2, false, false, EPI, true>(GemmParams)
MS_INST_EPI(EPI_KD_DZ); MS_INST_EPI(EPI_KD_STATS); MS_INST_EPI(EPI_SWIGLU);
#undef MS_INST_EPI

// Kernel selection switches, for measurements and tests only: the environment gives the process-wide setting
// (MS_GEMM_TILE = 128 / 256 forces the fast kernels' tile, -1 disables them; MS_GEMM_MFMA16 = 0 selects
// v_mfma_f32_32x32x16_bf16), ms_k_gemm_config overrides it at run time.  The overrides are atomics, so changing them
// from one thread while another launches is defined, but which setting a concurrent launch sees is not: production
// callers leave them alone (automatic choice by shape).
constexpr int kUnset = -1000;
std::atomic<int> g_tile_override{kUnset}, g_mfma16_override{kUnset};
int forced_tile() {
    static const int env = [] { const char *e = getenv("MS_GEMM_TILE"); return e ? atoi(e) : 0; }();
    const int o = g_tile_override.load(std::memory_order_relaxed);
    return o != kUnset ? o : env;
}
bool use_mfma16() {
    static const bool env = [] { const char *e = getenv("MS_GEMM_MFMA16"); return !e || atoi(e) != 0; }();
    const int o = g_mfma16_override.load(std::memory_order_relaxed);
    return o != kUnset ? o != 0 : env;
}

template <int BM, int BN, int WM, int WN, int EPI>
void launch_fast_epi(const GemmParams &p, dim3 grid, hipStream_t s) {
    // (the 128 x 128 dz variant would need more than the 256 registers that let two workgroups share a CU)
    if (use_mfma16() && !(BM == 128 && EPI == EPI_KD_DZ))
        gemm_bf16_fast_kernel<BM, BN, WM, WN, false, false, EPI, true><<<grid, 64 * WM * WN, 0, s>>>(p);
    else gemm_bf16_fast_kernel<BM, BN, WM, WN, false, false, EPI, false><<<grid, 64 * WM * WN, 0, s>>>(p);
}

template <int BM, int BN, int WM, int WN>
ms_status launch_bf16_fast(const GemmParams &p, int ta, int tb, int splits, hipStream_t s) {
    dim3 grid(p.tiles_m * p.tiles_n, splits);
    ProfScope ps((ta || tb) ? 1 : 0, 2.0 * p.M * p.N * p.K, s);
#define GO(TA, TB)                                                                                             \
    do {                                                                                                       \
        if (use_mfma16()) gemm_bf16_fast_kernel<BM, BN, WM, WN, TA, TB, EPI_NONE, true><<<grid, 64 * WM * WN, 0, s>>>(p);   \
        else gemm_bf16_fast_kernel<BM, BN, WM, WN, TA, TB, EPI_NONE, false><<<grid, 64 * WM * WN, 0, s>>>(p);  \
    } while (0)
    if (!ta && !tb) GO(false, false);
    else if (!ta && tb) GO(false, true);
    else if (ta && !tb) GO(true, false);
    else GO(true, true);
#undef GO
    MS_LAUNCH_CHECK();
    return MS_OK;
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

extern "C" ms_status ms_k_gemm_config(int32_t tile, int32_t mfma16) {
    if (!(tile == -1 || tile == 0 || tile == 128 || tile == 256) || mfma16 < -1 || mfma16 > 1)
        return ms_fail(MS_ERR_INVALID_ARG, "gemm_config: tile must be -1, 0, 128 or 256 and mfma16 -1, 0 or 1");
    g_tile_override = tile == 0 ? kUnset : tile;
    g_mfma16_override = mfma16 < 0 ? kUnset : mfma16;
    return MS_OK;
}

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
    GemmParams p = {};
    p.A = A; p.B = B; p.C = C; p.bias = bias; p.residual = residual;
    p.lda = lda; p.ldb = ldb; p.ldc = ldc; p.ldr = ldr; p.M = M; p.N = N; p.K = K; p.alpha = alpha;
    p.c_fp32 = c_fp32; p.accumulate = accumulate; p.res_fp32 = residual_fp32;
    // fast path (direct-to-LDS loads, descriptor-addressed epilogue) needs full K tiles for a K-contiguous
    // operand and 32-bit byte offsets; tile 256 x 256 when that still gives every CU work, else 128 x 128
    const int forced = forced_tile();
    const long lim = (1L << 32) - (1L << 20);
    const long rows_a = trans_a ? K : M, rows_b = trans_b ? K : N;
    const bool fast = forced >= 0 && ((trans_a && trans_b) || K % BK == 0) && (rows_a + 256) * lda * 2 < lim &&
                      (rows_b + 256) * ldb * 2 < lim && ((long)M + 256) * ldc * 4 < lim &&
                      (!residual || ((long)M + 256) * ldr * 4 < lim);
    // 256 x 256 (8 waves, one workgroup per CU) runs ~1.25x the rate of 128 x 128 (4 waves, two per CU) when the
    // grid fills whole rounds of CUs: pick by estimated rate x last-round occupancy
    const long tiles256 = (long)ms_cdiv(M, 256) * ms_cdiv(N, 256), tiles128 = (long)ms_cdiv(M, 128) * ms_cdiv(N, 128);
    const double eff256 = (double)tiles256 / (double)(ms_cdiv(tiles256, 256) * 256L);
    const double eff128 = (double)tiles128 / (double)(ms_cdiv(tiles128, 512) * 512L);
    bool big = fast && (forced > 0 ? forced == 256 : (tiles256 >= 192 && 1.25 * eff256 > eff128));
    const int kt_total = ms_cdiv(K, BK) < 1 ? 1 : ms_cdiv(K, BK);
    int splits = split_k;
    if (splits <= 0) {  // automatic: only when accumulating into fp32 (weight gradients: small M x N, long K)
        splits = 1;
        if (accumulate && c_fp32 && fast) {
            // Cost model fitted to measurements on wgrad shapes (microseconds): rounds of resident workgroups
            // x (K tiles per split x time per K tile + fixed part) + one pass of fp32 atomics over C per split
            // at ~2 TB/s.  256 x 256: one workgroup per CU, 1.57 us per K tile; 128 x 128: two per CU, 1.07 us.
            double best = 1e30;
            for (int t256 = 0; t256 <= 1; ++t256) {
                if (forced > 0 && (forced == 256) != (t256 == 1)) continue;
                const long tiles = t256 ? tiles256 : tiles128, slots = t256 ? 256 : 512;
                const double tk = t256 ? 1.57 : 1.07, fix = t256 ? 12.0 : 5.0;
                for (int sp = 1; sp <= 8 && (sp == 1 || kt_total / sp >= 8); ++sp) {
                    const double rounds = (double)ms_cdiv(tiles * sp, slots);
                    const double est = rounds * (ms_cdiv(kt_total, sp) * tk + fix) + (sp > 1 ? 4.0e-6 * M * N * sp / 2.0 : 0.0);
                    if (est < best) { best = est; splits = sp; big = t256 == 1; }
                }
            }
        } else if (accumulate && c_fp32) {
            const int tiles = (int)tiles128;
            while (tiles * splits < 512 && kt_total / (splits * 2) >= 8) splits *= 2;
        }
    }
    const int BM = big ? 256 : 128, BN = BM;
    p.tiles_m = ms_cdiv(M, BM); p.tiles_n = ms_cdiv(N, BN);
    if (splits > 1 && !(accumulate && c_fp32)) return ms_fail(MS_ERR_INVALID_ARG, "gemm: split_k needs accumulate into fp32");
    if (splits > kt_total) splits = kt_total;
    p.k_tiles_per_split = ms_cdiv(kt_total, splits);
    splits = ms_cdiv(kt_total, p.k_tiles_per_split);
    p.atomic = splits > 1;
    auto al16 = [](const void *q) { return ((uintptr_t)q & 15) == 0; };
    p.vec_epilogue = !p.atomic && N % 4 == 0 && ldc % 4 == 0 && al16(C) && (!residual || (ldr % 4 == 0 && al16(residual))) &&
                     (!bias || ((uintptr_t)bias & 7) == 0);
    if (big) return launch_bf16_fast<256, 256, 2, 4>(p, trans_a, trans_b, splits, s);
    if (fast) return launch_bf16_fast<128, 128, 2, 2>(p, trans_a, trans_b, splits, s);
    return launch_bf16<128, 128>(p, trans_a, trans_b, splits, s);
}

// ------------------------------------------------------------------ student-logits GEMM with KD epilogues
// zs = A[M,K] B[N,K]^T is never stored: mode EPI_KD_STATS folds it (with the teacher logits zt of the same
// chunk) into per-strip partial statistics, mode EPI_KD_DZ turns it into dz.  bf16 fast path only.
bool gemm_kd_epilogue_supported(int M, int N, int K, const void *A, long lda, const void *B, long ldb, const float *zt,
                                long ldz, const void *dz, long lddz, int dz_fp32) {
    auto al = [](const void *q) { return ((uintptr_t)q & 15) == 0; };
    const long lim = (1L << 32) - (1L << 20);
    const int forced = forced_tile();
    return forced >= 0 && M > 0 && N > 0 && K > 0 && K % BK == 0 && N % 4 == 0 && al(A) && al(B) && al(zt) && lda % 8 == 0 &&
           ldb % 8 == 0 && ldz % 4 == 0 && ((long)M + 256) * lda * 2 < lim && ((long)N + 256) * ldb * 2 < lim &&
           ((long)M + 256) * ldz * 4 < lim && (!dz || (al(dz) && lddz % 4 == 0 && ((long)M + 256) * lddz * (dz_fp32 ? 4 : 2) < lim));
}

ms_status gemm_kd_epilogue(int mode, int M, int N, int K, const void *A, long lda, const void *B, long ldb, const float *zt,
                           long ldz, float *stats, float *part, int nparts, float inv_t, float coef, void *dz, long lddz,
                           int dz_fp32, hipStream_t s) {
    if (!gemm_kd_epilogue_supported(M, N, K, A, lda, B, ldb, zt, ldz, mode == EPI_KD_DZ ? dz : nullptr, lddz, dz_fp32))
        return ms_fail(MS_ERR_UNSUPPORTED, "gemm_kd_epilogue: shape or alignment outside the fast path");
    if ((mode == EPI_KD_DZ && (!dz || !stats)) || (mode == EPI_KD_STATS && (!part || nparts < ms_cdiv(N, 64))) ||
        (mode != EPI_KD_DZ && mode != EPI_KD_STATS))
        return ms_fail(MS_ERR_INVALID_ARG, "gemm_kd_epilogue: bad mode or null buffer");
    GemmParams p = {};
    p.A = A; p.B = B; p.C = dz; p.lda = lda; p.ldb = ldb; p.ldc = lddz; p.M = M; p.N = N; p.K = K; p.alpha = 1.f;
    p.c_fp32 = dz_fp32;
    p.kd_zt = zt; p.kd_ldz = ldz; p.kd_stats = stats; p.kd_part = part; p.kd_nparts = nparts; p.kd_inv_t = inv_t; p.kd_coef = coef;
    const int forced = forced_tile();
    const long tiles256 = (long)ms_cdiv(M, 256) * ms_cdiv(N, 256), tiles128 = (long)ms_cdiv(M, 128) * ms_cdiv(N, 128);
    const double eff256 = (double)tiles256 / (double)(ms_cdiv(tiles256, 256) * 256L);
    const double eff128 = (double)tiles128 / (double)(ms_cdiv(tiles128, 512) * 512L);
    const bool big = forced > 0 ? forced == 256 : (tiles256 >= 192 && 1.25 * eff256 > eff128);
    const int BM = big ? 256 : 128;
    p.tiles_m = ms_cdiv(M, BM); p.tiles_n = ms_cdiv(N, BM);
    p.k_tiles_per_split = ms_cdiv(K, BK);
    dim3 grid(p.tiles_m * p.tiles_n, 1);
    ProfScope ps(0, 2.0 * M * N * K, s);
    if (big) {
        if (mode == EPI_KD_DZ) launch_fast_epi<256, 256, 2, 4, EPI_KD_DZ>(p, grid, s);
        else launch_fast_epi<256, 256, 2, 4, EPI_KD_STATS>(p, grid, s);
    } else {
        if (mode == EPI_KD_DZ) launch_fast_epi<128, 128, 2, 2, EPI_KD_DZ>(p, grid, s);
        else launch_fast_epi<128, 128, 2, 2, EPI_KD_STATS>(p, grid, s);
    }
    MS_LAUNCH_CHECK();
    return MS_OK;
}

// ------------------------------------------------------------------ fused gate/up GEMM + SwiGLU
// act[M, F] = silu(A W_gate^T) * (A W_up^T) with W = [gate rows | up rows] ([2F, K]); gate_up (optional,
// [M, 2F]) also receives the rounded pre-activations for the backward pass.  bf16 fast path only.
bool gemm_swiglu_supported(int M, int F, int K, const void *A, long lda, const void *W, long ldw, const void *act, long ldact,
                           const void *gate_up, long ldgu) {
    auto al = [](const void *q) { return ((uintptr_t)q & 15) == 0; };
    const long lim = (1L << 32) - (1L << 20);
    const int forced = forced_tile();
    return forced >= 0 && M > 0 && F > 0 && K > 0 && K % BK == 0 && F % 4 == 0 && al(A) && al(W) && al(act) && lda % 8 == 0 &&
           ldw % 8 == 0 && ldact % 4 == 0 && ((long)M + 256) * lda * 2 < lim && (2L * F + 256) * ldw * 2 < lim &&
           ((long)M + 256) * ldact * 2 < lim && (!gate_up || (al(gate_up) && ldgu % 4 == 0 && ((long)M + 256) * ldgu * 2 < lim));
}

ms_status gemm_swiglu(int M, int F, int K, const void *A, long lda, const void *W, long ldw, void *act, long ldact,
                      void *gate_up, long ldgu, hipStream_t s) {
    if (!gemm_swiglu_supported(M, F, K, A, lda, W, ldw, act, ldact, gate_up, ldgu))
        return ms_fail(MS_ERR_UNSUPPORTED, "gemm_swiglu: shape or alignment outside the fast path");
    GemmParams p = {};
    p.A = A; p.B = W; p.C = act; p.lda = lda; p.ldb = ldw; p.ldc = ldact; p.M = M; p.N = F; p.K = K; p.alpha = 1.f;
    p.sg_f = F; p.sg_gu = gate_up; p.sg_ldgu = ldgu;
    const int forced = forced_tile();
    // a tile covers BN/2 output columns (BN weight rows: gate and up)
    const long tiles256 = (long)ms_cdiv(M, 256) * ms_cdiv(F, 128), tiles128 = (long)ms_cdiv(M, 128) * ms_cdiv(F, 64);
    const double eff256 = (double)tiles256 / (double)(ms_cdiv(tiles256, 256) * 256L);
    const double eff128 = (double)tiles128 / (double)(ms_cdiv(tiles128, 512) * 512L);
    const bool big = forced > 0 ? forced == 256 : (tiles256 >= 192 && 1.25 * eff256 > eff128);
    const int BM = big ? 256 : 128;
    p.tiles_m = ms_cdiv(M, BM); p.tiles_n = ms_cdiv(F, BM / 2);
    p.k_tiles_per_split = ms_cdiv(K, BK);
    dim3 grid(p.tiles_m * p.tiles_n, 1);
    ProfScope ps(0, 4.0 * M * F * K, s);
    if (big) launch_fast_epi<256, 256, 2, 4, EPI_SWIGLU>(p, grid, s);
    else launch_fast_epi<128, 128, 2, 2, EPI_SWIGLU>(p, grid, s);
    MS_LAUNCH_CHECK();
    return MS_OK;
}

extern "C" ms_status ms_k_gemm_swiglu(int32_t M, int32_t F, int32_t K, const void *A, int64_t lda, const void *W, int64_t ldw,
                                      void *act, int64_t ldact, void *gate_up, int64_t ldgu, void *stream) {
    if (!A || !W || !act) return ms_fail(MS_ERR_INVALID_ARG, "gemm_swiglu: null pointer");
    return gemm_swiglu(M, F, K, A, lda, W, ldw, act, ldact, gate_up, ldgu, (hipStream_t)stream);
}
