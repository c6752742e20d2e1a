// LDS tile helpers shared by the matrix-core kernels (GEMM and attention).
//
// A tile is [rows][64] bf16: 128-byte rows of eight 16-byte chunks, chunk c of row r stored at position
// c ^ swz_row(r).  swz_row is linear over GF(2) in row bits b0..b4: b1 -> 4, b2 -> 3, b3 -> 2, b4 -> 1, b0 -> 1.
// Rows 32 apart use the same chunk order, so fragment addresses differ by compile-time constants.
// The choice follows from how the LDS serves a wave (measured with timing probes of in-bounds reads):
//   * 16-byte reads: 16 lanes per cycle, namely the lanes of one half of the wave with the same parity of
//     lane bits 2, 3 and 4; they must hit 16 different 16-byte slots modulo 256 bytes;
//   * 8-byte reads (also the transposing ds_read_b64_tr_b16): the 32 lanes of a half-wave per cycle, which must
//     hit 32 different 8-byte units modulo 256 bytes.
// With this swizzle the fragment reads of all four patterns in use are conflict-free: K-contiguous fragments of 16
// rows (lane = row + 16 * k-group) and of 32 rows (lane = row + 32 * k-group), and the transposing reads of
// K-major tiles for 16- and 32-column fragments.
// Stager moves one such tile global -> registers -> LDS; for an operand whose 64-wide dimension is the strided one
// in memory it transposes 8 x 8 blocks in registers on the way.
#pragma once
#include "common.h"

constexpr int BK = 64;

__device__ __forceinline__ int swz_row(int r) { return ((r & 2) << 1) | (((r >> 1) ^ (r >> 2)) & 2) | ((r ^ (r >> 2) ^ (r >> 4)) & 1); }
__device__ __forceinline__ int swz(int r, int c) { return c ^ swz_row(r); }

// element offset (in bf16) of 16-byte chunk c of row r in a [rows][64] tile
__device__ __forceinline__ int lds_off(int r, int c) { return r * BK + swz(r, c) * 8; }

// ---- direct global -> LDS loads through a buffer descriptor ----------------------------------
// buffer_load_dwordx4 ... lds: lane l of the wave writes its 16 bytes at (LDS base) + 16 l; a lane
// whose byte offset is outside the descriptor's range writes zeros.
typedef __attribute__((address_space(3))) void lds_void;
constexpr unsigned kOob = 0xFFFFF000u;   // byte offset beyond any descriptor range

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *p, long bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)(unsigned)bytes, 0x00020000);
}

// Barrier that hands a tile filled by direct-to-LDS loads to the other waves of the workgroup: a wave's own
// loads must have landed (vmcnt(0): the loads complete in order, and at every such barrier all outstanding ones
// belong to the tile being published) before it tells the others so.  The wait is written out rather than left
// to the compiler's lowering of the barrier's fence.  s_waitcnt operand (gfx9 encoding): vmcnt = bits 3:0 and
// 15:14, expcnt = bits 6:4, lgkmcnt = bits 11:8; 0x0F70 waits for vmcnt(0) only.
__device__ __forceinline__ void dma_publish_barrier() {
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
}

// ---- transposing LDS read (ds_read_b64_tr_b16) --------------------------------------------------
// Within each group of 16 lanes, lane r supplies the address of an 8-byte row (4 bf16); lane i
// receives element i%4 of rows i/4, 4 + i/4, 8 + i/4, 12 + i/4.  With a tile stored [k][m]
// (m contiguous) and lane r pointing at T[k0 + r/4][m0 + 4 (r%4)], lane i therefore receives
// T[k0 .. k0+3][m0 + i]: four consecutive k of its own column, i.e. MFMA operand slots.
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
__device__ __forceinline__ bf16x8 tr_frag(const bf16_t *p0, const bf16_t *p1) {
    const bf16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)p0);
    const bf16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)p1);
    return __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
}

// ---- "row tiles": 64 rows x W columns of a row-major matrix, kept as W/64 sub-tiles [64][64] --------
// One direct-to-LDS instruction: instruction idx fills 8-row group idx % 8 of sub-tile idx / 8 from rows
// row0.. of a matrix with leading dimension ld (elements), starting at column col0.  Columns past W
// arrive as zeros; rows past the end of the matrix are zeroed by the descriptor's range check.
template <int W>
__device__ __forceinline__ void rowtile_dma(__amdgpu_buffer_rsrc_t rs, bf16_t *tile, int row0, long ld, int col0, int idx,
                                            int lane, unsigned inv = 0) {
    const int sub = idx >> 3, g = idx & 7;
    const int r = g * 8 + (lane >> 3);
    const int c = (lane & 7) ^ swz_row(r);
    const int d = sub * 64 + c * 8;
    const unsigned voff = (d < W ? (unsigned)(((long)(row0 + r) * ld + col0 + d) * 2) : kOob) | inv;   // inv = kOob: all zeros
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void *)(tile + sub * 4096 + g * 512), 16, voff, 0, 0, 0);
}

// The same for a tile of 32 rows (sub-tiles [32][64]): instruction idx fills 8-row group idx % 4 of sub-tile idx / 4.
template <int W>
__device__ __forceinline__ void rowtile32_dma(__amdgpu_buffer_rsrc_t rs, bf16_t *tile, int row0, long ld, int col0, int idx,
                                              int lane, unsigned inv = 0) {
    const int sub = idx >> 2, g = idx & 3;
    const int r = g * 8 + (lane >> 3);
    const int c = (lane & 7) ^ swz_row(r);
    const int d = sub * 64 + c * 8;
    const unsigned voff = (d < W ? (unsigned)(((long)(row0 + r) * ld + col0 + d) * 2) : kOob) | inv;   // inv = kOob: all zeros
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void *)(tile + sub * 2048 + g * 512), 16, voff, 0, 0, 0);
}

// The same loads for a loop that fetches tile after tile: everything that depends on the lane alone is computed
// once (RowTileLane), everything that depends on the instruction index or the tile is wave-uniform and stays in
// scalar registers, so that a load costs three vector instructions (add, xor-shift, add) instead of a 64-bit
// address computation.  base = byte offset of (row0, col0) in the matrix, ld2 = bytes per matrix row; idx must be
// wave-uniform.  ROWS = 64 (rowtile_dma's layout) or 32 (rowtile32_dma's).
struct RowTileLane {
    unsigned rowpart;   // (lane / 8) * ld2: the lane's row within an 8-row group
    int x;              // (lane % 8) ^ swz_row(lane / 8): chunk position with the lane's part of the swizzle
    __device__ __forceinline__ void init(int lane, unsigned ld2) {
        rowpart = (unsigned)(lane >> 3) * ld2;
        x = (lane & 7) ^ swz_row(lane >> 3);
    }
};
template <int W, int ROWS>
__device__ __forceinline__ void rowtile_dma_lane(__amdgpu_buffer_rsrc_t rs, bf16_t *tile, unsigned base, unsigned ld2, int idx,
                                                 const RowTileLane &L, unsigned inv = 0) {
    constexpr int G = ROWS / 8;                              // 8-row groups per sub-tile
    const int sub = idx / G, g = idx % G;
    const int c = L.x ^ swz_row(8 * g);                      // swz_row is linear: swz_row(8 g + l) = swz_row(8 g) ^ swz_row(l)
    unsigned voff = L.rowpart + (base + (unsigned)(8 * g) * ld2 + (unsigned)sub * 128u) + ((unsigned)c << 4);
    if (W % 64 != 0 && sub == W / 64) voff = c * 8 < W % 64 ? voff : kOob;   // columns past W arrive as zeros
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void *)(tile + sub * (ROWS * 64) + g * 512), 16, voff | inv, 0, 0, 0);
}

// MFMA operand fragment whose 32 "rows" are tile columns m0 .. m0+31 and whose k-slots are tile rows:
// half h of the wave gets rows k0 + 4h + {0..3} (slots 0..3) and k0 + 8 + 4h + {0..3} (slots 4..7).
// SUB = elements per 64-column sub-tile (64 x tile height).
template <int SUB = 4096>
__device__ __forceinline__ bf16x8 rowtile_tr_frag(const bf16_t *tile, int k0, int m0, int lane) {
    const int h = lane >> 5, dg = (lane >> 4) & 1, r = lane & 15;
    const int row = k0 + 4 * h + (r >> 2);
    const int m = m0 + 16 * dg + 4 * (r & 3);
    const bf16_t *base = tile + (m >> 6) * SUB + (m & 7);
    const int chunk = (m & 63) >> 3;
    return tr_frag(base + lds_off(row, chunk), base + lds_off(row + 8, chunk));
}

// Same, in the standard k-slot order of a K-contiguous fragment: half h gets rows k0 + 8h + {0..7}, so it
// pairs with 16-byte reads of the other operand.
__device__ __forceinline__ bf16x8 rowtile_tr_frag_std(const bf16_t *tile, int k0, int m0, int lane) {
    const int h = lane >> 5, dg = (lane >> 4) & 1, r = lane & 15;
    const int row = k0 + 8 * h + (r >> 2);
    const int m = m0 + 16 * dg + 4 * (r & 3);
    const bf16_t *base = tile + (m >> 6) * 4096 + (m & 7);
    const int chunk = (m & 63) >> 3;
    return tr_frag(base + lds_off(row, chunk), base + lds_off(row + 4, chunk));
}

// Addresses of rowtile_tr_frag_std for one wave, factored so that only four registers per operand are
// live: the swizzle term depends on the k-step's parity alone, everything else is a constant offset.
// The wave's 32-column blocks start at column w32 * 32 of sub-tile pairs that the caller selects with
// a constant element offset (multiples of 4096).
struct TrFragAddr {
    int base[2][2];   // [k-step parity][first / second read], element offset within the tile
    __device__ __forceinline__ void init(int w32, int lane) {
        const int h = lane >> 5, dg = (lane >> 4) & 1, r = lane & 15, q = r >> 2;
        const int m = w32 * 32 + 16 * dg + 4 * (r & 3);
        const int sub = m >> 6, chunk = (m & 63) >> 3;
#pragma unroll
        for (int par = 0; par < 2; ++par)
#pragma unroll
            for (int rd = 0; rd < 2; ++rd) {
                const int rl = 8 * h + q + 4 * rd;                       // row within the 16-row k-step
                const int sw = swz_row(16 * par + rl);
                base[par][rd] = sub * 4096 + rl * 64 + ((chunk ^ sw) << 3) + (m & 7);
            }
    }
    __device__ __forceinline__ bf16x8 frag(const bf16_t *tile, int kk, int off) const {
        return tr_frag(tile + base[kk & 1][0] + kk * 1024 + off, tile + base[kk & 1][1] + kk * 1024 + off);
    }
};

__device__ __forceinline__ uint32_t pack_lo(uint32_t a, uint32_t b) { return (a & 0xffffu) | (b << 16); }
__device__ __forceinline__ uint32_t pack_hi(uint32_t a, uint32_t b) { return (a >> 16) | (b & 0xffff0000u); }

// Staging of one operand tile of ROWS x 64 (rows = m or n index, 64 = k).
template <int ROWS, bool TRANS, int NT = 256>
struct Stager {
    static constexpr int NB = (ROWS + NT - 1) / NT;          // 8 x 8 blocks per thread (transposed)
    static constexpr int RPP = NT / 8;                      // rows per pass (row-major)
    static constexpr int NREG = TRANS ? 8 * NB : ROWS / RPP;
    uint4 reg[NREG];

    // P: base pointer; ld: leading dimension; row0: first m/n of the tile; rows_total: M or N;
    // k0: first k of the tile; k_end: exclusive k bound.
    __device__ __forceinline__ void load(const bf16_t *P, long ld, int row0, int rows_total, int k0, int k_end, int tid) {
        if constexpr (!TRANS) {
            const int c = tid & 7, r0 = tid >> 3;
            const int k = k0 + c * 8;
#pragma unroll
            for (int i = 0; i < NREG; ++i) {
                const int r = row0 + r0 + RPP * i;
                if (r < rows_total && k < k_end) reg[i] = *(const uint4 *)(P + (long)r * ld + k);
                else reg[i] = make_uint4(0, 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const int blk = tid + NT * b;   // 8 x 8 block: k-block fastest, then m-block
                const int kb = blk & 7, mb = blk >> 3;
                const int m = row0 + mb * 8;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int k = k0 + kb * 8 + j;
                    if (blk < ROWS && m < rows_total && k < k_end) reg[b * 8 + j] = *(const uint4 *)(P + (long)k * ld + m);
                    else reg[b * 8 + j] = make_uint4(0, 0, 0, 0);
                }
            }
        }
    }

    __device__ __forceinline__ void store(bf16_t *tile, int tid) const {
        if constexpr (!TRANS) {
            const int c = tid & 7, r0 = tid >> 3;
#pragma unroll
            for (int i = 0; i < NREG; ++i) {
                const int r = r0 + RPP * i;
                *(uint4 *)(tile + lds_off(r, c)) = reg[i];
            }
        } else {
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const int blk = tid + NT * b;
                if (blk < ROWS) {
                    const int kb = blk & 7, mb = blk >> 3;
                    const uint4 *in = &reg[b * 8];
                    // in[j] = 8 m-values at k = j; out row i = 8 k-values at m = i
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        uint32_t w[4];
#pragma unroll
                        for (int pp = 0; pp < 4; ++pp) {
                            const uint32_t a = ((const uint32_t *)&in[2 * pp])[i >> 1];
                            const uint32_t bb = ((const uint32_t *)&in[2 * pp + 1])[i >> 1];
                            w[pp] = (i & 1) ? pack_hi(a, bb) : pack_lo(a, bb);
                        }
                        const int r = mb * 8 + i;
                        *(uint4 *)(tile + lds_off(r, kb)) = make_uint4(w[0], w[1], w[2], w[3]);
                    }
                }
            }
        }
    }
};

