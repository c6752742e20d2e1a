// Shared declarations of the HIP section-compute library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "maestro_section.h"
#include "maestro_kernels.h"

typedef __bf16 bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// ---- host-side error plumbing -------------------------------------------------------
ms_status ms_fail(ms_status code, const char *fmt, ...);
#define MS_CHECK_HIP(expr)                                                                 \
    do {                                                                                   \
        hipError_t e_ = (expr);                                                            \
        if (e_ != hipSuccess)                                                              \
            return ms_fail(MS_ERR_HIP, "%s: %s (%s:%d)", #expr, hipGetErrorString(e_),     \
                           __FILE__, __LINE__);                                            \
    } while (0)
#define MS_TRY(expr)                                                                       \
    do {                                                                                   \
        ms_status s_ = (expr);                                                             \
        if (s_ != MS_OK) return s_;                                                        \
    } while (0)
#define MS_LAUNCH_CHECK() MS_CHECK_HIP(hipGetLastError())

static inline size_t ms_align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }
static inline int ms_cdiv(long a, long b) { return (int)((a + b - 1) / b); }
static inline size_t ms_dtype_size(int dtype) { return dtype == MS_BF16 ? 2 : 4; }

// Shape limits of the kernels, in one place so that a section call can check them before its first launch.
constexpr int kNormMaxCache = 8;   // 16-byte vectors of a row that a lane of the norm kernels keeps in registers
static inline int ms_norm_backward_max_d(int dtype) { return 64 * kNormMaxCache * (dtype == MS_BF16 ? 8 : 4); }
// the matrix-core attention kernels address qkv through 32-bit byte offsets
static inline bool ms_attn_offsets_fit(long n, int nq, int nkv, int hd) {
    return n * (nq + 2 * nkv) * hd * 2 < (1L << 32) - (1L << 20);
}

// Linear carve-out of the caller's workspace; every piece 256-byte aligned.  A null base only counts bytes (the
// workspace-size queries) and hands out null pointers.
struct Arena {
    char *base;
    size_t off;
    explicit Arena(void *p) : base((char *)p), off(0) {}
    template <class T = void>
    T *take(size_t bytes) {
        T *p = base ? (T *)(base + off) : nullptr;
        off += ms_align_up(bytes);
        return p;
    }
};

// ---- device helpers -----------------------------------------------------------------
#ifdef __HIPCC__
template <class T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<bf16_t>(bf16_t v) { return (float)v; }
template <class T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }

// 16-byte vector of T: 8 bf16 or 4 fp32.
template <class T> struct Vec16 {
    static constexpr int N = 16 / sizeof(T);
    T v[N];
};
template <class T> __device__ __forceinline__ Vec16<T> ldv(const T *p) {
    Vec16<T> r;
    *(uint4 *)&r = *(const uint4 *)p;
    return r;
}
template <class T> __device__ __forceinline__ void stv(T *p, const Vec16<T> &r) {
    *(uint4 *)p = *(const uint4 *)&r;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
#endif
