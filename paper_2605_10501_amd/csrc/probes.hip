// Measurement probes (not on the section path): the matrix-core rate the chip sustains in a register-resident loop,
// and a clock monitor that reports the shader clock granted while other kernels run.
#include <type_traits>

#include "common.h"

namespace {
template <bool M16>
__global__ __launch_bounds__(512) void mfma_probe_kernel(int iters, int random_operands, float *sink) {
    // the same flops per iteration for both shapes: 8 x 32x32x16 or 16 x 16x16x32, all independent
    constexpr int NACC = M16 ? 16 : 8, ACC_N = M16 ? 4 : 16;
    std::conditional_t<M16, f32x4, f32x16> acc[NACC];
#pragma unroll
    for (int i = 0; i < NACC; ++i)
#pragma unroll
        for (int r = 0; r < ACC_N; ++r) acc[i][r] = 0.f;
    bf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) { a[e] = (bf16_t)(float)(threadIdx.x & 3); b[e] = (bf16_t)(1.f / 64.f); }
    if (random_operands) {
        // random sign and mantissa, magnitudes 2^-4 .. 2^4: the bit activity of real activations and weights,
        // which is what the chip's power management reacts to
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            unsigned h = (threadIdx.x * 8u + e) * 2654435761u + blockIdx.x * 40503u;
            h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
            unsigned g = h * 2654435761u + 12345u;
            g ^= g >> 16; g *= 2246822519u; g ^= g >> 13;
            a[e] = __builtin_bit_cast(bf16_t, (unsigned short)(((h & 1) << 15) | ((123 + ((h >> 1) & 7)) << 7) | ((h >> 4) & 127)));
            b[e] = __builtin_bit_cast(bf16_t, (unsigned short)(((g & 1) << 15) | ((123 + ((g >> 1) & 7)) << 7) | ((g >> 4) & 127)));
        }
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < NACC; ++i) {
            if constexpr (M16) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[i], 0, 0, 0);
            else acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
        }
    }
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < NACC; ++i)
#pragma unroll
        for (int r = 0; r < ACC_N; ++r) t += acc[i][r];
    sink[(long)blockIdx.x * 512 + threadIdx.x] = t;
}

// One wave that watches the clocks for a given time while other kernels run: the shader-clock counter
// (s_memtime) against the constant 100 MHz counter (s_memrealtime).  Ends after `ticks_100mhz` of the constant
// counter or after max_polls polls, whichever comes first.
__global__ __launch_bounds__(64) void clock_monitor_kernel(long ticks_100mhz, long max_polls, long long *out) {
    const long long c0 = clock64(), w0 = wall_clock64();
    long long w1 = w0;
    for (long i = 0; i < max_polls && w1 - w0 < ticks_100mhz; ++i) {
        __builtin_amdgcn_s_sleep(64);
        w1 = wall_clock64();
    }
    const long long c1 = clock64();
    w1 = wall_clock64();
    if (threadIdx.x == 0) { out[0] = c1 - c0; out[1] = w1 - w0; }
}
}  // namespace

extern "C" ms_status ms_k_clock_monitor(int32_t microseconds, int64_t *out_dev, void *stream) {
    if (microseconds <= 0 || microseconds > 1000000 || !out_dev) return ms_fail(MS_ERR_INVALID_ARG, "clock_monitor: bad argument");
    // a poll takes at least the 64 x 64 clocks of its sleep (> 1.5 us at any clock this chip runs at)
    clock_monitor_kernel<<<1, 64, 0, (hipStream_t)stream>>>(100L * microseconds, 2L * microseconds + 1000, (long long *)out_dev);
    MS_LAUNCH_CHECK();
    return MS_OK;
}

extern "C" ms_status ms_k_mfma_probe(int32_t workgroups, int32_t iters, int32_t random_operands, int32_t mfma16, float *sink_dev,
                                     void *stream) {
    if (workgroups <= 0 || iters <= 0 || !sink_dev) return ms_fail(MS_ERR_INVALID_ARG, "mfma_probe: bad argument");
    if (mfma16) mfma_probe_kernel<true><<<workgroups, 512, 0, (hipStream_t)stream>>>(iters, random_operands, sink_dev);
    else mfma_probe_kernel<false><<<workgroups, 512, 0, (hipStream_t)stream>>>(iters, random_operands, sink_dev);
    MS_LAUNCH_CHECK();
    return MS_OK;
}
