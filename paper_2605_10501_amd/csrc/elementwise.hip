// HBM-bound kernels of the section path: norms, rotary embedding, activations, embedding,
// column sums, fills and conversions.  Every kernel moves 16-byte vectors per lane, does its
// arithmetic in fp32 and touches each element once; rows are reduced with wave shuffles.
#include "common.h"
#include "launch.h"

namespace {

constexpr int kMaxCache = kNormMaxCache;   // 16-byte vectors a lane keeps in registers per row
constexpr int kPartialRows = 1024; // rows of the partial-sum scratch of column reductions

// ------------------------------------------------------------------ norm forward
// TX is the type of the normalised input (the residual stream: fp32 even for bf16 sections),
// T the type of gains, shifts and of the output.  A lane handles V = 16 / sizeof(T) columns at a time.
template <class TX, int V> __device__ __forceinline__ void load_row_vec(const TX *p, float *out) {
    if constexpr (sizeof(TX) == 4) {
#pragma unroll
        for (int q = 0; q < V / 4; ++q) {
            const float4 t = *(const float4 *)(p + 4 * q);
            out[4 * q] = t.x; out[4 * q + 1] = t.y; out[4 * q + 2] = t.z; out[4 * q + 3] = t.w;
        }
    } else {
        const Vec16<TX> t = ldv(p);
#pragma unroll
        for (int e = 0; e < V; ++e) out[e] = to_f32(t.v[e]);
    }
}

// NC = 16-byte vectors of the row that a lane keeps in registers (1, 2, 4 or kMaxCache; the caller picks the
// smallest that covers the row, which keeps the register count and with it the occupancy right for each width).
template <class T, class TX, int KIND, int NC>
__global__ __launch_bounds__(256) void norm_fwd_kernel(const TX *__restrict__ x, const T *__restrict__ g,
                                                        const T *__restrict__ b, T *__restrict__ y,
                                                        float *__restrict__ mean, float *__restrict__ rstd,
                                                        int n, int d, float eps) {
    constexpr int V = Vec16<T>::N;
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= n) return;
    const TX *xr = x + (size_t)row * d;
    T *yr = y + (size_t)row * d;
    const int nvec = d / V;
    float cache[NC][V];
    float s = 0.f, ss = 0.f;
#pragma unroll
    for (int i = 0; i < NC; ++i) {
        int idx = lane + 64 * i;
        if (idx < nvec) {
            load_row_vec<TX, V>(xr + (size_t)idx * V, cache[i]);
#pragma unroll
            for (int e = 0; e < V; ++e) {
                s += cache[i][e];
                ss += cache[i][e] * cache[i][e];
            }
        }
    }
    for (int idx = lane + 64 * NC; idx < nvec; idx += 64) {
        float t[V];
        load_row_vec<TX, V>(xr + (size_t)idx * V, t);
#pragma unroll
        for (int e = 0; e < V; ++e) {
            s += t[e];
            ss += t[e] * t[e];
        }
    }
    float mu = 0.f, var;
    if (KIND == 1) {
        mu = wave_sum(s) / d;
        float sq = 0.f;  // second pass over the cached row: sum (x - mu)^2
#pragma unroll
        for (int i = 0; i < NC; ++i) {
            int idx = lane + 64 * i;
            if (idx < nvec) {
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    float f = cache[i][e] - mu;
                    sq += f * f;
                }
            }
        }
        for (int idx = lane + 64 * NC; idx < nvec; idx += 64) {
            float t[V];
            load_row_vec<TX, V>(xr + (size_t)idx * V, t);
#pragma unroll
            for (int e = 0; e < V; ++e) {
                float f = t[e] - mu;
                sq += f * f;
            }
        }
        var = wave_sum(sq) / d;
    } else {
        var = wave_sum(ss) / d;
    }
    const float r = rsqrtf(var + eps);
    if (lane == 0) {
        rstd[row] = r;
        if (KIND == 1) mean[row] = mu;
    }
    auto emit = [&](int idx, const float *xv) {
        Vec16<T> gv = ldv(g + (size_t)idx * V), bv, out;
        if (KIND == 1) bv = ldv(b + (size_t)idx * V);
#pragma unroll
        for (int e = 0; e < V; ++e) {
            float f = (xv[e] - mu) * r * to_f32(gv.v[e]);
            if (KIND == 1) f += to_f32(bv.v[e]);
            out.v[e] = from_f32<T>(f);
        }
        stv(yr + (size_t)idx * V, out);
    };
#pragma unroll
    for (int i = 0; i < NC; ++i) {
        int idx = lane + 64 * i;
        if (idx < nvec) emit(idx, cache[i]);
    }
    for (int idx = lane + 64 * NC; idx < nvec; idx += 64) {
        float t[V];
        load_row_vec<TX, V>(xr + (size_t)idx * V, t);
        emit(idx, t);
    }
}

// ------------------------------------------------------------------ norm backward
// One wave per row, rows strided over the grid; each lane keeps the dg (and db) sums of its
// columns in registers; the four waves of a workgroup add theirs up through LDS and write one
// partial row per workgroup.  NC as in the forward kernel.
template <class T, class TX, int KIND, int NC>
__global__ __launch_bounds__(256) void norm_bwd_kernel(const T *__restrict__ dy, const TX *__restrict__ x,
                                                        const T *__restrict__ g, const float *__restrict__ mean,
                                                        const float *__restrict__ rstd, const T *__restrict__ add,
                                                        T *__restrict__ dx, float *__restrict__ part_g,
                                                        float *__restrict__ part_b, int n, int d) {
    constexpr int V = Vec16<T>::N;
    __shared__ float red[3][64 * NC * V];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int w = blockIdx.x * 4 + wv;
    const int nw = gridDim.x * 4;
    const int nvec = d / V;
    float accg[NC][V], accb[KIND == 1 ? NC : 1][V];
    Vec16<T> gv[NC];
#pragma unroll
    for (int i = 0; i < NC; ++i) {
        int idx = lane + 64 * i;
        if (idx < nvec) gv[i] = ldv(g + (size_t)idx * V);
#pragma unroll
        for (int e = 0; e < V; ++e) {
            accg[i][e] = 0.f;
            if constexpr (KIND == 1) accb[i][e] = 0.f;
        }
    }
    for (int row = w; row < n; row += nw) {
        const size_t ro = (size_t)row * d;
        const float r = rstd[row];
        const float mu = KIND == 1 ? mean[row] : 0.f;
        float xh[NC][V];
        Vec16<T> dv[NC];
        float c1 = 0.f, c2 = 0.f;
#pragma unroll
        for (int i = 0; i < NC; ++i) {
            int idx = lane + 64 * i;
            if (idx < nvec) {
                load_row_vec<TX, V>(x + ro + (size_t)idx * V, xh[i]);
                dv[i] = ldv(dy + ro + (size_t)idx * V);
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    xh[i][e] = (xh[i][e] - mu) * r;
                    float dyv = to_f32(dv[i].v[e]);
                    float t = dyv * to_f32(gv[i].v[e]);
                    c1 += t * xh[i][e];
                    c2 += t;
                    accg[i][e] += dyv * xh[i][e];
                    if constexpr (KIND == 1) accb[i][e] += dyv;
                }
            }
        }
        c1 = wave_sum(c1) / d;
        c2 = KIND == 1 ? wave_sum(c2) / d : 0.f;
#pragma unroll
        for (int i = 0; i < NC; ++i) {
            int idx = lane + 64 * i;
            if (idx < nvec) {
                Vec16<T> av, out;
                if (add) av = ldv(add + ro + (size_t)idx * V);
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    float t = to_f32(dv[i].v[e]) * to_f32(gv[i].v[e]);
                    float f = r * (t - c2 - xh[i][e] * c1);
                    if (add) f += to_f32(av.v[e]);
                    out.v[e] = from_f32<T>(f);
                }
                stv(dx + ro + (size_t)idx * V, out);
            }
        }
    }
    // waves 1..3 park their sums in LDS, wave 0 adds them and writes the workgroup's partial row
    auto reduce_and_store = [&](float (*acc)[V], float *part) {
        if (wv > 0) {
#pragma unroll
            for (int i = 0; i < NC; ++i)
#pragma unroll
                for (int e = 0; e < V; ++e) red[wv - 1][(i * V + e) * 64 + lane] = acc[i][e];
        }
        __syncthreads();
        if (wv == 0) {
#pragma unroll
            for (int i = 0; i < NC; ++i) {
                int idx = lane + 64 * i;
                if (idx < nvec) {
#pragma unroll
                    for (int e = 0; e < V; ++e) {
                        const int k = (i * V + e) * 64 + lane;
                        part[(size_t)blockIdx.x * d + idx * V + e] = acc[i][e] + red[0][k] + red[1][k] + red[2][k];
                    }
                }
            }
        }
        __syncthreads();
    };
    reduce_and_store(accg, part_g);
    if constexpr (KIND == 1) reduce_and_store(accb, part_b);
}

// out[j] += sum_p part[p, j]; block = 32 columns x 32 row lanes (many short dependent-load chains
// instead of a few long ones: the partial matrix is small and the kernel is latency-bound).
__global__ __launch_bounds__(1024) void reduce_partials_kernel(const float *__restrict__ part, int np, int c,
                                                                float *__restrict__ out) {
    __shared__ float sm[32][33];
    const int cl = threadIdx.x & 31, pl = threadIdx.x >> 5;
    const int col = blockIdx.x * 32 + cl;
    float s = 0.f;
    if (col < c)
        for (int p = pl; p < np; p += 32) s += part[(size_t)p * c + col];
    sm[pl][cl] = s;
    __syncthreads();
    if (pl == 0 && col < c) {
        float t = 0.f;
#pragma unroll
        for (int i = 0; i < 32; ++i) t += sm[i][cl];
        out[col] += t;
    }
}

// partial column sums: lane <-> one 16-byte column vector, waves stride over rows.
template <class T>
__global__ __launch_bounds__(256) void colsum_partial_kernel(const T *__restrict__ x, int n, int c,
                                                              float *__restrict__ part) {
    constexpr int V = Vec16<T>::N;
    const int cv = blockIdx.x * 64 + (threadIdx.x & 63);
    const int w = blockIdx.y * 4 + (threadIdx.x >> 6);
    const int nw = gridDim.y * 4;
    if (cv * V >= c) return;
    float acc[V];
#pragma unroll
    for (int e = 0; e < V; ++e) acc[e] = 0.f;
    for (int row = w; row < n; row += nw) {
        Vec16<T> t = ldv(x + (size_t)row * c + (size_t)cv * V);
#pragma unroll
        for (int e = 0; e < V; ++e) acc[e] += to_f32(t.v[e]);
    }
#pragma unroll
    for (int e = 0; e < V; ++e) part[(size_t)w * c + cv * V + e] = acc[e];
}

// ------------------------------------------------------------------ rotary embedding
__global__ void positions_kernel(int n, int n_seqs, const int *__restrict__ cu, int *__restrict__ pos) {
    int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n) return;
    int lo = 0, hi = n_seqs;  // largest b with cu[b] <= t
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (cu[mid] <= t) lo = mid; else hi = mid;
    }
    pos[t] = t - cu[lo];
}

__global__ void rope_table_kernel(int max_pos, int half, int hd, double base, float2 *__restrict__ table) {
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= max_pos * half) return;
    int p = idx / half, i = idx % half;
    double ang = (double)p * pow(base, -2.0 * (double)i / (double)hd);
    table[idx] = make_float2((float)cos(ang), (float)sin(ang));
}

template <class T>
__global__ __launch_bounds__(256) void rope_kernel(T *__restrict__ x, const int *__restrict__ pos,
                                                   const float2 *__restrict__ table, long total, int n_heads,
                                                   int hd, long row_stride, float sign) {
    constexpr int V = Vec16<T>::N;
    const int half = hd / 2, vph = half / V;
    long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    int iv = idx % vph;
    long th = idx / vph;
    int h = th % n_heads;
    long t = th / n_heads;
    T *p = x + t * row_stride + (long)h * hd + iv * V;
    const float2 *cs = table + (long)pos[t] * half + iv * V;
    Vec16<T> lo = ldv(p), hi = ldv(p + half), olo, ohi;
#pragma unroll
    for (int e = 0; e < V; ++e) {
        float c = cs[e].x, s = sign * cs[e].y;
        float a = to_f32(lo.v[e]), b = to_f32(hi.v[e]);
        olo.v[e] = from_f32<T>(a * c - b * s);
        ohi.v[e] = from_f32<T>(b * c + a * s);
    }
    stv(p, olo);
    stv(p + half, ohi);
}

// ------------------------------------------------------------------ activations
template <class T, int KIND>
__global__ __launch_bounds__(256) void act_fwd_kernel(const T *__restrict__ up, T *__restrict__ a, long nvec_total,
                                                      int f) {
    constexpr int V = Vec16<T>::N;
    long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= nvec_total) return;
    const int vpr = f / V;
    long row = idx / vpr;
    int cv = idx % vpr;
    Vec16<T> out;
    if (KIND == 0) {
        const T *base = up + row * 2 * f + (long)cv * V;
        Vec16<T> gv = ldv(base), uv = ldv(base + f);
#pragma unroll
        for (int e = 0; e < V; ++e) {
            float gg = to_f32(gv.v[e]);
            out.v[e] = from_f32<T>(gg / (1.f + __expf(-gg)) * to_f32(uv.v[e]));
        }
    } else {
        Vec16<T> xv = ldv(up + row * f + (long)cv * V);
#pragma unroll
        for (int e = 0; e < V; ++e) {
            float xx = to_f32(xv.v[e]);
            out.v[e] = from_f32<T>(0.5f * xx * (1.f + erff(xx * 0.70710678118654752f)));
        }
    }
    stv(a + row * f + (long)cv * V, out);
}

template <class T, int KIND>
__global__ __launch_bounds__(256) void act_bwd_kernel(const T *__restrict__ da, const T *__restrict__ up,
                                                      T *__restrict__ dup, long nvec_total, int f) {
    constexpr int V = Vec16<T>::N;
    long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= nvec_total) return;
    const int vpr = f / V;
    long row = idx / vpr;
    int cv = idx % vpr;
    Vec16<T> dav = ldv(da + row * f + (long)cv * V);
    if (KIND == 0) {
        const T *base = up + row * 2 * f + (long)cv * V;
        Vec16<T> gv = ldv(base), uv = ldv(base + f), dg, du;
#pragma unroll
        for (int e = 0; e < V; ++e) {
            float gg = to_f32(gv.v[e]), uu = to_f32(uv.v[e]), d = to_f32(dav.v[e]);
            float s = 1.f / (1.f + __expf(-gg));
            dg.v[e] = from_f32<T>(d * uu * s * (1.f + gg * (1.f - s)));
            du.v[e] = from_f32<T>(d * gg * s);
        }
        T *ob = dup + row * 2 * f + (long)cv * V;
        stv(ob, dg);
        stv(ob + f, du);
    } else {
        Vec16<T> xv = ldv(up + row * f + (long)cv * V), out;
#pragma unroll
        for (int e = 0; e < V; ++e) {
            float xx = to_f32(xv.v[e]);
            float cdf = 0.5f * (1.f + erff(xx * 0.70710678118654752f));
            float pdf = 0.3989422804014327f * __expf(-0.5f * xx * xx);
            out.v[e] = from_f32<T>(to_f32(dav.v[e]) * (cdf + xx * pdf));
        }
        stv(dup + row * f + (long)cv * V, out);
    }
}

// ------------------------------------------------------------------ embedding
template <class T, class TO>
__global__ __launch_bounds__(256) void embedding_fwd_kernel(const int *__restrict__ ids, const T *__restrict__ table,
                                                            TO *__restrict__ x, long nvec_total, int d, int vocab) {
    constexpr int V = Vec16<T>::N;
    long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= nvec_total) return;
    const int vpr = d / V;
    long t = idx / vpr;
    int cv = idx % vpr;
    const int id = ids[t];
    Vec16<T> v;
    if ((unsigned)id < (unsigned)vocab) v = ldv(table + (long)id * d + (long)cv * V);
    else                                  // an id outside the table embeds as zeros: never an out-of-bounds read
#pragma unroll
        for (int e = 0; e < V; ++e) v.v[e] = from_f32<T>(0.f);
    TO *o = x + t * d + (long)cv * V;
    if constexpr (sizeof(TO) == sizeof(T)) {
        stv(o, v);
    } else {
#pragma unroll
        for (int q = 0; q < V / 4; ++q)
            *(float4 *)(o + 4 * q) = make_float4(to_f32(v.v[4 * q]), to_f32(v.v[4 * q + 1]), to_f32(v.v[4 * q + 2]), to_f32(v.v[4 * q + 3]));
    }
}

// one workgroup per token; consecutive lanes add to consecutive floats, so that one atomic instruction
// touches 256 contiguous bytes of the table row
template <class T>
__global__ __launch_bounds__(256) void embedding_bwd_kernel(const int *__restrict__ ids, const T *__restrict__ dx,
                                                            float *__restrict__ dtab, int d, int vocab) {
    const long t = blockIdx.x;
    const T *src = dx + t * d;
    const int id = ids[t];
    if ((unsigned)id >= (unsigned)vocab) return;   // an id outside the table receives no gradient
    float *o = dtab + (long)id * d;
    for (int c = threadIdx.x; c < d; c += 256) unsafeAtomicAdd(o + c, to_f32(src[c]));
}

// ------------------------------------------------------------------ fills / conversions
__global__ void fill_f32_kernel(float *p, long n, float v) {
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    long stride = (long)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = v;
}

__global__ void convert_bf16_to_f32_kernel(const bf16_t *__restrict__ src, float *__restrict__ dst, long n) {
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    long stride = (long)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = (float)src[i];
}

template <class T>
__global__ void convert_from_f32_kernel(const float *__restrict__ src, T *__restrict__ dst, long n) {
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    long stride = (long)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = from_f32<T>(src[i]);
}

// Reference copy (measurements only).  The configuration is the best of a sweep on MI355X over grid-stride and
// chunked indexing, 256 / 512 / 1024 threads, 1 / 4 / 8 loads in flight per thread and cache policies (5.6-6.0 TB/s
// read+write against 5.0 for the runtime's device-to-device copy): each workgroup owns a contiguous chunk, 1024
// threads, four 16-byte non-temporal loads in flight per thread before their stores.
typedef unsigned int copy_u32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(1024) void copy_kernel(const copy_u32x4 *__restrict__ src, copy_u32x4 *__restrict__ dst, long nvec) {
    const long per = (nvec + gridDim.x - 1) / gridDim.x;
    const long b = (long)blockIdx.x * per, e = b + per < nvec ? b + per : nvec;
    long i = b + threadIdx.x;
    for (; i + 3 * 1024 < e; i += 4 * 1024) {
        copy_u32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(src + i + u * 1024);
#pragma unroll
        for (int u = 0; u < 4; ++u) __builtin_nontemporal_store(v[u], dst + i + u * 1024);
    }
    for (; i < e; i += 1024) dst[i] = src[i];
}

template <class T> constexpr int vec_of() { return 16 / sizeof(T); }

}  // namespace

// ===================================================================== host launchers
#define DISPATCH_T(dtype, ...)                                  \
    if ((dtype) == MS_BF16) { using T = bf16_t; __VA_ARGS__; }  \
    else { using T = float; __VA_ARGS__; }

static bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }

extern "C" ms_status ms_k_norm_forward(int32_t kind, int32_t dtype, int32_t x_fp32, int32_t n, int32_t d, float eps,
                                       const void *x, const void *g, const void *b, void *y, float *mean,
                                       float *rstd, void *stream) {
    if (n == 0) return MS_OK;
    if (!x || !g || !y || !rstd || (kind == 1 && (!b || !mean)) || n < 0 || d <= 0)
        return ms_fail(MS_ERR_INVALID_ARG, "norm_forward: null pointer or bad size");
    const int V = dtype == MS_BF16 ? 8 : 4;
    if (d % V || !aligned16(x) || !aligned16(y) || !aligned16(g))
        return ms_fail(MS_ERR_UNSUPPORTED, "norm_forward: d=%d must be a multiple of %d and rows 16-byte aligned", d, V);
    hipStream_t s = (hipStream_t)stream;
    const bool xf = x_fp32 || dtype == MS_F32;
    ProfScope ps(4, (double)n * d * ((xf ? 4 : 2) + (dtype == MS_BF16 ? 2 : 4)), s);
    const int nc = ms_cdiv(d / (dtype == MS_BF16 ? 8 : 4), 64);
#define NORM_FWD_NC(T, TX, K, NC) norm_fwd_kernel<T, TX, K, NC><<<ms_cdiv(n, 4), 256, 0, s>>>((const TX *)x, (const T *)g, (const T *)b, (T *)y, mean, rstd, n, d, eps)
#define NORM_FWD(T, TX, K)                                   \
    do {                                                     \
        if (nc <= 1) NORM_FWD_NC(T, TX, K, 1);               \
        else if (nc <= 2) NORM_FWD_NC(T, TX, K, 2);          \
        else if (nc <= 4) NORM_FWD_NC(T, TX, K, 4);          \
        else NORM_FWD_NC(T, TX, K, kMaxCache);               \
    } while (0)
    if (dtype == MS_F32) { if (kind == 1) NORM_FWD(float, float, 1); else NORM_FWD(float, float, 0); }
    else if (xf) { if (kind == 1) NORM_FWD(bf16_t, float, 1); else NORM_FWD(bf16_t, float, 0); }
    else { if (kind == 1) NORM_FWD(bf16_t, bf16_t, 1); else NORM_FWD(bf16_t, bf16_t, 0); }
#undef NORM_FWD
#undef NORM_FWD_NC
    MS_LAUNCH_CHECK();
    return MS_OK;
}

extern "C" size_t ms_k_norm_backward_scratch_bytes(int32_t d) {
    return d > 0 ? 2 * ms_align_up((size_t)kPartialRows * d * sizeof(float)) : 0;
}

static ms_status reduce_partials(const float *part, int np, int c, float *out, hipStream_t s) {
    reduce_partials_kernel<<<ms_cdiv(c, 32), 1024, 0, s>>>(part, np, c, out);
    MS_LAUNCH_CHECK();
    return MS_OK;
}

extern "C" ms_status ms_k_norm_backward(int32_t kind, int32_t dtype, int32_t x_fp32, int32_t n, int32_t d,
                                        const void *dy, const void *x, const void *g, const float *mean, const float *rstd,
                                        const void *add, void *dx, float *dg, float *db, void *scratch,
                                        void *stream) {
    if (n == 0) return MS_OK;
    if (!dy || !x || !g || !rstd || !dx || !dg || !scratch || (kind == 1 && (!mean || !db)) || n < 0 || d <= 0)
        return ms_fail(MS_ERR_INVALID_ARG, "norm_backward: null pointer or bad size");
    const int V = dtype == MS_BF16 ? 8 : 4;
    if (d % V || d > ms_norm_backward_max_d(dtype))
        return ms_fail(MS_ERR_UNSUPPORTED, "norm_backward: d=%d must be a multiple of %d and at most %d", d, V,
                       ms_norm_backward_max_d(dtype));
    hipStream_t s = (hipStream_t)stream;
    float *pg = (float *)scratch;
    float *pb = (float *)((char *)scratch + ms_align_up((size_t)kPartialRows * d * sizeof(float)));
    const int grid = n / 4 < 1 ? 1 : (n / 4 > kPartialRows ? kPartialRows : n / 4);   // one partial row per workgroup
    const int nc = ms_cdiv(d / V, 64);
    {
    const bool xf = x_fp32 || dtype == MS_F32;
    const double es = dtype == MS_BF16 ? 2 : 4;
    ProfScope ps(5, (double)n * d * ((xf ? 4 : 2) + (add ? 3.0 : 2.0) * es), s);
#define NORM_BWD_NC(T, TX, K, NC) norm_bwd_kernel<T, TX, K, NC><<<grid, 256, 0, s>>>((const T *)dy, (const TX *)x, (const T *)g, mean, rstd, (const T *)add, (T *)dx, pg, pb, n, d)
#define NORM_BWD(T, TX, K)                                   \
    do {                                                     \
        if (nc <= 1) NORM_BWD_NC(T, TX, K, 1);               \
        else if (nc <= 2) NORM_BWD_NC(T, TX, K, 2);          \
        else if (nc <= 4) NORM_BWD_NC(T, TX, K, 4);          \
        else NORM_BWD_NC(T, TX, K, kMaxCache);               \
    } while (0)
    if (dtype == MS_F32) { if (kind == 1) NORM_BWD(float, float, 1); else NORM_BWD(float, float, 0); }
    else if (xf) { if (kind == 1) NORM_BWD(bf16_t, float, 1); else NORM_BWD(bf16_t, float, 0); }
    else { if (kind == 1) NORM_BWD(bf16_t, bf16_t, 1); else NORM_BWD(bf16_t, bf16_t, 0); }
#undef NORM_BWD
#undef NORM_BWD_NC
    }
    MS_LAUNCH_CHECK();
    MS_TRY(reduce_partials(pg, grid, d, dg, s));
    if (kind == 1) MS_TRY(reduce_partials(pb, grid, d, db, s));
    return MS_OK;
}

extern "C" ms_status ms_k_colsum(int32_t dtype, int32_t n, int32_t c, const void *x, float *out, void *scratch,
                                 void *stream) {
    if (n == 0) return MS_OK;
    if (!x || !out || !scratch || n < 0 || c <= 0) return ms_fail(MS_ERR_INVALID_ARG, "colsum: null pointer or bad size");
    const int V = dtype == MS_BF16 ? 8 : 4;
    if (c % V) return ms_fail(MS_ERR_UNSUPPORTED, "colsum: c=%d must be a multiple of %d", c, V);
    hipStream_t s = (hipStream_t)stream;
    const int gy = n / 16 < 1 ? 1 : (n / 16 > kPartialRows / 4 ? kPartialRows / 4 : n / 16);
    dim3 grid(ms_cdiv(c / V, 64), gy);
    DISPATCH_T(dtype, { colsum_partial_kernel<T><<<grid, 256, 0, s>>>((const T *)x, n, c, (float *)scratch); });
    MS_LAUNCH_CHECK();
    return reduce_partials((const float *)scratch, gy * 4, c, out, s);
}

extern "C" ms_status ms_k_positions(int32_t n_tokens, int32_t n_seqs, const int32_t *cu, int32_t *pos, void *stream) {
    if (n_tokens == 0) return MS_OK;
    if (!cu || !pos || n_seqs <= 0 || n_tokens < 0) return ms_fail(MS_ERR_INVALID_ARG, "positions: bad argument");
    positions_kernel<<<ms_cdiv(n_tokens, 256), 256, 0, (hipStream_t)stream>>>(n_tokens, n_seqs, cu, pos);
    MS_LAUNCH_CHECK();
    return MS_OK;
}

extern "C" ms_status ms_k_rope_table(int32_t max_pos, int32_t head_dim, float base, float *table, void *stream) {
    if (max_pos == 0) return MS_OK;
    if (!table || max_pos < 0 || head_dim <= 0 || head_dim % 2) return ms_fail(MS_ERR_INVALID_ARG, "rope_table: bad argument");
    const int half = head_dim / 2;
    rope_table_kernel<<<ms_cdiv((long)max_pos * half, 256), 256, 0, (hipStream_t)stream>>>(max_pos, half, head_dim, (double)base, (float2 *)table);
    MS_LAUNCH_CHECK();
    return MS_OK;
}

extern "C" ms_status ms_k_rope(int32_t dtype, int32_t n, int32_t n_heads, int32_t head_dim, int64_t row_stride, void *x,
                               const int32_t *pos, const float *table, int32_t inverse, void *stream) {
    if (n == 0 || n_heads == 0) return MS_OK;
    if (!x || !pos || !table || n < 0 || n_heads < 0) return ms_fail(MS_ERR_INVALID_ARG, "rope: bad argument");
    const int V = dtype == MS_BF16 ? 8 : 4;
    if (head_dim % (2 * V) || row_stride % V || !aligned16(x))
        return ms_fail(MS_ERR_UNSUPPORTED, "rope: head_dim=%d must be a multiple of %d", head_dim, 2 * V);
    const long total = (long)n * n_heads * (head_dim / 2 / V);
    ProfScope ps(8, 2.0 * n * n_heads * head_dim * (dtype == MS_BF16 ? 2 : 4), (hipStream_t)stream);
    DISPATCH_T(dtype, {
        rope_kernel<T><<<ms_cdiv(total, 256), 256, 0, (hipStream_t)stream>>>((T *)x, pos, (const float2 *)table, total, n_heads, head_dim, row_stride, inverse ? -1.f : 1.f);
    });
    MS_LAUNCH_CHECK();
    return MS_OK;
}

extern "C" ms_status ms_k_act_forward(int32_t kind, int32_t dtype, int32_t n, int32_t f, const void *up, void *a, void *stream) {
    if (n == 0) return MS_OK;
    if (!up || !a || n < 0 || f <= 0) return ms_fail(MS_ERR_INVALID_ARG, "act_forward: bad argument");
    const int V = dtype == MS_BF16 ? 8 : 4;
    if (f % V) return ms_fail(MS_ERR_UNSUPPORTED, "act_forward: f=%d must be a multiple of %d", f, V);
    const long total = (long)n * (f / V);
    hipStream_t s = (hipStream_t)stream;
    ProfScope ps(6, (kind == 0 ? 3.0 : 2.0) * n * f * (dtype == MS_BF16 ? 2 : 4), s);
    DISPATCH_T(dtype, {
        if (kind == 0) act_fwd_kernel<T, 0><<<ms_cdiv(total, 256), 256, 0, s>>>((const T *)up, (T *)a, total, f);
        else act_fwd_kernel<T, 1><<<ms_cdiv(total, 256), 256, 0, s>>>((const T *)up, (T *)a, total, f);
    });
    MS_LAUNCH_CHECK();
    return MS_OK;
}

extern "C" ms_status ms_k_act_backward(int32_t kind, int32_t dtype, int32_t n, int32_t f, const void *da, const void *up,
                                       void *dup, void *stream) {
    if (n == 0) return MS_OK;
    if (!da || !up || !dup || n < 0 || f <= 0) return ms_fail(MS_ERR_INVALID_ARG, "act_backward: bad argument");
    const int V = dtype == MS_BF16 ? 8 : 4;
    if (f % V) return ms_fail(MS_ERR_UNSUPPORTED, "act_backward: f=%d must be a multiple of %d", f, V);
    const long total = (long)n * (f / V);
    hipStream_t s = (hipStream_t)stream;
    ProfScope ps(7, (kind == 0 ? 5.0 : 3.0) * n * f * (dtype == MS_BF16 ? 2 : 4), s);
    DISPATCH_T(dtype, {
        if (kind == 0) act_bwd_kernel<T, 0><<<ms_cdiv(total, 256), 256, 0, s>>>((const T *)da, (const T *)up, (T *)dup, total, f);
        else act_bwd_kernel<T, 1><<<ms_cdiv(total, 256), 256, 0, s>>>((const T *)da, (const T *)up, (T *)dup, total, f);
    });
    MS_LAUNCH_CHECK();
    return MS_OK;
}

extern "C" ms_status ms_k_embedding_forward(int32_t dtype, int32_t out_fp32, int32_t n, int32_t d, int32_t vocab,
                                            const int32_t *ids, const void *table, void *x, void *stream) {
    if (n == 0) return MS_OK;
    if (!ids || !table || !x || n < 0 || d <= 0 || vocab <= 0) return ms_fail(MS_ERR_INVALID_ARG, "embedding_forward: bad argument");
    const int V = dtype == MS_BF16 ? 8 : 4;
    if (d % V) return ms_fail(MS_ERR_UNSUPPORTED, "embedding: d=%d must be a multiple of %d", d, V);
    const long total = (long)n * (d / V);
    hipStream_t s = (hipStream_t)stream;
    if (dtype == MS_F32) embedding_fwd_kernel<float, float><<<ms_cdiv(total, 256), 256, 0, s>>>(ids, (const float *)table, (float *)x, total, d, vocab);
    else if (out_fp32) embedding_fwd_kernel<bf16_t, float><<<ms_cdiv(total, 256), 256, 0, s>>>(ids, (const bf16_t *)table, (float *)x, total, d, vocab);
    else embedding_fwd_kernel<bf16_t, bf16_t><<<ms_cdiv(total, 256), 256, 0, s>>>(ids, (const bf16_t *)table, (bf16_t *)x, total, d, vocab);
    MS_LAUNCH_CHECK();
    return MS_OK;
}

extern "C" ms_status ms_k_embedding_backward(int32_t dtype, int32_t n, int32_t d, int32_t vocab, const int32_t *ids,
                                             const void *dx, float *d_table, void *stream) {
    if (n == 0) return MS_OK;
    if (!ids || !dx || !d_table || n < 0 || d <= 0 || vocab <= 0) return ms_fail(MS_ERR_INVALID_ARG, "embedding_backward: bad argument");
    const int V = dtype == MS_BF16 ? 8 : 4;
    if (d % V) return ms_fail(MS_ERR_UNSUPPORTED, "embedding: d=%d must be a multiple of %d", d, V);
    DISPATCH_T(dtype, { embedding_bwd_kernel<T><<<n, 256, 0, (hipStream_t)stream>>>(ids, (const T *)dx, d_table, d, vocab); });
    MS_LAUNCH_CHECK();
    return MS_OK;
}

extern "C" ms_status ms_k_copy(const void *src, void *dst, size_t bytes, void *stream) {
    if (bytes == 0) return MS_OK;
    if (!src || !dst || bytes % 16 || !aligned16(src) || !aligned16(dst)) return ms_fail(MS_ERR_INVALID_ARG, "copy: need 16-byte multiples");
    const long nvec = bytes / 16;
    const int grid = ms_cdiv(nvec, 4096) > 4096 ? 4096 : ms_cdiv(nvec, 4096);
    copy_kernel<<<grid, 1024, 0, (hipStream_t)stream>>>((const copy_u32x4 *)src, (copy_u32x4 *)dst, nvec);
    MS_LAUNCH_CHECK();
    return MS_OK;
}

// internal helpers declared in launch.h
ms_status launch_fill_f32(float *p, long n, float v, hipStream_t s) {
    if (n <= 0) return MS_OK;
    const int grid = ms_cdiv(n, 256) > 8192 ? 8192 : ms_cdiv(n, 256);
    fill_f32_kernel<<<grid, 256, 0, s>>>(p, n, v);
    MS_LAUNCH_CHECK();
    return MS_OK;
}

ms_status launch_convert_bf16_to_f32(const void *src, float *dst, long n, hipStream_t s) {
    if (n <= 0) return MS_OK;
    const int grid = ms_cdiv(n, 256) > 16384 ? 16384 : ms_cdiv(n, 256);
    convert_bf16_to_f32_kernel<<<grid, 256, 0, s>>>((const bf16_t *)src, dst, n);
    MS_LAUNCH_CHECK();
    return MS_OK;
}

ms_status launch_convert_from_f32(int dtype, const float *src, void *dst, long n, hipStream_t s) {
    if (n <= 0) return MS_OK;
    const int grid = ms_cdiv(n, 256) > 16384 ? 16384 : ms_cdiv(n, 256);
    DISPATCH_T(dtype, { convert_from_f32_kernel<T><<<grid, 256, 0, s>>>(src, (T *)dst, n); });
    MS_LAUNCH_CHECK();
    return MS_OK;
}

// ------------------------------------------------------------------ AdamW (the student's parameter update)
// 4 elements per thread: 16-byte loads and stores of the four fp32 streams, 8 bytes of bf16 weights.
namespace {
template <class T>
__global__ __launch_bounds__(256) void adamw_kernel(long n4, float *__restrict__ grad, float *__restrict__ master,
                                                     float *__restrict__ m, float *__restrict__ v, T *__restrict__ w,
                                                     float lr, float b1, float b2, float eps, float decay, float gscale,
                                                     float inv_c1, float inv_c2, int zero_grad) {
    const long stride = (long)gridDim.x * 256;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
        const float4 g4 = ((const float4 *)grad)[i], w4 = ((const float4 *)master)[i];
        const float4 m4 = ((const float4 *)m)[i], v4 = ((const float4 *)v)[i];
        const float g[4] = {g4.x, g4.y, g4.z, g4.w};
        float ww[4] = {w4.x, w4.y, w4.z, w4.w}, mm[4] = {m4.x, m4.y, m4.z, m4.w}, vv[4] = {v4.x, v4.y, v4.z, v4.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float ge = gscale * g[e];
            mm[e] = b1 * mm[e] + (1.f - b1) * ge;
            vv[e] = b2 * vv[e] + (1.f - b2) * ge * ge;
            ww[e] = ww[e] * decay - lr * (mm[e] * inv_c1) / (sqrtf(vv[e] * inv_c2) + eps);
        }
        ((float4 *)master)[i] = make_float4(ww[0], ww[1], ww[2], ww[3]);
        ((float4 *)m)[i] = make_float4(mm[0], mm[1], mm[2], mm[3]);
        ((float4 *)v)[i] = make_float4(vv[0], vv[1], vv[2], vv[3]);
        if (zero_grad) ((float4 *)grad)[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (w) {
#pragma unroll
            for (int e = 0; e < 4; ++e) w[4 * i + e] = from_f32<T>(ww[e]);
        }
    }
}
}  // namespace

extern "C" ms_status ms_adamw_step(const ms_adamw_config *cfg, int32_t dtype, int64_t n, float *grad, float *master,
                                   float *m, float *v, void *weight, void *stream) {
    if (!cfg || n < 0) return ms_fail(MS_ERR_INVALID_ARG, "adamw: null config or negative size");
    if (n == 0) return MS_OK;
    if (!grad || !master || !m || !v) return ms_fail(MS_ERR_INVALID_ARG, "adamw: null pointer");
    if (dtype != MS_BF16 && dtype != MS_F32) return ms_fail(MS_ERR_INVALID_ARG, "adamw: bad dtype");
    if (cfg->step < 1 || !(cfg->beta1 >= 0.f && cfg->beta1 < 1.f) || !(cfg->beta2 >= 0.f && cfg->beta2 < 1.f) || !(cfg->eps >= 0.f) ||
        !(cfg->lr >= 0.f) || !(cfg->weight_decay >= 0.f))
        return ms_fail(MS_ERR_INVALID_ARG, "adamw: step must be >= 1, betas in [0, 1), lr, eps and weight decay >= 0");
    if (n % 4 || !aligned16(grad) || !aligned16(master) || !aligned16(m) || !aligned16(v) || (weight && ((uintptr_t)weight & 7)))
        return ms_fail(MS_ERR_UNSUPPORTED, "adamw: n must be a multiple of 4 and the arrays 16-byte aligned");
    // bias corrections in double on the host: 1 - beta^step loses digits in fp32 for small steps
    const float inv_c1 = (float)(1.0 / (1.0 - pow((double)cfg->beta1, (double)cfg->step)));
    const float inv_c2 = (float)(1.0 / (1.0 - pow((double)cfg->beta2, (double)cfg->step)));
    const float decay = 1.f - cfg->lr * cfg->weight_decay;
    const long n4 = n / 4;
    const int grid = ms_cdiv(n4, 256) > 16384 ? 16384 : (int)ms_cdiv(n4, 256);
    hipStream_t s = (hipStream_t)stream;
    ProfScope ps(11, (double)n * (4 * 7 + (weight ? (dtype == MS_BF16 ? 2 : 4) : 0) + (cfg->zero_grad ? 4 : 0)), s);
    if (dtype == MS_BF16) adamw_kernel<bf16_t><<<grid, 256, 0, s>>>(n4, grad, master, m, v, (bf16_t *)weight, cfg->lr, cfg->beta1, cfg->beta2, cfg->eps, decay, cfg->grad_scale, inv_c1, inv_c2, cfg->zero_grad);
    else adamw_kernel<float><<<grid, 256, 0, s>>>(n4, grad, master, m, v, (float *)weight, cfg->lr, cfg->beta1, cfg->beta2, cfg->eps, decay, cfg->grad_scale, inv_c1, inv_c2, cfg->zero_grad);
    MS_LAUNCH_CHECK();
    return MS_OK;
}
