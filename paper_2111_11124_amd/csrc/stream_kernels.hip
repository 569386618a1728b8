// stream_kernels.hip -- the HBM-bound element-wise half of libmesa for gfx950:
//   per-group min/max + running-estimate update   (Sec. 3.2 Eq. 6-7)
//   quantize with nearest or stochastic rounding  (Sec. 3.2 Eq. 3-4)
//   de-quantize                                    (Sec. 3.2 Eq. 5)
//   GELU backward at the de-quantized input        (Sec. 3.1 Eq. 2)
// plus a plain copy kernel and HIP-event helpers for measurement.
//
// Shape of every kernel: 256-thread workgroups, grid-stride; per iteration a thread owns U
// vectors of 8 consecutive elements (one 128-bit load of binary16, one 64-bit access of codes),
// a whole grid apart from each other so that each wave instruction touches one contiguous span.
// The group of a vector is tracked by a cursor (adds and compares only); vectors that cross a
// slab end, and the ragged tail, take a per-element path.
//
// Everything that feeds a code or a running parameter is binary32 with separately rounded
// operations: contraction into fused multiply-adds is switched off for this file, and the one
// kernel that may fuse (GELU backward) asks for it explicitly with fmaf.
#include <hip/hip_runtime.h>

#include "api_util.hpp"
#include "common.hpp"

#pragma clang fp contract(off)

namespace mesa {

constexpr int kU = 4;            // vectors in flight per thread and iteration
constexpr int kGridCap = 2048;   // 8 workgroups of 4 waves on each of the 256 CUs

// ---------------------------------------------------------------------------------------------
// per-group parameter table in LDS: (scale, beta) per group
// ---------------------------------------------------------------------------------------------
enum class Scale { Quant, Dequant };

template <Scale S>
__device__ __forceinline__ void fill_table(float2 *tab, const float *alpha, const float *beta, uint32_t groups)
{
    for (uint32_t g = threadIdx.x; g < groups; g += kThreads) {
        float a = alpha[g];
        float s;
        if (S == Scale::Quant) s = (a > 0.0f) ? 255.0f / a : 0.0f;  // correctly rounded division
        else s = a / 255.0f;
        tab[g] = make_float2(s, beta[g]);
    }
    __syncthreads();
}

// ---------------------------------------------------------------------------------------------
// min / max
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ int order_key(float f)  // monotone map binary32 -> int32 (an involution)
{
    int b = __float_as_int(f);
    return b >= 0 ? b : b ^ 0x7FFFFFFF;
}
__device__ __forceinline__ float order_val(int k) { return __int_as_float(k >= 0 ? k : k ^ 0x7FFFFFFF); }

template <typename T> struct MinMax;

template <> struct MinMax<float> {
    float mn, mx;
    __device__ __forceinline__ void init() { mn = __builtin_inff(); mx = -__builtin_inff(); }
    __device__ __forceinline__ void add(const Store<float>::raw_t &v)
    {
        float f[8];
        Store<float>::unpack(v, f);
#pragma unroll
        for (int j = 0; j < 8; ++j) { mn = fminf(mn, f[j]); mx = fmaxf(mx, f[j]); }
    }
    __device__ __forceinline__ void add1(float f) { mn = fminf(mn, f); mx = fmaxf(mx, f); }
    __device__ __forceinline__ float lo() const { return mn; }
    __device__ __forceinline__ float hi() const { return mx; }
};

// binary16 data: selection is exact in any precision, so compare packed pairs directly
template <> struct MinMax<_Float16> {
    h2 mn, mx;
    __device__ __forceinline__ void init()
    {
        mn = as_h2(0x7C007C00u);  // +inf, +inf
        mx = as_h2(0xFC00FC00u);  // -inf, -inf
    }
    __device__ __forceinline__ void add(const Store<_Float16>::raw_t &v)
    {
        h2 a = as_h2(v[0]), b = as_h2(v[1]), c = as_h2(v[2]), d = as_h2(v[3]);
        mn = __builtin_elementwise_min(mn, __builtin_elementwise_min(__builtin_elementwise_min(a, b),
                                                                     __builtin_elementwise_min(c, d)));
        mx = __builtin_elementwise_max(mx, __builtin_elementwise_max(__builtin_elementwise_max(a, b),
                                                                     __builtin_elementwise_max(c, d)));
    }
    __device__ __forceinline__ void add1(float f)
    {
        h2 p;
        p.x = _Float16(f);
        p.y = p.x;
        mn = __builtin_elementwise_min(mn, p);
        mx = __builtin_elementwise_max(mx, p);
    }
    __device__ __forceinline__ float lo() const { return fminf(float(mn.x), float(mn.y)); }
    __device__ __forceinline__ float hi() const { return fmaxf(float(mx.x), float(mx.y)); }
};

__device__ __forceinline__ void flush_lane(int *lmn, int *lmx, uint32_t g, float lo, float hi)
{
    if (lo <= hi) {  // something was accumulated
        atomicMin(&lmn[g], order_key(lo));
        atomicMax(&lmx[g], order_key(hi));
    }
}

// partial extrema of each workgroup: part[wg][0..G) = min, part[wg][G..2G) = max
template <typename T, int U>
__global__ __launch_bounds__(kThreads) void k_minmax_partial(const void *__restrict__ x, int64_t numel, GroupGeom gg,
                                                             float *__restrict__ part)
{
    extern __shared__ int lds_mm[];
    int *lmn = lds_mm;
    int *lmx = lds_mm + gg.groups;
    for (uint32_t g = threadIdx.x; g < gg.groups; g += kThreads) {
        lmn[g] = order_key(__builtin_inff());
        lmx[g] = order_key(-__builtin_inff());
    }
    __syncthreads();

    const int64_t span = int64_t(gridDim.x) * kThreads * kVec;
    const int64_t step = span * U;
    int64_t e[U];
    Cursor c[U];
    MinMax<T> acc[U];
    uint32_t cur[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        e[u] = u * span + (int64_t(blockIdx.x) * kThreads + threadIdx.x) * kVec;
        c[u] = cursor_init(e[u], gg);
        cur[u] = c[u].g;
        acc[u].init();
    }

    while (e[0] < numel) {
        typename Store<T>::raw_t v[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (e[u] + kVec <= numel) v[u] = Store<T>::load(x, e[u]);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (e[u] + kVec <= numel && c[u].rem + kVec <= gg.inner) {
                if (c[u].g != cur[u]) {
                    flush_lane(lmn, lmx, cur[u], acc[u].lo(), acc[u].hi());
                    cur[u] = c[u].g;
                    acc[u].init();
                }
                acc[u].add(v[u]);
            } else if (e[u] < numel) {  // crosses a slab end, or is the ragged tail
                int64_t left = numel - e[u];
                int n = left < kVec ? int(left) : kVec;
                for (int j = 0; j < n; ++j) {
                    uint32_t g = group_of(c[u], j, gg);
                    if (g != cur[u]) {
                        flush_lane(lmn, lmx, cur[u], acc[u].lo(), acc[u].hi());
                        cur[u] = g;
                        acc[u].init();
                    }
                    acc[u].add1(Store<T>::load1(x, e[u] + j));
                }
            }
            e[u] += step;
            cursor_advance(c[u], gg);
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        // a wave whose lanes all sit in one group (head-wise tensors) combines in registers first
        float lo = acc[u].lo(), hi = acc[u].hi();
        uint32_t g0 = __builtin_amdgcn_readfirstlane(cur[u]);
        if (__all(cur[u] == g0)) {
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) {
                lo = fminf(lo, __shfl_xor(lo, off, 64));
                hi = fmaxf(hi, __shfl_xor(hi, off, 64));
            }
            if ((threadIdx.x & 63) == 0) flush_lane(lmn, lmx, g0, lo, hi);
        } else {
            flush_lane(lmn, lmx, cur[u], lo, hi);
        }
    }
    __syncthreads();
    float *out = part + int64_t(blockIdx.x) * 2 * gg.groups;
    for (uint32_t g = threadIdx.x; g < gg.groups; g += kThreads) {
        out[g] = order_val(lmn[g]);
        out[gg.groups + g] = order_val(lmx[g]);
    }
}

// one workgroup per group: combine the partial extrema, then Eq. (6)-(7)
__global__ __launch_bounds__(kThreads) void k_ema_finalize(const float *__restrict__ part, int nwg, uint32_t groups,
                                                           float *alpha, float *beta, float lambda, int first_call)
{
    __shared__ float smn[kThreads / 64], smx[kThreads / 64];
    const uint32_t g = blockIdx.x;
    float mn = __builtin_inff(), mx = -__builtin_inff();
    for (int w = threadIdx.x; w < nwg; w += kThreads) {
        mn = fminf(mn, part[int64_t(w) * 2 * groups + g]);
        mx = fmaxf(mx, part[int64_t(w) * 2 * groups + groups + g]);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        mn = fminf(mn, __shfl_xor(mn, off, 64));
        mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    }
    if ((threadIdx.x & 63) == 0) { smn[threadIdx.x >> 6] = mn; smx[threadIdx.x >> 6] = mx; }
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < kThreads / 64; ++w) { mn = fminf(mn, smn[w]); mx = fmaxf(mx, smx[w]); }
        mn = mn + 0.0f;  // -0.0 -> +0.0
        mx = mx + 0.0f;
        float range = mx - mn;
        if (first_call) {
            alpha[g] = range;
            beta[g] = mn;
        } else {
            float a = lambda * alpha[g];
            float b = 1.0f - lambda;
            float c = b * range;
            alpha[g] = a + c;
            float e = lambda * beta[g];
            float f = b * mn;
            beta[g] = e + f;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Philox-4x32-10 (Salmon et al., SC'11): ten rounds of two 32x32->64 multiplies and a key bump
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t k0, uint32_t k1, uint32_t out[4])
{
    uint32_t c2 = 0u, c3 = 0u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        uint64_t p0 = uint64_t(0xD2511F53u) * uint64_t(c0);
        uint64_t p1 = uint64_t(0xCD9E8D57u) * uint64_t(c2);
        uint32_t n0 = uint32_t(p1 >> 32) ^ c1 ^ k0;
        uint32_t n2 = uint32_t(p0 >> 32) ^ c3 ^ k1;
        c1 = uint32_t(p1);
        c3 = uint32_t(p0);
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// the eight random fractions of the block of elements [8b, 8b+8): 16 bits each, u = bits * 2^-16
__device__ __forceinline__ void sr_fractions(uint64_t seed, uint64_t counter, float u[8])
{
    uint32_t w[4];
    philox4x32_10(uint32_t(counter), uint32_t(counter >> 32), uint32_t(seed), uint32_t(seed >> 32), w);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        u[2 * k] = float(w[k] & 0xFFFFu) * 1.52587890625e-05f;
        u[2 * k + 1] = float(w[k] >> 16) * 1.52587890625e-05f;
    }
}

template <bool SR> __device__ __forceinline__ float quantize_one(float x, float r, float b, float u)
{
    float t = x - b;
    float v = t * r;
    float w;
    if (SR) {
        float s = v + u;
        w = floorf(s);
    } else {
        w = rintf(v);  // nearest, ties to even
    }
    return clamp_code(w);
}

template <typename T, int U, bool SR>
__global__ __launch_bounds__(kThreads) void k_quantize(const void *__restrict__ x, int8_t *__restrict__ q, int64_t numel,
                                                       GroupGeom gg, const float *__restrict__ alpha,
                                                       const float *__restrict__ beta, uint64_t seed, uint64_t offset)
{
    extern __shared__ float2 lds_tab[];
    fill_table<Scale::Quant>(lds_tab, alpha, beta, gg.groups);

    const int64_t span = int64_t(gridDim.x) * kThreads * kVec;
    const int64_t step = span * U;
    int64_t e[U];
    Cursor c[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        e[u] = u * span + (int64_t(blockIdx.x) * kThreads + threadIdx.x) * kVec;
        c[u] = cursor_init(e[u], gg);
    }
    while (e[0] < numel) {
        typename Store<T>::raw_t v[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (e[u] + kVec <= numel) v[u] = Store<T>::load(x, e[u]);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (e[u] < numel) {
                float rnd[8];
                if (SR) sr_fractions(seed, offset + uint64_t(e[u] >> 3), rnd);
                if (e[u] + kVec <= numel) {
                    float f[8], w[8];
                    Store<T>::unpack(v[u], f);
                    if (c[u].rem + kVec <= gg.inner) {
                        float2 p = lds_tab[c[u].g];
#pragma unroll
                        for (int j = 0; j < 8; ++j) w[j] = quantize_one<SR>(f[j], p.x, p.y, SR ? rnd[j] : 0.0f);
                    } else {
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            float2 p = lds_tab[group_of(c[u], j, gg)];
                            w[j] = quantize_one<SR>(f[j], p.x, p.y, SR ? rnd[j] : 0.0f);
                        }
                    }
                    *reinterpret_cast<u32x2 *>(q + e[u]) = float_to_codes(w);
                } else {
                    int n = int(numel - e[u]);
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        if (j < n) {
                            float2 p = lds_tab[group_of(c[u], j, gg)];
                            float w = quantize_one<SR>(Store<T>::load1(x, e[u] + j), p.x, p.y, SR ? rnd[j] : 0.0f);
                            q[e[u] + j] = int8_t(int(w) - 128);
                        }
                    }
                }
            }
            e[u] += step;
            cursor_advance(c[u], gg);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// de-quantize
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float dequant_exact(float u, float s, float b)
{
    float xh = u * s;
    xh = xh + b;
    return xh;
}

template <typename T, int U>
__global__ __launch_bounds__(kThreads) void k_dequantize(const int8_t *__restrict__ q, void *__restrict__ xh, int64_t numel,
                                                         GroupGeom gg, const float *__restrict__ alpha,
                                                         const float *__restrict__ beta)
{
    extern __shared__ float2 lds_tab[];
    fill_table<Scale::Dequant>(lds_tab, alpha, beta, gg.groups);

    const int64_t span = int64_t(gridDim.x) * kThreads * kVec;
    const int64_t step = span * U;
    int64_t e[U];
    Cursor c[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        e[u] = u * span + (int64_t(blockIdx.x) * kThreads + threadIdx.x) * kVec;
        c[u] = cursor_init(e[u], gg);
    }
    while (e[0] < numel) {
        u32x2 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (e[u] + kVec <= numel) v[u] = load_codes8(q, e[u]);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (e[u] + kVec <= numel) {
                float uu[8], f[8];
                codes_to_float(v[u], uu);
                if (c[u].rem + kVec <= gg.inner) {
                    float2 p = lds_tab[c[u].g];
#pragma unroll
                    for (int j = 0; j < 8; ++j) f[j] = dequant_exact(uu[j], p.x, p.y);
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        float2 p = lds_tab[group_of(c[u], j, gg)];
                        f[j] = dequant_exact(uu[j], p.x, p.y);
                    }
                }
                Store<T>::store(xh, e[u], Store<T>::pack(f));
            } else if (e[u] < numel) {
                int n = int(numel - e[u]);
                for (int j = 0; j < n; ++j) {
                    float2 p = lds_tab[group_of(c[u], j, gg)];
                    Store<T>::store1(xh, e[u] + j, dequant_exact(code_to_float(q[e[u] + j]), p.x, p.y));
                }
            }
            e[u] += step;
            cursor_advance(c[u], gg);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// GELU backward at x_hat
// ---------------------------------------------------------------------------------------------
// gelu'(x) = Phi(x) + x*phi(x).  With E = exp(-x^2/2):  phi = E/sqrt(2 pi) and
// Phi(-|x|) = erfc(|x|/sqrt 2)/2 = P(t)*E/2, t = 1/(1 + p|x|/sqrt 2), P the degree-5 polynomial of
// Abramowitz & Stegun 7.1.26 (|error| <= 1.5e-7 on erf): one exponential serves both terms.
__device__ __forceinline__ float gelu_grad(float x)
{
    float ax = fabsf(x);
    float t = __builtin_amdgcn_rcpf(fmaf(ax, 0.3275911f * 0.70710678118654752f, 1.0f));
    float poly = fmaf(t, 1.061405429f, -1.453152027f);
    poly = fmaf(poly, t, 1.421413741f);
    poly = fmaf(poly, t, -0.284496736f);
    poly = fmaf(poly, t, 0.254829592f);
    poly = poly * t;
    float E = __builtin_amdgcn_exp2f(x * x * -0.72134752044448170f);  // exp(-x^2/2)
    float h = 0.5f * poly * E;
    float cdf = (x >= 0.0f) ? 1.0f - h : h;
    return fmaf(x * E, 0.39894228040143268f, cdf);
}

template <typename T, int U>
__global__ __launch_bounds__(kThreads) void k_gelu_bwd(const int8_t *__restrict__ q, const void *dy, void *dx, int64_t numel,
                                                       GroupGeom gg, const float *__restrict__ alpha,
                                                       const float *__restrict__ beta)
{
    extern __shared__ float2 lds_tab[];
    fill_table<Scale::Dequant>(lds_tab, alpha, beta, gg.groups);

    const int64_t span = int64_t(gridDim.x) * kThreads * kVec;
    const int64_t step = span * U;
    int64_t e[U];
    Cursor c[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        e[u] = u * span + (int64_t(blockIdx.x) * kThreads + threadIdx.x) * kVec;
        c[u] = cursor_init(e[u], gg);
    }
    while (e[0] < numel) {
        u32x2 v[U];
        typename Store<T>::raw_t d[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (e[u] + kVec <= numel) {
                v[u] = load_codes8(q, e[u]);
                d[u] = Store<T>::load(dy, e[u]);
            }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (e[u] + kVec <= numel) {
                float uu[8], g[8];
                codes_to_float(v[u], uu);
                Store<T>::unpack(d[u], g);
                if (c[u].rem + kVec <= gg.inner) {
                    float2 p = lds_tab[c[u].g];
#pragma unroll
                    for (int j = 0; j < 8; ++j) g[j] = g[j] * gelu_grad(fmaf(uu[j], p.x, p.y));
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        float2 p = lds_tab[group_of(c[u], j, gg)];
                        g[j] = g[j] * gelu_grad(fmaf(uu[j], p.x, p.y));
                    }
                }
                Store<T>::store(dx, e[u], Store<T>::pack(g));
            } else if (e[u] < numel) {
                int n = int(numel - e[u]);
                for (int j = 0; j < n; ++j) {
                    float2 p = lds_tab[group_of(c[u], j, gg)];
                    float xh = fmaf(code_to_float(q[e[u] + j]), p.x, p.y);
                    Store<T>::store1(dx, e[u] + j, Store<T>::load1(dy, e[u] + j) * gelu_grad(xh));
                }
            }
            e[u] += step;
            cursor_advance(c[u], gg);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// plain copy (measurement)
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void k_copy(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, int64_t n16)
{
    const int64_t span = int64_t(gridDim.x) * kThreads;
    int64_t i = int64_t(blockIdx.x) * kThreads + threadIdx.x;
    for (; i + 3 * span < n16; i += 4 * span) {
        u32x4 a = src[i], b = src[i + span], c = src[i + 2 * span], d = src[i + 3 * span];
        dst[i] = a; dst[i + span] = b; dst[i + 2 * span] = c; dst[i + 3 * span] = d;
    }
    for (; i < n16; i += span) dst[i] = src[i];
}

}  // namespace mesa

// =================================================================================================
// entry points
// =================================================================================================
using namespace mesa;

static int stream_grid(int64_t numel, int64_t row)
{
    return plan_grid(numel, int64_t(kThreads) * kVec * kU, kGridCap, row);
}

static int minmax_grid(const mesa_layout &L)
{
    int64_t numel = layout_numel(L);
    // many groups: every workgroup writes 2*groups partial values, so keep their number down
    int cap = kGridCap;
    if (L.groups > 64) {
        cap = int(int64_t(kGridCap) * 64 / L.groups);
        if (cap < 32) cap = 32;
    }
    return plan_grid(numel, int64_t(kThreads) * kVec * kU, cap, L.groups > 1 ? L.groups * L.inner : 0);
}

extern "C" MESA_EXPORT mesa_status mesa_update_running_params(const void *x, mesa_dtype dt, mesa_layout L, float *alpha, float *beta,
                                                  float lambda, int first_call, void *ws, size_t ws_bytes, void *stream)
{
    if (!valid_dtype(dt)) return MESA_ERR_INVALID_ARG;
    mesa_status st = check_layout(L);
    if (st != MESA_OK) return st;
    if (!(lambda >= 0.0f && lambda <= 1.0f)) return MESA_ERR_INVALID_ARG;
    const int64_t numel = layout_numel(L);
    if (numel == 0) return MESA_OK;
    if (!x || !alpha || !beta || !aligned16(x) || !aligned4(alpha) || !aligned4(beta)) return MESA_ERR_INVALID_ARG;
    if (!ws || !aligned16(ws) || ws_bytes < update_ws_bytes(L.outer, L.groups, L.inner))
        return MESA_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int grid = minmax_grid(L);
    const int64_t step = int64_t(grid) * kThreads * kVec * kU;
    GroupGeom gg = make_geom(L.groups, L.inner, step);
    const size_t lds = size_t(2) * gg.groups * sizeof(int);
    float *part = static_cast<float *>(ws);
    if (dt == MESA_F16)
        hipLaunchKernelGGL((k_minmax_partial<_Float16, kU>), dim3(grid), dim3(kThreads), lds, s, x, numel, gg, part);
    else
        hipLaunchKernelGGL((k_minmax_partial<float, kU>), dim3(grid), dim3(kThreads), lds, s, x, numel, gg, part);
    hipLaunchKernelGGL(k_ema_finalize, dim3(gg.groups), dim3(kThreads), 0, s, part, grid, gg.groups, alpha, beta, lambda,
                       first_call);
    return launch_status();
}

extern "C" MESA_EXPORT mesa_status mesa_quantize_headwise(const void *x, mesa_dtype dt, mesa_layout L, const float *alpha,
                                              const float *beta, int8_t *q, mesa_round mode, uint64_t seed, uint64_t offset,
                                              void *stream)
{
    if (!valid_dtype(dt) || (mode != MESA_ROUND_NEAREST_EVEN && mode != MESA_ROUND_STOCHASTIC)) return MESA_ERR_INVALID_ARG;
    mesa_status st = check_layout(L);
    if (st != MESA_OK) return st;
    const int64_t numel = layout_numel(L);
    if (numel == 0) return MESA_OK;
    if (!x || !q || !alpha || !beta || !aligned16(x) || !aligned16(q) || !aligned4(alpha) || !aligned4(beta))
        return MESA_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int grid = stream_grid(numel, L.groups > 1 ? L.groups * L.inner : 0);
    GroupGeom gg = make_geom(L.groups, L.inner, int64_t(grid) * kThreads * kVec * kU);
    const size_t lds = size_t(gg.groups) * sizeof(float2);
    const bool sr = mode == MESA_ROUND_STOCHASTIC;
#define MESA_LAUNCH_Q(T, SRF) \
    hipLaunchKernelGGL((k_quantize<T, kU, SRF>), dim3(grid), dim3(kThreads), lds, s, x, q, numel, gg, alpha, beta, seed, offset)
    if (dt == MESA_F16) { if (sr) MESA_LAUNCH_Q(_Float16, true); else MESA_LAUNCH_Q(_Float16, false); }
    else { if (sr) MESA_LAUNCH_Q(float, true); else MESA_LAUNCH_Q(float, false); }
#undef MESA_LAUNCH_Q
    return launch_status();
}

extern "C" MESA_EXPORT mesa_status mesa_dequantize(const int8_t *q, mesa_layout L, const float *alpha, const float *beta, void *x_hat,
                                       mesa_dtype dt, void *stream)
{
    if (!valid_dtype(dt)) return MESA_ERR_INVALID_ARG;
    mesa_status st = check_layout(L);
    if (st != MESA_OK) return st;
    const int64_t numel = layout_numel(L);
    if (numel == 0) return MESA_OK;
    if (!q || !x_hat || !alpha || !beta || !aligned16(q) || !aligned16(x_hat) || !aligned4(alpha) || !aligned4(beta))
        return MESA_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int grid = stream_grid(numel, L.groups > 1 ? L.groups * L.inner : 0);
    GroupGeom gg = make_geom(L.groups, L.inner, int64_t(grid) * kThreads * kVec * kU);
    const size_t lds = size_t(gg.groups) * sizeof(float2);
    if (dt == MESA_F16)
        hipLaunchKernelGGL((k_dequantize<_Float16, kU>), dim3(grid), dim3(kThreads), lds, s, q, x_hat, numel, gg, alpha, beta);
    else
        hipLaunchKernelGGL((k_dequantize<float, kU>), dim3(grid), dim3(kThreads), lds, s, q, x_hat, numel, gg, alpha, beta);
    return launch_status();
}

extern "C" MESA_EXPORT mesa_status mesa_gelu_bwd_q(const int8_t *xq, mesa_layout L, const float *alpha, const float *beta, const void *dy,
                                       void *dx, mesa_dtype dt, void *stream)
{
    if (!valid_dtype(dt)) return MESA_ERR_INVALID_ARG;
    mesa_status st = check_layout(L);
    if (st != MESA_OK) return st;
    const int64_t numel = layout_numel(L);
    if (numel == 0) return MESA_OK;
    if (!xq || !dy || !dx || !alpha || !beta || !aligned16(xq) || !aligned16(dy) || !aligned16(dx) || !aligned4(alpha) ||
        !aligned4(beta))
        return MESA_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int grid = stream_grid(numel, L.groups > 1 ? L.groups * L.inner : 0);
    GroupGeom gg = make_geom(L.groups, L.inner, int64_t(grid) * kThreads * kVec * kU);
    const size_t lds = size_t(gg.groups) * sizeof(float2);
    if (dt == MESA_F16)
        hipLaunchKernelGGL((k_gelu_bwd<_Float16, kU>), dim3(grid), dim3(kThreads), lds, s, xq, dy, dx, numel, gg, alpha, beta);
    else
        hipLaunchKernelGGL((k_gelu_bwd<float, kU>), dim3(grid), dim3(kThreads), lds, s, xq, dy, dx, numel, gg, alpha, beta);
    return launch_status();
}

extern "C" MESA_EXPORT mesa_status mesa_stream_copy(const void *src, void *dst, size_t bytes, void *stream)
{
    if (bytes == 0) return MESA_OK;
    if (!src || !dst || !aligned16(src) || !aligned16(dst) || (bytes & 15u)) return MESA_ERR_INVALID_ARG;
    const int64_t n16 = int64_t(bytes / 16);
    const int grid = plan_grid(n16, int64_t(kThreads) * 4, kGridCap, 0);
    hipLaunchKernelGGL(k_copy, dim3(grid), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4 *>(src), static_cast<u32x4 *>(dst), n16);
    return launch_status();
}

extern "C" MESA_EXPORT mesa_status mesa_event_create(void **event)
{
    if (!event) return MESA_ERR_INVALID_ARG;
    hipEvent_t ev;
    if (hipEventCreate(&ev) != hipSuccess) return MESA_ERR_LAUNCH;
    *event = ev;
    return MESA_OK;
}

extern "C" MESA_EXPORT mesa_status mesa_event_record(void *event, void *stream)
{
    if (!event) return MESA_ERR_INVALID_ARG;
    return hipEventRecord(static_cast<hipEvent_t>(event), static_cast<hipStream_t>(stream)) == hipSuccess ? MESA_OK
                                                                                                           : MESA_ERR_LAUNCH;
}

extern "C" MESA_EXPORT mesa_status mesa_event_elapsed_ms(void *start, void *stop, float *ms)
{
    if (!start || !stop || !ms) return MESA_ERR_INVALID_ARG;
    if (hipEventSynchronize(static_cast<hipEvent_t>(stop)) != hipSuccess) return MESA_ERR_LAUNCH;
    return hipEventElapsedTime(ms, static_cast<hipEvent_t>(start), static_cast<hipEvent_t>(stop)) == hipSuccess
               ? MESA_OK
               : MESA_ERR_LAUNCH;
}

extern "C" MESA_EXPORT mesa_status mesa_event_destroy(void *event)
{
    if (!event) return MESA_ERR_INVALID_ARG;
    return hipEventDestroy(static_cast<hipEvent_t>(event)) == hipSuccess ? MESA_OK : MESA_ERR_LAUNCH;
}

extern "C" MESA_EXPORT const char *mesa_status_string(mesa_status s)
{
    switch (s) {
    case MESA_OK: return "ok";
    case MESA_ERR_INVALID_ARG: return "invalid argument";
    case MESA_ERR_UNSUPPORTED: return "unsupported shape";
    case MESA_ERR_WORKSPACE: return "workspace missing or too small";
    case MESA_ERR_LAUNCH: return "HIP runtime error";
    }
    return "unknown status";
}

extern "C" MESA_EXPORT int mesa_version(void) { return 100; }

extern "C" MESA_EXPORT size_t mesa_workspace_bytes(mesa_op op, int64_t d0, int64_t d1, int64_t d2, mesa_dtype dt)
{
    switch (op) {
    case MESA_OP_UPDATE_RUNNING_PARAMS: return update_ws_bytes(d0, d1, d2);
    case MESA_OP_LAYERNORM_BWD_Q: return layernorm_ws_bytes(d0, d1);
    case MESA_OP_LINEAR_DW_Q: return linear_dw_ws_bytes(d0, d1, d2, dt);
    }
    return 0;
}

// size of the min/max partials; must agree with minmax_grid()
size_t mesa::update_ws_bytes(int64_t outer, int64_t groups, int64_t inner)
{
    mesa_layout L = {outer, groups, inner};
    if (check_layout(L) != MESA_OK || layout_numel(L) == 0) return 16;
    return size_t(minmax_grid(L)) * 2 * size_t(groups < 1 ? 1 : groups) * sizeof(float);
}
