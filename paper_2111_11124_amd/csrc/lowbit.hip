// lowbit.hip -- four-bit codes: Eq. (3)-(5) of Sec. 3.2 with 2^4 - 1 = 15 steps across the clipping range (Sec. 4.2
// names lower bit widths as the step beyond the method's fixed eight bits), two codes per byte, and the GELU backward
// at that reconstruction.  Half the bytes of the 8-bit codes on every pass that moves them:
//   quantize     2 + 0.5 bytes per binary16 element (8-bit: 2 + 1)
//   de-quantize  0.5 + 2                             (1 + 2)
//   GELU bwd     0.5 + 2 + 2                         (1 + 2 + 2)
// Element e sits in byte e/2, low four bits for even e; a thread's vector of eight consecutive elements is therefore
// one aligned 32-bit word of codes, next to its one 128-bit word of binary16 values.  The arithmetic that decides a
// code is the 8-bit quantizer's, operation for operation (quantize.hpp), with 15 in place of 255; the random
// fractions of stochastic rounding are the same ones (counter = offset + e/8, sixteen bits per element).
// Plain grid-stride kernels: a vector's group comes from two divisions by multiplication per vector rather than from
// the incremental cursors of the 8-bit kernels -- the passes are bound by memory either way.
#include <hip/hip_runtime.h>

#include "api_util.hpp"
#include "common.hpp"
#include "quantize.hpp"

#pragma clang fp contract(off)

namespace mesa {

constexpr int kB4GridCap = 16384;
constexpr int kB4LutMaxGroups = 1024;   // GELU-gradient table: groups * 16 floats in LDS

// group of flat element e; e < 2^31 goes through the 32-bit reciprocals, beyond that through binary64
__device__ __forceinline__ Cursor b4_cursor(int64_t e, const GroupGeom &gg, bool small)
{
    if (small) {
        Cursor z;
        z.rem = 0u;
        z.g = 0u;
        return cursor_offset(z, uint32_t(e), gg);
    }
    return cursor_init(e, gg);
}

template <bool QUANT>
__device__ __forceinline__ void b4_table(float2 *tab, const float *alpha, const float *beta, uint32_t groups)
{
    for (uint32_t g = threadIdx.x; g < groups; g += kThreads) {
        const float a = alpha[g];
        tab[g] = make_float2(QUANT ? ((a > 0.0f) ? 15.0f / a : 0.0f) : a / 15.0f, beta[g]);
    }
    __syncthreads();
}

// eight integers (as floats, any range) -> eight four-bit codes in one word, element j in bits 4j .. 4j+3.
// Four clipped values are summed with weights 1, 16, 256, 4096 in binary32 (exact: the sum stays below 2^16), so a
// half-word costs four clamps, three multiply-adds and one conversion.
__device__ __forceinline__ uint32_t pack_nibbles(const float w[8])
{
    uint32_t half[2];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        float c[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) c[j] = __builtin_amdgcn_fmed3f(w[4 * k + j], 0.0f, 15.0f);
        float s = fmaf(c[3], 16.0f, c[2]);
        s = fmaf(s, 16.0f, c[1]);
        s = fmaf(s, 16.0f, c[0]);
        half[k] = uint32_t(s);
    }
    return half[0] | (half[1] << 16);
}

template <typename T, bool SR>
__global__ __launch_bounds__(kThreads) void k_quantize_b4(const void *__restrict__ x, uint8_t *__restrict__ q4, int64_t numel,
                                                          GroupGeom gg, const float *__restrict__ alpha,
                                                          const float *__restrict__ beta, uint64_t seed, uint64_t offset)
{
    extern __shared__ float2 b4_tab[];
    b4_table<true>(b4_tab, alpha, beta, gg.groups);
    const bool small = numel < (int64_t(1) << 31);
    const int64_t nfull = numel / kVec;
    const int64_t stride = int64_t(gridDim.x) * kThreads;
    int64_t v = int64_t(blockIdx.x) * kThreads + threadIdx.x;
    // the next vector's load is in flight while this one's random bits and codes are computed
    decltype(Nt<T>::load(x, 0)) nxt = {};
    if (v < nfull) nxt = Nt<T>::load(x, v * kVec);
    for (; v < nfull; v += stride) {
        const auto raw = nxt;
        if (v + stride < nfull) nxt = Nt<T>::load(x, (v + stride) * kVec);
        const int64_t e = v * kVec;
        const Cursor c = b4_cursor(e, gg, small);
        float bits[8], w[8], f[8];
        if (SR) sr_bits(seed, offset + uint64_t(v), bits);
        Store<T>::unpack(raw, f);
        if (c.rem + kVec <= gg.inner) {
            const float2 p = b4_tab[c.g];
#pragma unroll
            for (int j = 0; j < 8; ++j) w[j] = quantize_one<SR>(f[j], p.x, p.y, SR ? bits[j] : 0.0f);
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float2 p = b4_tab[group_of(c, j, gg)];
                w[j] = quantize_one<SR>(f[j], p.x, p.y, SR ? bits[j] : 0.0f);
            }
        }
        nt_store<uint32_t>(q4 + (e >> 1), pack_nibbles(w));
    }
    // the ragged end of the tensor, one thread of the launch: whole bytes, the odd last code's partner zero
    const int cnt = int(numel - nfull * kVec);
    if (cnt > 0 && blockIdx.x == 0 && threadIdx.x == 0) {
        const int64_t e = nfull * kVec;
        const Cursor c = b4_cursor(e, gg, small);
        float bits[8], w[8];
        if (SR) sr_bits(seed, offset + uint64_t(nfull), bits);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            w[j] = 0.0f;
            if (j < cnt) {
                const float2 p = b4_tab[group_of(c, j, gg)];
                w[j] = quantize_one<SR>(Store<T>::load1(x, e + j), p.x, p.y, SR ? bits[j] : 0.0f);
            }
        }
        const uint32_t word = pack_nibbles(w);
        for (int k = 0; 2 * k < cnt; ++k) q4[(e >> 1) + k] = uint8_t(word >> (8 * k));
    }
}

__device__ __forceinline__ float b4_code(uint32_t word, int j) { return float((word >> (4 * j)) & 0xFu); }

// GELU = false: x_hat (separately rounded product and sum, as mesa_dequantize).  GELU = true: dx = dy * gelu'(x_hat).
__device__ __forceinline__ float b4_gelu_grad(float x)
{
    // Phi(-|x|) by Abramowitz & Stegun 7.1.26 (|error| <= 1.5e-7 on erf); one exponential serves Phi and phi
    const float ax = fabsf(x);
    const float t = __builtin_amdgcn_rcpf(fmaf(ax, 0.3275911f * 0.70710678118654752f, 1.0f));
    float poly = fmaf(t, 1.061405429f, -1.453152027f);
    poly = fmaf(poly, t, 1.421413741f);
    poly = fmaf(poly, t, -0.284496736f);
    poly = fmaf(poly, t, 0.254829592f);
    poly = poly * t;
    const float E = __builtin_amdgcn_exp2f(x * x * -0.72134752044448170f);
    const float h = 0.5f * poly * E;
    const float cdf = (x >= 0.0f) ? 1.0f - h : h;
    return fmaf(x * E, 0.39894228040143268f, cdf);
}

template <typename T, bool GELU, bool LUT>
__global__ __launch_bounds__(kThreads) void k_consume_b4(const uint8_t *__restrict__ q4, const void *dy, void *out, int64_t numel,
                                                         GroupGeom gg, const float *__restrict__ alpha,
                                                         const float *__restrict__ beta)
{
    extern __shared__ float b4_lds[];
    float2 *tab = reinterpret_cast<float2 *>(b4_lds);
    if (GELU && LUT) {   // gelu'(x_hat) for each of a group's sixteen reconstruction levels
        for (uint32_t i = threadIdx.x; i < gg.groups * 16u; i += kThreads) {
            const uint32_t g = i >> 4;
            b4_lds[i] = b4_gelu_grad(fmaf(float(i & 15u), alpha[g] / 15.0f, beta[g]));
        }
        __syncthreads();
    } else {
        b4_table<false>(tab, alpha, beta, gg.groups);
    }
    auto value = [&](uint32_t g, float u) -> float {   // what one code contributes: x_hat, or gelu'(x_hat)
        if (GELU && LUT) return b4_lds[g * 16u + uint32_t(u)];
        const float2 p = tab[g];
        if (GELU) return b4_gelu_grad(fmaf(u, p.x, p.y));
        float xh = u * p.x;
        xh = xh + p.y;
        return xh;
    };
    const bool small = numel < (int64_t(1) << 31);
    const int64_t nvec = (numel + kVec - 1) / kVec;
    for (int64_t v = int64_t(blockIdx.x) * kThreads + threadIdx.x; v < nvec; v += int64_t(gridDim.x) * kThreads) {
        const int64_t e = v * kVec;
        const Cursor c = b4_cursor(e, gg, small);
        if (e + kVec <= numel) {
            const uint32_t word = nt_load<uint32_t>(q4 + (e >> 1));
            float f[8], d[8];
            if (GELU) Store<T>::unpack(Nt<T>::load(dy, e), d);
            const bool one = c.rem + kVec <= gg.inner;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float t = value(one ? c.g : group_of(c, j, gg), b4_code(word, j));
                f[j] = GELU ? d[j] * t : t;
            }
            Nt<T>::store(out, e, Store<T>::pack(f));
        } else {
            for (int j = 0; e + j < numel; ++j) {
                const uint32_t byte = q4[(e + j) >> 1];
                const float t = value(group_of(c, j, gg), float((byte >> (4 * (j & 1))) & 0xFu));
                Store<T>::store1(out, e + j, GELU ? Store<T>::load1(dy, e + j) * t : t);
            }
        }
    }
}

static int b4_grid(int64_t numel)
{
    const int64_t nvec = ceil_div(numel, kVec);
    return plan_grid(nvec, kThreads, kB4GridCap, 0);
}

}  // namespace mesa

using namespace mesa;

extern "C" MESA_EXPORT mesa_status mesa_quantize_headwise_b4(const void *x, mesa_dtype dt, mesa_layout L, const float *alpha,
                                                             const float *beta, uint8_t *q4, mesa_round mode, uint64_t seed,
                                                             uint64_t offset, void *stream)
{
    if (!valid_dtype(dt) || (mode != MESA_ROUND_NEAREST_EVEN && mode != MESA_ROUND_STOCHASTIC)) return MESA_ERR_INVALID_ARG;
    mesa_status st = check_layout(L);
    if (st != MESA_OK) return st;
    const int64_t numel = layout_numel(L);
    if (numel == 0) return MESA_OK;
    if (!x || !q4 || !alpha || !beta || !aligned16(x) || !aligned16(q4) || !aligned4(alpha) || !aligned4(beta))
        return MESA_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int grid = b4_grid(numel);
    GroupGeom gg = make_geom(L.groups, L.inner, 0);
    const size_t lds = size_t(gg.groups) * sizeof(float2);
    const bool sr = mode == MESA_ROUND_STOCHASTIC;
#define MESA_LAUNCH_Q4(T) \
    do { \
        if (sr) hipLaunchKernelGGL((k_quantize_b4<T, true>), dim3(grid), dim3(kThreads), lds, s, x, q4, numel, gg, alpha, beta, seed, offset); \
        else hipLaunchKernelGGL((k_quantize_b4<T, false>), dim3(grid), dim3(kThreads), lds, s, x, q4, numel, gg, alpha, beta, seed, offset); \
    } while (0)
    MESA_FOR_DTYPE(dt, MESA_LAUNCH_Q4);
#undef MESA_LAUNCH_Q4
    return launch_status();
}

template <bool GELU>
static mesa_status consume_b4(const uint8_t *q4, mesa_layout L, const float *alpha, const float *beta, const void *dy, void *out,
                              mesa_dtype dt, void *stream)
{
    if (!valid_dtype(dt)) return MESA_ERR_INVALID_ARG;
    mesa_status st = check_layout(L);
    if (st != MESA_OK) return st;
    const int64_t numel = layout_numel(L);
    if (numel == 0) return MESA_OK;
    if (!q4 || !out || !alpha || !beta || !aligned16(q4) || !aligned16(out) || !aligned4(alpha) || !aligned4(beta))
        return MESA_ERR_INVALID_ARG;
    if (GELU && (!dy || !aligned16(dy))) return MESA_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int grid = b4_grid(numel);
    GroupGeom gg = make_geom(L.groups, L.inner, 0);
    const bool lut = GELU && gg.groups <= uint32_t(kB4LutMaxGroups);
    const size_t lds = lut ? size_t(gg.groups) * 16 * sizeof(float) : size_t(gg.groups) * sizeof(float2);
#define MESA_LAUNCH_C4(T) \
    do { \
        if (lut) hipLaunchKernelGGL((k_consume_b4<T, GELU, true>), dim3(grid), dim3(kThreads), lds, s, q4, dy, out, numel, gg, alpha, beta); \
        else hipLaunchKernelGGL((k_consume_b4<T, GELU, false>), dim3(grid), dim3(kThreads), lds, s, q4, dy, out, numel, gg, alpha, beta); \
    } while (0)
    MESA_FOR_DTYPE(dt, MESA_LAUNCH_C4);
#undef MESA_LAUNCH_C4
    return launch_status();
}

extern "C" MESA_EXPORT mesa_status mesa_dequantize_b4(const uint8_t *q4, mesa_layout L, const float *alpha, const float *beta,
                                                      void *x_hat, mesa_dtype dt, void *stream)
{
    return consume_b4<false>(q4, L, alpha, beta, nullptr, x_hat, dt, stream);
}

extern "C" MESA_EXPORT mesa_status mesa_gelu_bwd_q_b4(const uint8_t *q4, mesa_layout L, const float *alpha, const float *beta,
                                                      const void *dy, void *dx, mesa_dtype dt, void *stream)
{
    return consume_b4<true>(q4, L, alpha, beta, dy, dx, dt, stream);
}
