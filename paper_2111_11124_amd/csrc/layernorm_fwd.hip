// layernorm_fwd.hip -- a Mesa LayerNorm layer's forward in one pass over x (Sec. 3.1: the forward output is
// computed from the exact input; the input is what the layer saves, compressed -- Sec. 3.2 Eq. 3-4, 6-7 --
// together with the row statistics the backward needs):
//   per row  mean = sum x / D,  rstd = 1 / sqrt(sum (x - mean)^2 / D + eps),  y = (x - mean) * rstd * gamma + bias;
//   codes of x in G channel groups with the running estimates as they are on entry; then the estimates
//   moved by this batch's per-group extrema (the single-pass forward).
//
// A row lives in the registers of a group of LPR lanes (VPL vectors of 8 columns per lane), as in the
// backward kernel; the two row sums are lane-group reductions.  A lane always holds the same columns, hence
// the same channel groups: its extrema accumulate in registers over all its rows and reach LDS once.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "api_util.hpp"
#include "common.hpp"
#include "quantize.hpp"

namespace mesa {

constexpr int kLfMaxGroups = 1024;
constexpr int kLfRows = 2;          // rows per lane group in flight

template <typename T, int LPR, int VPL, bool SR>
__global__ __launch_bounds__(kThreads, 3) void k_layernorm_fwd(const void *__restrict__ x, void *__restrict__ y,
                                                               int8_t *__restrict__ q, float *__restrict__ mean,
                                                               float *__restrict__ rstd, const void *__restrict__ gamma,
                                                               const void *__restrict__ bias, float eps, int64_t M, uint32_t D,
                                                               FastDiv div_vpg, uint32_t groups, float inv_D,
                                                               const float *__restrict__ alpha, const float *__restrict__ beta,
                                                               uint64_t seed, uint64_t offset, float *__restrict__ part)
{
    constexpr int RPW = 64 / LPR;                   // rows per wave and pass
    constexpr int kWaves = kThreads / 64;
    constexpr int kBlockRows = kWaves * kLfRows * RPW;
    __shared__ int lmn[kLfMaxGroups], lmx[kLfMaxGroups];
    for (uint32_t g = threadIdx.x; g < groups; g += kThreads) {
        lmn[g] = order_key(__builtin_inff());
        lmx[g] = order_key(-__builtin_inff());
    }
    __syncthreads();

    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint32_t sub = lane / LPR, l = lane % LPR;
    const uint32_t vpr = D / kVec;

    // gamma and bias stay in registers for rows of up to 1024 elements; for longer rows they are read again for
    // every row (a few KB that stay in the cache), which costs less than the registers would
    constexpr bool kKeep = VPL <= 2 || (VPL == 3 && Store<T>::kBytes == 2);
    constexpr int kHeld = kKeep ? VPL : 1;
    uint32_t col[VPL], grp[VPL];
    bool act[VPL];
    float gam[kHeld][8], bia[kHeld][8], mn[VPL], mx[VPL];
    float2 prm[VPL];                                // (255 / alpha, beta) of the vector's channel group
#pragma unroll
    for (int k = 0; k < VPL; ++k) {
        const uint32_t cv = k * LPR + l;
        act[k] = cv < vpr;
        col[k] = cv * kVec;
        grp[k] = 0;
        mn[k] = __builtin_inff();
        mx[k] = -__builtin_inff();
        prm[k] = make_float2(0.0f, 0.0f);
        if (kKeep) {
#pragma unroll
            for (int j = 0; j < 8; ++j) { gam[k % kHeld][j] = 0.0f; bia[k % kHeld][j] = 0.0f; }
        }
        if (act[k]) {
            if (kKeep) {
                Store<T>::unpack(Store<T>::load(gamma, col[k]), gam[k % kHeld]);
                Store<T>::unpack(Store<T>::load(bias, col[k]), bia[k % kHeld]);
            }
            grp[k] = fastdiv(cv, div_vpg);
            const float a = alpha[grp[k]];
            prm[k] = make_float2(a > 0.0f ? 255.0f / a : 0.0f, beta[grp[k]]);
        }
    }

    const int64_t stride = int64_t(gridDim.x) * kBlockRows;
    for (int64_t base = int64_t(blockIdx.x) * kBlockRows; base < M; base += stride) {
        typename Store<T>::raw_t raw[kLfRows][VPL];
        const typename Store<T>::raw_t zero = Store<T>::pack((const float[8]){0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f});
#pragma unroll
        for (int p = 0; p < kLfRows; ++p) {
            const int64_t row = base + int64_t((p * kWaves + wave) * RPW + sub);
#pragma unroll
            for (int k = 0; k < VPL; ++k) {
                raw[p][k] = zero;                   // lanes without a row or a vector work on zeros; only loads and stores are predicated
                if (row < M && act[k]) raw[p][k] = Nt<T>::load(x, row * D + col[k]);
            }
        }
#pragma unroll
        for (int p = 0; p < kLfRows; ++p) {
            const int64_t row = base + int64_t((p * kWaves + wave) * RPW + sub);
            const bool ok = row < M;
            float f[VPL][8];
            float s1 = 0.0f;
#pragma unroll
            for (int k = 0; k < VPL; ++k) {
                Store<T>::unpack(raw[p][k], f[k]);
#pragma unroll
                for (int j = 0; j < 8; ++j) s1 += f[k][j];
            }
            const float mu = lanes_sum_dpp<LPR>(s1) * inv_D;
            float s2 = 0.0f;
#pragma unroll
            for (int k = 0; k < VPL; ++k)
                if (act[k]) {                       // columns past the row's end would add mu^2 each
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const float d = f[k][j] - mu;
                        s2 = fmaf(d, d, s2);
                    }
                }
            const float var = lanes_sum_dpp<LPR>(s2) * inv_D;
            const float rs = 1.0f / sqrtf(var + eps);
            if (ok && l == 0) {
                mean[row] = mu;
                rstd[row] = rs;
            }
#pragma unroll
            for (int k = 0; k < VPL; ++k) {
                if (ok && act[k]) {
                    const int64_t e = row * D + col[k];
                    float o[8], w[8], bits[8];
                    if (!kKeep) {
                        Store<T>::unpack(Store<T>::load(gamma, col[k]), gam[0]);
                        Store<T>::unpack(Store<T>::load(bias, col[k]), bia[0]);
                    }
#pragma unroll
                    for (int j = 0; j < 8; ++j) o[j] = fmaf((f[k][j] - mu) * rs, gam[k % kHeld][j], bia[k % kHeld][j]);
                    Nt<T>::store(y, e, Store<T>::pack(o));
                    if (SR) sr_bits(seed, offset + uint64_t(e >> 3), bits);
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        w[j] = quantize_one<SR>(f[k][j], prm[k].x, prm[k].y, SR ? bits[j] : 0.0f);
                        mn[k] = vmin(mn[k], f[k][j]);
                        mx[k] = vmax(mx[k], f[k][j]);
                    }
                    nt_store<u32x2>(q + e, pack_codes(w));
                }
            }
        }
    }

    // this thread's extrema to its groups' slots, the workgroup's to its row of the partials
#pragma unroll
    for (int k = 0; k < VPL; ++k)
        if (act[k] && mn[k] <= mx[k]) {
            atomicMin(&lmn[grp[k]], order_key(mn[k]));
            atomicMax(&lmx[grp[k]], order_key(mx[k]));
        }
    __syncthreads();
    float *out = part + int64_t(blockIdx.x) * 2 * groups;
    for (uint32_t g = threadIdx.x; g < groups; g += kThreads) {
        out[g] = order_val(lmn[g]);
        out[groups + g] = order_val(lmx[g]);
    }
}

struct LfPlan {
    bool ok;
    int lpr, vpl, grid;
};

static LfPlan lf_plan(int64_t M, int64_t D)
{
    LfPlan p{};
    const int64_t vpr = D / kVec;
    p.ok = D % kVec == 0 && vpr >= 1 && vpr <= 256;
    if (!p.ok) return p;
    // lanes per row (a power of two) x vectors per lane with the fewest idle slots: three vectors per lane fit the
    // widths of the paper's models (96, 192, 384, 768 = 3 * 2^k vectors of 8) exactly, where a power of two wastes a quarter
    int best = 1 << 30;
    for (int vpl = 1; vpl <= 4; ++vpl) {
        int lpr = 8;                                           // at least 128 contiguous bytes of a row per load instruction
        while (int64_t(lpr) * vpl < vpr) lpr *= 2;
        if (lpr > 64 || (vpl == 4 && lpr != 64)) continue;     // four vectors per lane: only for the longest rows
        if (lpr * vpl < best) { best = lpr * vpl; p.lpr = lpr; p.vpl = vpl; }
    }
    const int64_t block_rows = int64_t(kThreads / 64) * kLfRows * (64 / p.lpr);
    const int64_t wgs = ceil_div(M, block_rows);
    const int64_t resident = 256 * 3;
    p.grid = int(wgs < resident ? wgs : resident);
    return p;
}

// Rows the kernel above does not take (lengths or groups that are no multiples of 8, rows beyond 2048 elements, more
// groups than its tables hold): mean, 1/sqrt(var + eps) and y by a plain kernel -- one workgroup per row, the row read
// three times, sums added in a fixed order --, the codes and the estimates by the single-pass quantizer on x, which is
// how the call is defined.
template <typename T>
__global__ __launch_bounds__(kThreads) void k_layernorm_fwd_plain_y(const void *__restrict__ x, void *__restrict__ y,
                                                                    float *__restrict__ mean, float *__restrict__ rstd,
                                                                    const void *__restrict__ gamma, const void *__restrict__ bias,
                                                                    float eps, int64_t M, uint32_t D)
{
    __shared__ float red[kThreads / 64];
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    auto block_sum = [&](float v) {   // the same value in every thread
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
        if (lane == 0) red[wave] = v;
        __syncthreads();
        float r = red[0];
#pragma unroll
        for (int w = 1; w < kThreads / 64; ++w) r += red[w];
        __syncthreads();
        return r;
    };
    const float inv_D = 1.0f / float(D);
    for (int64_t row = blockIdx.x; row < M; row += gridDim.x) {
        const int64_t e0 = row * int64_t(D);
        float s1 = 0.0f;
        for (uint32_t c = threadIdx.x; c < D; c += kThreads) s1 += Store<T>::load1(x, e0 + c);
        const float mu = block_sum(s1) * inv_D;
        float s2 = 0.0f;
        for (uint32_t c = threadIdx.x; c < D; c += kThreads) {
            const float d = Store<T>::load1(x, e0 + c) - mu;
            s2 = fmaf(d, d, s2);
        }
        const float rs = 1.0f / sqrtf(block_sum(s2) * inv_D + eps);
        if (threadIdx.x == 0) { mean[row] = mu; rstd[row] = rs; }
        for (uint32_t c = threadIdx.x; c < D; c += kThreads) {
            const float xn = (Store<T>::load1(x, e0 + c) - mu) * rs;
            Store<T>::store1(y, e0 + c, fmaf(xn, Store<T>::load1(gamma, c), Store<T>::load1(bias, c)));
        }
    }
}

static bool lf_two_step(const LfPlan &p, int64_t D, int64_t G) { return !p.ok || (D / G) % kVec != 0 || G > kLfMaxGroups; }

size_t layernorm_fwd_ws_bytes(int64_t M, int64_t D, int64_t G)
{
    if (M <= 0 || D <= 0 || G <= 0 || D % G != 0) return 16;
    const LfPlan p = lf_plan(M, D);
    if (lf_two_step(p, D, G)) return update_ws_bytes(M, G, D / G) + 16;
    return size_t(p.grid) * 2 * size_t(G) * sizeof(float) + 16;
}

}  // namespace mesa

using namespace mesa;

extern "C" MESA_EXPORT mesa_status mesa_layernorm_fwd_q(const void *x, int64_t M, int64_t D, int64_t G, const void *gamma,
                                                        const void *bias, float eps, float *alpha, float *beta, float lambda, void *y,
                                                        float *mean, float *rstd, int8_t *q, mesa_round mode, uint64_t seed,
                                                        uint64_t offset, void *ws, size_t ws_bytes, mesa_dtype dt, void *stream)
{
    if (!valid_dtype(dt) || M < 0 || D < 0 || G < 0) return MESA_ERR_INVALID_ARG;
    if (mode != MESA_ROUND_NEAREST_EVEN && mode != MESA_ROUND_STOCHASTIC) return MESA_ERR_INVALID_ARG;
    if (!(lambda >= 0.0f && lambda <= 1.0f) || !(eps >= 0.0f)) return MESA_ERR_INVALID_ARG;
    if (M == 0 || D == 0) return MESA_OK;
    if (G == 0 || D % G != 0) return MESA_ERR_INVALID_ARG;
    if (!x || !y || !q || !mean || !rstd || !gamma || !bias || !alpha || !beta || !aligned16(x) || !aligned16(y) || !aligned16(q) ||
        !aligned16(gamma) || !aligned16(bias) || !aligned4(mean) || !aligned4(rstd) || !aligned4(alpha) || !aligned4(beta) || y == x)
        return MESA_ERR_INVALID_ARG;
    const LfPlan p = lf_plan(M, D);
    if (M >= (int64_t(1) << 40) || D >= (int64_t(1) << 31)) return MESA_ERR_UNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (lf_two_step(p, D, G)) {
        // the single-pass quantizer checks its own limits (up to 4096 groups) before it launches anything; y follows
        const mesa_layout L = {M, G, D / G};
        const mesa_status st = mesa_quantize_update_fused(x, dt, L, alpha, beta, lambda, q, mode, seed, offset, ws, ws_bytes, stream);
        if (st != MESA_OK) return st;
        const unsigned grid = unsigned(M < (int64_t(1) << 20) ? M : (int64_t(1) << 20));
#define MESA_LAUNCH_LP(T) \
        hipLaunchKernelGGL((k_layernorm_fwd_plain_y<T>), dim3(grid), dim3(kThreads), 0, s, x, y, mean, rstd, gamma, bias, eps, M, uint32_t(D))
        MESA_FOR_DTYPE(dt, MESA_LAUNCH_LP);
#undef MESA_LAUNCH_LP
        return launch_status();
    }
    if (!ws || !aligned16(ws) || ws_bytes < layernorm_fwd_ws_bytes(M, D, G)) return MESA_ERR_WORKSPACE;
    float *part = static_cast<float *>(ws);
    FastDiv dv = make_fastdiv(uint32_t((D / G) / kVec));
    const float inv_D = 1.0f / float(D);
    const bool sr = mode == MESA_ROUND_STOCHASTIC;
#define MESA_LAUNCH_LF(T, LPR_, VPL_, SR_) \
    hipLaunchKernelGGL((k_layernorm_fwd<T, LPR_, VPL_, SR_>), dim3(p.grid), dim3(kThreads), 0, s, x, y, q, mean, rstd, gamma, bias, eps, M, \
                       uint32_t(D), dv, uint32_t(G), inv_D, alpha, beta, seed, offset, part)
#define MESA_LAUNCH_LF_S(T, LPR_, VPL_) \
    do { if (sr) MESA_LAUNCH_LF(T, LPR_, VPL_, true); else MESA_LAUNCH_LF(T, LPR_, VPL_, false); } while (0)
#define MESA_LAUNCH_LF_T(T) \
    do { \
        if (p.vpl == 4) MESA_LAUNCH_LF_S(T, 64, 4); \
        else if (p.vpl == 3 && p.lpr == 8) MESA_LAUNCH_LF_S(T, 8, 3); \
        else if (p.vpl == 3 && p.lpr == 16) MESA_LAUNCH_LF_S(T, 16, 3); \
        else if (p.vpl == 3 && p.lpr == 32) MESA_LAUNCH_LF_S(T, 32, 3); \
        else if (p.vpl == 3) MESA_LAUNCH_LF_S(T, 64, 3); \
        else if (p.vpl == 2) MESA_LAUNCH_LF_S(T, 64, 2);   /* two vectors per lane never win below 64 lanes */ \
        else if (p.lpr == 8) MESA_LAUNCH_LF_S(T, 8, 1); \
        else if (p.lpr == 16) MESA_LAUNCH_LF_S(T, 16, 1); \
        else if (p.lpr == 32) MESA_LAUNCH_LF_S(T, 32, 1); \
        else MESA_LAUNCH_LF_S(T, 64, 1); \
    } while (0)
    MESA_FOR_DTYPE(dt, MESA_LAUNCH_LF_T);
#undef MESA_LAUNCH_LF_T
#undef MESA_LAUNCH_LF_S
#undef MESA_LAUNCH_LF
    if (launch_status() != MESA_OK) return MESA_ERR_LAUNCH;   // the consumer must not run on a workspace nobody wrote
    launch_ema_finalize(part, p.grid, uint32_t(G), alpha, beta, lambda, 0, 0, 0.0f, s);
    return launch_status();
}
