// layernorm_bwd.hip -- LayerNorm backward at the de-quantized input (Sec. 3.1 Eq. 2):
//   xn = (x_hat - mean)*rstd,  g = dy*gamma,
//   dx = rstd*(g - mean_j(g) - xn*mean_j(g*xn)),   dgamma_j = sum_rows dy*xn,  dbeta_j = sum_rows dy.
//
// A workgroup takes tiles of R whole rows (R*D <= 4096 elements) and reads them flat as 8-element
// vectors; codes and dy stay in registers between the reduction pass and the output pass, two
// partial sums per vector go through LDS (16 lanes per row add them in a fixed order).  A thread
// meets the same columns in every tile, so it keeps its share of the column sums in registers
// for the whole kernel; they are combined per workgroup in LDS, written as partials, and a small
// second kernel adds the partials of all workgroups -- fixed order throughout, no float atomics.
#include <hip/hip_runtime.h>

#include "api_util.hpp"
#include "common.hpp"

namespace mesa {

constexpr int kLnU = 2;
constexpr int kLnTileVec = kThreads * kLnU;   // 512 vectors = 4096 elements
constexpr int kLnMaxGroups = kLnTileVec;      // (D/G) % 8 == 0 and D <= 4096
constexpr int kLnGridCap = 512;

template <typename T>
__global__ __launch_bounds__(kThreads) void k_layernorm_bwd(const int8_t *__restrict__ xq, const void *dy, void *dx,
                                                            const void *__restrict__ gamma, const float *__restrict__ mean,
                                                            const float *__restrict__ rstd, const float *__restrict__ alpha,
                                                            const float *__restrict__ beta, int64_t M, uint32_t D,
                                                            uint32_t R, int64_t tiles, uint32_t groups, FastDiv div_vpr,
                                                            FastDiv div_vpg, float inv_D, float *__restrict__ part)
{
    __shared__ float2 tab[kLnMaxGroups];
    __shared__ float P1[kLnTileVec], P2[kLnTileVec];
    __shared__ float C1[kLnTileVec], C2[kLnTileVec];
    __shared__ float colG[kLnTileVec * kVec], colB[kLnTileVec * kVec];   // [slot r][D], R*D <= 4096

    const uint32_t tid = threadIdx.x;
    const uint32_t vpr = div_vpr.d;   // vectors per row = D/8
    for (uint32_t g = tid; g < groups; g += kThreads) tab[g] = make_float2(alpha[g] / 255.0f, beta[g]);

    // this thread's fixed place in every tile
    uint32_t rr[kLnU], col[kLnU];
    bool act[kLnU];
    float gam[kLnU][8], accG[kLnU][8], accB[kLnU][8];
    float2 prm[kLnU];
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kLnU; ++u) {
        const uint32_t v = u * kThreads + tid;
        act[u] = v < R * vpr;
        rr[u] = fastdiv(v, div_vpr);
        const uint32_t cv = v - rr[u] * vpr;
        col[u] = cv * kVec;
#pragma unroll
        for (int j = 0; j < 8; ++j) { gam[u][j] = 0.0f; accG[u][j] = 0.0f; accB[u][j] = 0.0f; }
        prm[u] = make_float2(0.0f, 0.0f);
        if (act[u]) {
            Store<T>::unpack(Store<T>::load(gamma, col[u]), gam[u]);
            prm[u] = tab[fastdiv(cv, div_vpg)];
        }
    }

    for (int64_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
        const int64_t row0 = tile * R;
        const uint32_t nrows = uint32_t((M - row0 < int64_t(R)) ? (M - row0) : int64_t(R));

        u32x2 cq[kLnU];
        typename Store<T>::raw_t cd[kLnU];
        float mu[kLnU], rs[kLnU];
#pragma unroll
        for (int u = 0; u < kLnU; ++u) {
            const uint32_t v = u * kThreads + tid;
            if (act[u] && rr[u] < nrows) {
                const int64_t row = row0 + rr[u];
                const int64_t e = row * D + col[u];
                cq[u] = load_codes8(xq, e);
                cd[u] = Store<T>::load(dy, e);
                mu[u] = mean[row];
                rs[u] = rstd[row];
                float y[8], d[8];
                codes_to_float(cq[u], y);
                Store<T>::unpack(cd[u], d);
                float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float xn = (fmaf(y[j], prm[u].x, prm[u].y) - mu[u]) * rs[u];
                    const float gg = d[j] * gam[u][j];
                    s1 += gg;
                    s2 = fmaf(gg, xn, s2);
                    accG[u][j] = fmaf(d[j], xn, accG[u][j]);
                    accB[u][j] += d[j];
                }
                P1[v] = s1;
                P2[v] = s2;
            }
        }
        __syncthreads();
        {
            const uint32_t lane16 = tid & 15u;
            for (uint32_t r = tid >> 4; r < nrows; r += kThreads / 16) {
                float s1 = 0.0f, s2 = 0.0f;
                for (uint32_t k = lane16; k < vpr; k += 16) { s1 += P1[r * vpr + k]; s2 += P2[r * vpr + k]; }
                s1 = lanes_sum<16>(s1);
                s2 = lanes_sum<16>(s2);
                if (lane16 == 0) { C1[r] = s1 * inv_D; C2[r] = s2 * inv_D; }
            }
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < kLnU; ++u) {
            if (act[u] && rr[u] < nrows) {
                const int64_t e = (row0 + rr[u]) * D + col[u];
                const float c1 = C1[rr[u]], c2 = C2[rr[u]];
                float y[8], d[8], o[8];
                codes_to_float(cq[u], y);
                Store<T>::unpack(cd[u], d);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float xn = (fmaf(y[j], prm[u].x, prm[u].y) - mu[u]) * rs[u];
                    const float gg = d[j] * gam[u][j];
                    o[j] = rs[u] * (gg - c1 - xn * c2);
                }
                Store<T>::store(dx, e, Store<T>::pack(o));
            }
        }
        __syncthreads();
    }

    // column sums of this workgroup: slot r of the tile holds what its threads gathered
#pragma unroll
    for (int u = 0; u < kLnU; ++u) {
        if (act[u]) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                colG[rr[u] * D + col[u] + j] = accG[u][j];
                colB[rr[u] * D + col[u] + j] = accB[u][j];
            }
        }
    }
    __syncthreads();
    float *pg = part + int64_t(blockIdx.x) * 2 * D;
    for (uint32_t c = tid; c < D; c += kThreads) {
        float sg = 0.0f, sb = 0.0f;
        for (uint32_t r = 0; r < R; ++r) { sg += colG[r * D + c]; sb += colB[r * D + c]; }
        pg[c] = sg;
        pg[D + c] = sb;
    }
}

// dgamma / dbeta = sum over workgroups of their partial column sums; 64 columns per workgroup,
// four interleaved slices of the workgroup list, combined in a fixed order
__global__ __launch_bounds__(kThreads) void k_layernorm_finalize(const float *__restrict__ part, int nwg, uint32_t D,
                                                                 float *__restrict__ dgamma, float *__restrict__ dbeta)
{
    __shared__ float sg[4][64], sb[4][64];
    const uint32_t c = blockIdx.x * 64 + (threadIdx.x & 63u);
    const uint32_t k = threadIdx.x >> 6;
    float ag = 0.0f, ab = 0.0f;
    if (c < D)
        for (int w = k; w < nwg; w += 4) {
            ag += part[int64_t(w) * 2 * D + c];
            ab += part[int64_t(w) * 2 * D + D + c];
        }
    sg[k][threadIdx.x & 63u] = ag;
    sb[k][threadIdx.x & 63u] = ab;
    __syncthreads();
    if (k == 0 && c < D) {
        const uint32_t i = threadIdx.x;
        dgamma[c] = ((sg[0][i] + sg[1][i]) + sg[2][i]) + sg[3][i];
        dbeta[c] = ((sb[0][i] + sb[1][i]) + sb[2][i]) + sb[3][i];
    }
}

static int ln_plan(int64_t M, int64_t D, int64_t *R_out, int64_t *tiles_out)
{
    int64_t R = int64_t(kLnTileVec) * kVec / D;
    if (R > M) R = M;
    if (R < 1) R = 1;
    int64_t tiles = ceil_div(M, R);
    *R_out = R;
    *tiles_out = tiles;
    return int(tiles < kLnGridCap ? tiles : kLnGridCap);
}

size_t layernorm_ws_bytes(int64_t M, int64_t D)
{
    if (M <= 0 || D <= 0 || D > int64_t(kLnTileVec) * kVec) return 16;
    int64_t R, tiles;
    int grid = ln_plan(M, D, &R, &tiles);
    return size_t(grid) * 2 * size_t(D) * sizeof(float);
}

}  // namespace mesa

using namespace mesa;

extern "C" MESA_EXPORT mesa_status mesa_layernorm_bwd_q(const int8_t *xq, int64_t M, int64_t D, int64_t G, const float *alpha,
                                                        const float *beta, const float *mean, const float *rstd,
                                                        const void *gamma, const void *dy, void *dx, float *dgamma,
                                                        float *dbeta, mesa_dtype dt, void *ws, size_t ws_bytes, void *stream)
{
    if (!valid_dtype(dt) || M < 0 || D < 0 || G < 0) return MESA_ERR_INVALID_ARG;
    if (M == 0 || D == 0) return MESA_OK;
    if (G == 0 || D % G != 0) return MESA_ERR_INVALID_ARG;
    if (!xq || !alpha || !beta || !mean || !rstd || !gamma || !dy || !dx || !dgamma || !dbeta) return MESA_ERR_INVALID_ARG;
    if (!aligned16(xq) || !aligned16(dy) || !aligned16(dx) || !aligned16(gamma) || !aligned4(alpha) || !aligned4(beta) ||
        !aligned4(mean) || !aligned4(rstd) || !aligned4(dgamma) || !aligned4(dbeta))
        return MESA_ERR_INVALID_ARG;
    if (D % kVec != 0 || (D / G) % kVec != 0 || D > int64_t(kLnTileVec) * kVec) return MESA_ERR_UNSUPPORTED;
    if (!ws || !aligned16(ws) || ws_bytes < layernorm_ws_bytes(M, D)) return MESA_ERR_WORKSPACE;
    int64_t R, tiles;
    const int grid = ln_plan(M, D, &R, &tiles);
    FastDiv dvpr = make_fastdiv(uint32_t(D / kVec)), dvpg = make_fastdiv(uint32_t(D / G / kVec));
    hipStream_t s = static_cast<hipStream_t>(stream);
    float *part = static_cast<float *>(ws);
    const float inv_D = 1.0f / float(D);
    if (dt == MESA_F16)
        hipLaunchKernelGGL((k_layernorm_bwd<_Float16>), dim3(grid), dim3(kThreads), 0, s, xq, dy, dx, gamma, mean, rstd, alpha,
                           beta, M, uint32_t(D), uint32_t(R), tiles, uint32_t(G), dvpr, dvpg, inv_D, part);
    else
        hipLaunchKernelGGL((k_layernorm_bwd<float>), dim3(grid), dim3(kThreads), 0, s, xq, dy, dx, gamma, mean, rstd, alpha,
                           beta, M, uint32_t(D), uint32_t(R), tiles, uint32_t(G), dvpr, dvpg, inv_D, part);
    hipLaunchKernelGGL(k_layernorm_finalize, dim3(int(ceil_div(D, 64))), dim3(kThreads), 0, s, part, grid, uint32_t(D), dgamma,
                       dbeta);
    return launch_status();
}
