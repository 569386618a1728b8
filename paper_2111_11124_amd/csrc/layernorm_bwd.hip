// layernorm_bwd.hip -- LayerNorm backward at the de-quantized input (Sec. 3.1 Eq. 2):
//   xn = (x_hat - mean)*rstd,  g = dy*gamma,
//   dx = rstd*(g - mean_j(g) - xn*mean_j(g*xn)),   dgamma_j = sum_rows dy*xn,  dbeta_j = sum_rows dy.
//
// Rows of up to 1024 elements (the usual case): a row lives in an aligned group of 8..64 lanes of
// one wave, one or two 8-element vectors per lane, so the two row means are lane-group sums taken
// inside the adder instructions -- no LDS, no barrier, nothing between the loads and the stores
// but arithmetic.  A wave has several rows in flight and a workgroup walks a contiguous run of
// rows.  A lane meets the same columns in every row, so it keeps its share of the column sums
// (dgamma, dbeta) in registers for the whole kernel; they are combined per workgroup in LDS,
// written as partials, and a small second kernel adds the partials of all workgroups -- fixed
// order throughout, no float atomics.
// Longer rows (up to 4096 elements): a workgroup takes one row at a time, reads it flat as
// 8-element vectors, and the row sums go through LDS.
#include <hip/hip_runtime.h>

#include "api_util.hpp"
#include "common.hpp"

namespace mesa {

constexpr int kLnU = 2;                 // vectors per thread in a tile
constexpr int kLnGridCap = 1024;
constexpr int kLnMaxD = kThreads * kLnU * kVec;   // 4096: a row must fit a workgroup tile
constexpr int kLnRowsInFlight = 2;      // wave-row kernel: row groups a wave has in flight
// ... and the workgroups per CU its register budget is set for (two blocks of rows live at a time)
constexpr int ln_rows_wg_per_cu(size_t elem_bytes, int vpl) { return vpl == 1 ? (elem_bytes == 2 ? 4 : 3) : 2; }
constexpr int kLnFinThreads = 1024;               // finalize: 32 columns x 32 slices of the workgroup list

template <int TPT> __device__ __forceinline__ void ln_sync()
{
    if (TPT == kThreads) {
        __syncthreads();
    } else {  // one wave owns the tile: order its own LDS traffic, nothing more
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
}

__device__ __forceinline__ void ln_opaque(u32x2 &a, u32x4 &b) { asm volatile("" : "+v"(a), "+v"(b)); }
__device__ __forceinline__ void ln_opaque(u32x2 &a, Store<float>::raw_t &b)
{
    asm volatile("" : "+v"(a), "+v"(b.lo), "+v"(b.hi));
}

// Rows inside a wave.  LPR lanes per row (a power of two), VPL vectors per lane: lane l of a row's
// group holds the vectors l, l + LPR, ... of the row.  RPW = 64/LPR rows per wave at a time, U such
// groups in flight; the four waves of a workgroup take neighbouring row groups, so that what the
// workgroup has in flight is one contiguous block of rows, and the workgroups stride over the blocks.
template <typename T, int LPR, int VPL>
__global__ __launch_bounds__(kThreads, ln_rows_wg_per_cu(sizeof(T), VPL)) void k_layernorm_bwd_rows(const int8_t *__restrict__ xq, const void *dy, void *dx,
                                                                    const void *__restrict__ gamma, const float *__restrict__ mean,
                                                                    const float *__restrict__ rstd, const float *__restrict__ alpha,
                                                                    const float *__restrict__ beta, int64_t M, uint32_t D,
                                                                    FastDiv div_vpg, float inv_D,
                                                                    float *__restrict__ part)
{
    constexpr int RPW = 64 / LPR;
    constexpr int U = kLnRowsInFlight;
    constexpr int kWaves = kThreads / 64;
    constexpr int kBlockRows = kWaves * U * RPW;     // rows a workgroup has in flight
    __shared__ float colG[kLnMaxD], colB[kLnMaxD];   // [wave][row slot][D]: kWaves * RPW * D <= 4096

    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint32_t sub = lane / LPR, l = lane % LPR;
    const uint32_t vpr = D / kVec;

    uint32_t col[VPL];
    bool act[VPL];
    float gam[VPL][8], accG[VPL][8], accB[VPL][8];
    float2 prm[VPL];
#pragma unroll
    for (int k = 0; k < VPL; ++k) {
        const uint32_t cv = k * LPR + l;
        act[k] = cv < vpr;
        col[k] = cv * kVec;
#pragma unroll
        for (int j = 0; j < 8; ++j) { gam[k][j] = 0.0f; accG[k][j] = 0.0f; accB[k][j] = 0.0f; }
        prm[k] = make_float2(0.0f, 0.0f);
        if (act[k]) {
            Store<T>::unpack(Store<T>::load(gamma, col[k]), gam[k]);
            const uint32_t g = fastdiv(cv, div_vpg);
            prm[k] = make_float2(alpha[g] / 255.0f, beta[g]);
        }
    }

    // One block of rows is in registers while the previous one is worked on: the loads of block
    // i+1 are issued before the arithmetic, the lane-group sums and the stores of block i.
    // Lanes without a row or a vector work on zeros: dy = 0 adds nothing to any sum, and only the
    // loads and the stores are predicated.
    struct Block {
        u32x2 cq[U][VPL];
        typename Store<T>::raw_t cd[U][VPL];
        float mu[U], rs[U];
    };
    const typename Store<T>::raw_t zero_d = Store<T>::pack((const float[8]){0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f});
    auto load_block = [&](int64_t base, Block &blk) {
#pragma unroll
        for (int p = 0; p < U; ++p) {
            const int64_t row = base + int64_t((p * kWaves + wave) * RPW + sub);
            const bool ok = row < M;
            blk.mu[p] = 0.0f;
            blk.rs[p] = 0.0f;
            if (ok) { blk.mu[p] = mean[row]; blk.rs[p] = rstd[row]; }
#pragma unroll
            for (int k = 0; k < VPL; ++k) {
                blk.cq[p][k] = u32x2{0u, 0u};
                blk.cd[p][k] = zero_d;
                if (ok && act[k]) {
                    const int64_t e = row * D + col[k];
                    blk.cq[p][k] = nt_load<u32x2>(xq + e);
                    blk.cd[p][k] = Nt<T>::load(dy, e);
                }
            }
        }
    };
    const int64_t stride = int64_t(gridDim.x) * kBlockRows;
    int64_t base = int64_t(blockIdx.x) * kBlockRows;
    Block cur, nxt;
    if (base < M) load_block(base, cur);
    for (; base < M; base += stride) {
        load_block(base + stride, nxt);    // past the last block: every row fails its check, nothing is read
#pragma unroll
        for (int p = 0; p < U; ++p) {
            const int64_t row = base + int64_t((p * kWaves + wave) * RPW + sub);
            const bool ok = row < M;
            float xn[VPL][8], gg[VPL][8];
            float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
            for (int k = 0; k < VPL; ++k) {
                float y[8], d[8];
                codes_to_float(cur.cq[p][k], y);
                Store<T>::unpack(cur.cd[p][k], d);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    xn[k][j] = (fmaf(y[j], prm[k].x, prm[k].y) - cur.mu[p]) * cur.rs[p];
                    gg[k][j] = d[j] * gam[k][j];
                    s1 += gg[k][j];
                    s2 = fmaf(gg[k][j], xn[k][j], s2);
                    accG[k][j] = fmaf(d[j], xn[k][j], accG[k][j]);
                    accB[k][j] += d[j];
                }
            }
            const float c1 = lanes_sum_dpp<LPR>(s1) * inv_D;
            const float c2 = lanes_sum_dpp<LPR>(s2) * inv_D;
#pragma unroll
            for (int k = 0; k < VPL; ++k) {
                float o[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) o[j] = cur.rs[p] * (gg[k][j] - c1 - xn[k][j] * c2);
                if (ok && act[k]) Nt<T>::store(dx, row * D + col[k], Store<T>::pack(o));
            }
        }
        cur = nxt;
    }

    // column sums of this workgroup: slot (wave, sub) holds what its lanes gathered
#pragma unroll
    for (int k = 0; k < VPL; ++k) {
        if (act[k]) {
            const uint32_t o = (wave * RPW + sub) * D + col[k];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                colG[o + j] = accG[k][j];
                colB[o + j] = accB[k][j];
            }
        }
    }
    __syncthreads();
    float *pg = part + int64_t(blockIdx.x) * 2 * D;
    for (uint32_t c = threadIdx.x; c < D; c += kThreads) {
        float sg = 0.0f, sb = 0.0f;
#pragma unroll
        for (uint32_t r = 0; r < kWaves * RPW; ++r) { sg += colG[r * D + c]; sb += colB[r * D + c]; }
        pg[c] = sg;
        pg[D + c] = sb;
    }
}

// Long rows.  TPT threads (the workgroup) own a tile of R rows (R = 1 for rows this long).
template <typename T, int TPT>
__global__ __launch_bounds__(kThreads, 4) void k_layernorm_bwd(const int8_t *__restrict__ xq, const void *dy, void *dx,
                                                               const void *__restrict__ gamma, const float *__restrict__ mean,
                                                               const float *__restrict__ rstd, const float *__restrict__ alpha,
                                                               const float *__restrict__ beta, int64_t M, uint32_t D,
                                                               uint32_t R, int64_t tiles, uint32_t groups, FastDiv div_vpr,
                                                               FastDiv div_vpg, float inv_D, float *__restrict__ part)
{
    constexpr int kTileVec = TPT * kLnU;
    constexpr int kTeams = kThreads / TPT;
    __shared__ float P1[kTeams][kTileVec], P2[kTeams][kTileVec];
    __shared__ float C1[kTeams][kTileVec], C2[kTeams][kTileVec];
    __shared__ float colG[kLnMaxD], colB[kLnMaxD];   // [team][slot r][D]: kTeams * R * D <= 4096

    const uint32_t team = threadIdx.x / TPT;
    const uint32_t tid = threadIdx.x % TPT;
    const uint32_t vpr = div_vpr.d;   // vectors per row = D/8
    float *p1 = P1[team], *p2 = P2[team], *c1s = C1[team], *c2s = C2[team];

    // this thread's fixed place in every tile: row slot rr, columns col..col+7
    uint32_t rr[kLnU], col[kLnU];
    bool act[kLnU];
    float gam[kLnU][8], accG[kLnU][8], accB[kLnU][8];
    float2 prm[kLnU];
#pragma unroll
    for (int u = 0; u < kLnU; ++u) {
        const uint32_t v = u * TPT + tid;
        act[u] = v < R * vpr;
        rr[u] = fastdiv(v, div_vpr);
        const uint32_t cv = v - rr[u] * vpr;
        col[u] = cv * kVec;
#pragma unroll
        for (int j = 0; j < 8; ++j) { gam[u][j] = 0.0f; accG[u][j] = 0.0f; accB[u][j] = 0.0f; }
        prm[u] = make_float2(0.0f, 0.0f);
        if (act[u]) {
            Store<T>::unpack(Store<T>::load(gamma, col[u]), gam[u]);
            const uint32_t g = fastdiv(cv, div_vpg);
            prm[u] = make_float2(alpha[g] / 255.0f, beta[g]);
        }
    }

    for (int64_t tile = int64_t(blockIdx.x) * kTeams + team; tile < tiles; tile += int64_t(gridDim.x) * kTeams) {
        const int64_t row0 = tile * R;
        const uint32_t nrows = uint32_t((M - row0 < int64_t(R)) ? (M - row0) : int64_t(R));

        u32x2 cq[kLnU];
        typename Store<T>::raw_t cd[kLnU];
        float mu[kLnU], rs[kLnU];
#pragma unroll
        for (int u = 0; u < kLnU; ++u) {
            if (act[u] && rr[u] < nrows) {
                const int64_t row = row0 + rr[u];
                const int64_t e = row * D + col[u];
                cq[u] = nt_load<u32x2>(xq + e);
                cd[u] = Nt<T>::load(dy, e);
                mu[u] = mean[row];
                rs[u] = rstd[row];
            }
        }
#pragma unroll
        for (int u = 0; u < kLnU; ++u) {
            const uint32_t v = u * TPT + tid;
            if (act[u] && rr[u] < nrows) {
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
                p1[v] = s1;
                p2[v] = s2;
            }
        }
        ln_sync<TPT>();
        {
            const uint32_t lane16 = tid & 15u;
            for (uint32_t r = tid >> 4; r < nrows; r += TPT / 16) {
                float s1 = 0.0f, s2 = 0.0f;
                for (uint32_t k = lane16; k < vpr; k += 16) { s1 += p1[r * vpr + k]; s2 += p2[r * vpr + k]; }
                s1 = lanes_sum<16>(s1);
                s2 = lanes_sum<16>(s2);
                if (lane16 == 0) { c1s[r] = s1 * inv_D; c2s[r] = s2 * inv_D; }
            }
        }
        ln_sync<TPT>();
#pragma unroll
        for (int u = 0; u < kLnU; ++u) ln_opaque(cq[u], cd[u]);   // rebuild the unpacked values instead of holding them
#pragma unroll
        for (int u = 0; u < kLnU; ++u) {
            if (act[u] && rr[u] < nrows) {
                const int64_t e = (row0 + rr[u]) * D + col[u];
                const float c1 = c1s[rr[u]], c2 = c2s[rr[u]];
                float y[8], d[8], o[8];
                codes_to_float(cq[u], y);
                Store<T>::unpack(cd[u], d);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float xn = (fmaf(y[j], prm[u].x, prm[u].y) - mu[u]) * rs[u];
                    const float gg = d[j] * gam[u][j];
                    o[j] = rs[u] * (gg - c1 - xn * c2);
                }
                Nt<T>::store(dx, e, Store<T>::pack(o));
            }
        }
        ln_sync<TPT>();
    }

    // column sums of this workgroup: slot (team, r) holds what its threads gathered
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kLnU; ++u) {
        if (act[u]) {
            const uint32_t o = (team * R + rr[u]) * D + col[u];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                colG[o + j] = accG[u][j];
                colB[o + j] = accB[u][j];
            }
        }
    }
    __syncthreads();
    float *pg = part + int64_t(blockIdx.x) * 2 * D;
    for (uint32_t c = threadIdx.x; c < D; c += kThreads) {
        float sg = 0.0f, sb = 0.0f;
        for (uint32_t r = 0; r < kTeams * R; ++r) { sg += colG[r * D + c]; sb += colB[r * D + c]; }
        pg[c] = sg;
        pg[D + c] = sb;
    }
}

// dgamma / dbeta = sum over workgroups of their partial column sums.  32 columns per workgroup,
// 32 interleaved slices of the workgroup list (four loads in flight each), combined in a fixed order.
__global__ __launch_bounds__(kLnFinThreads) void k_layernorm_finalize(const float *__restrict__ part, int nwg, uint32_t D,
                                                                      float *__restrict__ dgamma, float *__restrict__ dbeta)
{
    __shared__ float sg[32][33], sb[32][33];
    const uint32_t cl = threadIdx.x & 31u, k = threadIdx.x >> 5;
    const uint32_t c = blockIdx.x * 32 + cl;
    float ag[4] = {0.0f, 0.0f, 0.0f, 0.0f}, ab[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (c < D) {
        int w = int(k);
        for (; w + 96 < nwg; w += 128) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                ag[i] += part[int64_t(w + 32 * i) * 2 * D + c];
                ab[i] += part[int64_t(w + 32 * i) * 2 * D + D + c];
            }
        }
        for (int i = 0; w < nwg; w += 32, ++i) {
            ag[i] += part[int64_t(w) * 2 * D + c];
            ab[i] += part[int64_t(w) * 2 * D + D + c];
        }
    }
    sg[k][cl] = (ag[0] + ag[1]) + (ag[2] + ag[3]);
    sb[k][cl] = (ab[0] + ab[1]) + (ab[2] + ab[3]);
    __syncthreads();
    if (k == 0 && c < D) {
        float tg = 0.0f, tb = 0.0f;
#pragma unroll
        for (int i = 0; i < 32; ++i) { tg += sg[i][cl]; tb += sb[i][cl]; }
        dgamma[c] = tg;
        dbeta[c] = tb;
    }
}

struct LnPlan {
    bool in_wave;          // rows of at most 128 vectors: the wave-row kernel
    int lpr, vpl;          // its lanes per row and vectors per lane
    int64_t R, tiles;      // long rows: rows per workgroup tile, number of tiles
    int grid;
};

static LnPlan ln_plan(int64_t M, int64_t D, mesa_dtype dt)
{
    LnPlan p{};
    const int64_t vpr = D / kVec;
    p.in_wave = vpr <= 128;
    if (p.in_wave) {
        p.lpr = vpr <= 8 ? 8 : vpr <= 16 ? 16 : vpr <= 32 ? 32 : 64;
        p.vpl = vpr <= 64 ? 1 : 2;
        const int64_t block_rows = (kThreads / 64) * kLnRowsInFlight * (64 / p.lpr);   // rows a workgroup has in flight
        const int64_t wgs = ceil_div(M, block_rows);
        // one round of workgroups: every workgroup writes 2 D partial sums, and two / four / eight rounds' worth measured
        // 0.49 / 0.41 / 0.32 against 0.54 of the HBM peak (768-wide rows)
        const int64_t resident = 256 * ln_rows_wg_per_cu(size_t(dtype_bytes(dt)), p.vpl);
        p.grid = int(wgs < resident ? wgs : resident);
        return p;
    }
    const int64_t cap = kThreads * int64_t(kLnU);   // vectors per tile
    p.R = cap / vpr;
    if (p.R > M) p.R = M;
    if (p.R < 1) p.R = 1;
    p.tiles = ceil_div(M, p.R);
    p.grid = int(p.tiles < kLnGridCap ? p.tiles : kLnGridCap);
    return p;
}

// ---- rows the vector kernels cannot take (D or D/G no multiple of 8, D above kLnMaxD): element by element ---------------
// dx: one workgroup per row, the row read twice (the two row sums, then the result); any D.  dx may alias dy: a thread
// writes only elements it has just read, after both sums are complete.
template <typename T>
__global__ __launch_bounds__(kThreads) void k_layernorm_bwd_plain_dx(const int8_t *__restrict__ xq, const void *dy, void *dx,
                                                                     const void *__restrict__ gamma, const float *__restrict__ mean,
                                                                     const float *__restrict__ rstd, const float *__restrict__ alpha,
                                                                     const float *__restrict__ beta, int64_t M, uint32_t D, uint32_t dpg,
                                                                     float inv_D)
{
    __shared__ float p1[kThreads / 64], p2[kThreads / 64];
    for (int64_t row = blockIdx.x; row < M; row += gridDim.x) {
        const float mu = mean[row], rs = rstd[row];
        const int64_t e0 = row * int64_t(D);
        float s1 = 0.0f, s2 = 0.0f;
        for (uint32_t j = threadIdx.x; j < D; j += kThreads) {
            const uint32_t g = j / dpg;
            const float xn = (fmaf(code_to_float(xq[e0 + j]), alpha[g] / 255.0f, beta[g]) - mu) * rs;
            const float gg = Store<T>::load1(dy, e0 + j) * Store<T>::load1(gamma, j);
            s1 += gg;
            s2 = fmaf(gg, xn, s2);
        }
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) { s1 += __shfl_xor(s1, m); s2 += __shfl_xor(s2, m); }
        if ((threadIdx.x & 63) == 0) { p1[threadIdx.x >> 6] = s1; p2[threadIdx.x >> 6] = s2; }
        __syncthreads();
        const float c1 = ((p1[0] + p1[1]) + (p1[2] + p1[3])) * inv_D, c2 = ((p2[0] + p2[1]) + (p2[2] + p2[3])) * inv_D;
        for (uint32_t j = threadIdx.x; j < D; j += kThreads) {
            const uint32_t g = j / dpg;
            const float xn = (fmaf(code_to_float(xq[e0 + j]), alpha[g] / 255.0f, beta[g]) - mu) * rs;
            const float gg = Store<T>::load1(dy, e0 + j) * Store<T>::load1(gamma, j);
            Store<T>::store1(dx, e0 + j, rs * (gg - c1 - xn * c2));
        }
        __syncthreads();                                   // the next row's sums reuse p1, p2
    }
}

// dgamma, dbeta: a workgroup takes 64 columns; its four waves walk the rows r = wave, wave + 4, .. in order, a lane per
// column (consecutive lanes read consecutive elements), and the four partial sums are added in a fixed order.  Runs
// BEFORE the dx kernel, so that dx may alias dy.
template <typename T>
__global__ __launch_bounds__(kThreads) void k_layernorm_bwd_plain_cols(const int8_t *__restrict__ xq, const void *__restrict__ dy,
                                                                       const float *__restrict__ mean, const float *__restrict__ rstd,
                                                                       const float *__restrict__ alpha, const float *__restrict__ beta,
                                                                       int64_t M, uint32_t D, uint32_t dpg, float *__restrict__ dgamma,
                                                                       float *__restrict__ dbeta)
{
    __shared__ float sg[kThreads / 64][64], sb[kThreads / 64][64];
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t c = blockIdx.x * 64 + lane;
    float ag = 0.0f, ab = 0.0f;
    if (c < D) {
        const uint32_t g = c / dpg;
        const float st = alpha[g] / 255.0f, b = beta[g];
        for (int64_t r = wave; r < M; r += kThreads / 64) {
            const float d = Store<T>::load1(dy, r * int64_t(D) + c);
            const float xn = (fmaf(code_to_float(xq[r * int64_t(D) + c]), st, b) - mean[r]) * rstd[r];
            ag = fmaf(d, xn, ag);
            ab += d;
        }
    }
    sg[wave][lane] = ag;
    sb[wave][lane] = ab;
    __syncthreads();
    if (wave == 0 && c < D) {
        dgamma[c] = (sg[0][lane] + sg[1][lane]) + (sg[2][lane] + sg[3][lane]);
        dbeta[c] = (sb[0][lane] + sb[1][lane]) + (sb[2][lane] + sb[3][lane]);
    }
}

static bool ln_vector_path(int64_t D, int64_t G) { return D % kVec == 0 && (D / G) % kVec == 0 && D <= kLnMaxD; }

size_t layernorm_ws_bytes(int64_t M, int64_t D)
{
    if (M <= 0 || D <= 0 || D > kLnMaxD || D % kVec != 0) return 16;
    const int g16 = ln_plan(M, D, MESA_F16).grid, g32 = ln_plan(M, D, MESA_F32).grid;   // enough for either type
    return size_t(g16 > g32 ? g16 : g32) * 2 * size_t(D) * sizeof(float);
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
    if (D >= (int64_t(1) << 31)) return MESA_ERR_UNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!ln_vector_path(D, G)) {                           // element by element, no workspace
        const unsigned grid_rows = unsigned(M < (int64_t(1) << 20) ? M : (int64_t(1) << 20));
#define MESA_LAUNCH_LN_PLAIN(T) \
    do { \
        hipLaunchKernelGGL((k_layernorm_bwd_plain_cols<T>), dim3(unsigned(ceil_div(D, 64))), dim3(kThreads), 0, s, xq, dy, mean, rstd, \
                           alpha, beta, M, uint32_t(D), uint32_t(D / G), dgamma, dbeta); \
        hipLaunchKernelGGL((k_layernorm_bwd_plain_dx<T>), dim3(grid_rows), dim3(kThreads), 0, s, xq, dy, dx, gamma, mean, rstd, alpha, \
                           beta, M, uint32_t(D), uint32_t(D / G), 1.0f / float(D)); \
    } while (0)
        MESA_FOR_DTYPE(dt, MESA_LAUNCH_LN_PLAIN);
#undef MESA_LAUNCH_LN_PLAIN
        return launch_status();
    }
    if (!ws || !aligned16(ws) || ws_bytes < layernorm_ws_bytes(M, D)) return MESA_ERR_WORKSPACE;
    const LnPlan p = ln_plan(M, D, dt);
    FastDiv dvpr = make_fastdiv(uint32_t(D / kVec)), dvpg = make_fastdiv(uint32_t(D / G / kVec));
    float *part = static_cast<float *>(ws);
    const float inv_D = 1.0f / float(D);
#define MESA_LAUNCH_ROWS(T, LPR_, VPL_) \
    hipLaunchKernelGGL((k_layernorm_bwd_rows<T, LPR_, VPL_>), dim3(p.grid), dim3(kThreads), 0, s, xq, dy, dx, gamma, mean, rstd, \
                       alpha, beta, M, uint32_t(D), dvpg, inv_D, part)
#define MESA_LAUNCH_ROWS_T(T) \
    do { \
        if (p.vpl == 2) MESA_LAUNCH_ROWS(T, 64, 2); \
        else if (p.lpr == 64) MESA_LAUNCH_ROWS(T, 64, 1); \
        else if (p.lpr == 32) MESA_LAUNCH_ROWS(T, 32, 1); \
        else if (p.lpr == 16) MESA_LAUNCH_ROWS(T, 16, 1); \
        else MESA_LAUNCH_ROWS(T, 8, 1); \
    } while (0)
#define MESA_LAUNCH_LN(T) \
    hipLaunchKernelGGL((k_layernorm_bwd<T, kThreads>), dim3(p.grid), dim3(kThreads), 0, s, xq, dy, dx, gamma, mean, rstd, alpha, \
                       beta, M, uint32_t(D), uint32_t(p.R), p.tiles, uint32_t(G), dvpr, dvpg, inv_D, part)
    if (p.in_wave) {
        MESA_FOR_DTYPE(dt, MESA_LAUNCH_ROWS_T);
    } else {
        MESA_FOR_DTYPE(dt, MESA_LAUNCH_LN);
    }
#undef MESA_LAUNCH_LN
#undef MESA_LAUNCH_ROWS_T
#undef MESA_LAUNCH_ROWS
    if (launch_status() != MESA_OK) return MESA_ERR_LAUNCH;   // the consumer must not run on a workspace nobody wrote
    hipLaunchKernelGGL(k_layernorm_finalize, dim3(unsigned(ceil_div(D, 32))), dim3(kLnFinThreads), 0, s, part, p.grid,
                       uint32_t(D), dgamma, dbeta);
    return launch_status();
}
