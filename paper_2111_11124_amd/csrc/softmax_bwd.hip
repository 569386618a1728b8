// softmax_bwd.hip -- softmax backward at the de-quantized attention map (Sec. 3.1 Eq. 2):
//   per row  d = sum_j dy_j*y_hat_j,  dx_j = y_hat_j*(dy_j - d),  y_hat = (q+128)*alpha_h/255 + beta_h.
//
// Rows of 197 or 49 elements start at odd byte offsets, so a workgroup takes a tile of R
// consecutive rows with R*cols a multiple of 8: the tile is then a run of whole 8-element vectors
// that start 16-byte aligned in dy / dx and 8-byte aligned in the codes, and is read and written
// flat with full-width accesses.  Codes and dy stay in registers between the two passes; only two
// partial sums per vector (a vector touches at most two rows when cols >= 8) go through LDS,
// where 16 lanes per row add them in a fixed order.  One HBM read of codes and dy, one write of dx.
#include <hip/hip_runtime.h>

#include "api_util.hpp"
#include "common.hpp"

namespace mesa {

constexpr int kSmU = 4;             // vectors per thread in a tile
constexpr int kSmMaxHeads = 1024;

// Synchronisation among the TPT threads that share a tile: a workgroup barrier, or -- when a tile
// belongs to one wave -- only an ordering of that wave's own LDS traffic (its lanes run in lockstep).
template <int TPT> __device__ __forceinline__ void tile_sync()
{
    if (TPT == kThreads) {
        __syncthreads();
    } else {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
}

__device__ __forceinline__ void opaque(u32x2 &a, u32x4 &b)
{
    asm volatile("" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ void opaque(u32x2 &a, Store<float>::raw_t &b)
{
    asm volatile("" : "+v"(a), "+v"(b.lo), "+v"(b.hi));
}

// TPT threads (one wave, or the whole workgroup for long rows) own a tile of up to TPT*4 vectors.
template <typename T, int TPT>
__global__ __launch_bounds__(kThreads, 4) void k_softmax_bwd(const int8_t *__restrict__ yq, const void *dy, void *dx,
                                                          int64_t total_rows, uint32_t cols, uint32_t R, int64_t tiles,
                                                          FastDiv div_cols, FastDiv div_rows, FastDiv div_heads,
                                                          const float *__restrict__ alpha, const float *__restrict__ beta)
{
    constexpr int kTileVec = TPT * kSmU;          // vectors per tile
    constexpr int kTeams = kThreads / TPT;        // tiles in flight per workgroup
    __shared__ float2 head_tab[kSmMaxHeads];   // (step, beta) per head
    __shared__ float PA[kTeams][kTileVec], PB[kTeams][kTileVec], rowD[kTeams][kTileVec];

    const uint32_t heads = div_heads.d;
    for (uint32_t h = threadIdx.x; h < heads; h += kThreads) head_tab[h] = make_float2(alpha[h] / 255.0f, beta[h]);
    __syncthreads();

    const uint32_t team = threadIdx.x / TPT;
    const uint32_t tid = threadIdx.x % TPT;
    float *pa = PA[team], *pb = PB[team], *rd = rowD[team];

    for (int64_t tile = int64_t(blockIdx.x) * kTeams + team; tile < tiles; tile += int64_t(gridDim.x) * kTeams) {
        const int64_t row0 = tile * R;
        const uint32_t nrows = uint32_t((total_rows - row0 < int64_t(R)) ? (total_rows - row0) : int64_t(R));
        const uint32_t nelem = nrows * cols;
        const uint32_t nvec = (nelem + kVec - 1) / kVec;
        const int64_t e0 = row0 * cols;

        u32x2 cq[kSmU];
        typename Store<T>::raw_t cd[kSmU];
        uint32_t r1[kSmU], nb[kSmU];
        float2 prmA[kSmU], prmB[kSmU];
#pragma unroll
        for (int u = 0; u < kSmU; ++u) {
            const uint32_t v = u * TPT + tid;
            if (v < nvec) {
                const uint32_t le = v * kVec;
                const int64_t e = e0 + le;
                if (le + kVec <= nelem) {
                    cq[u] = nt_load<u32x2>(yq + e);
                    cd[u] = Nt<T>::load(dy, e);
                } else {  // ragged end of the whole tensor
                    float g[8];
                    uint32_t w[2] = {0u, 0u};
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const bool in = le + j < nelem;
                        w[j >> 2] |= uint32_t(in ? uint8_t(yq[e + j]) : uint8_t(0x80)) << (8 * (j & 3));
                        g[j] = in ? Store<T>::load1(dy, e + j) : 0.0f;
                    }
                    cq[u][0] = w[0];
                    cq[u][1] = w[1];
                    cd[u] = Store<T>::pack(g);   // exact: g came from T
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kSmU; ++u) {
            const uint32_t v = u * TPT + tid;
            if (v < nvec) {
                const uint32_t le = v * kVec;
                r1[u] = fastdiv(le, div_cols);
                nb[u] = (r1[u] + 1) * cols - le;   // elements of this vector that lie in row r1
                // head of row r1 and of the row after it
                const uint32_t grow = uint32_t(row0) + r1[u];
                const uint32_t slab = fastdiv(grow, div_rows);
                const uint32_t h = slab - fastdiv(slab, div_heads) * heads;
                const uint32_t h2 = (grow + 1 - slab * div_rows.d == div_rows.d) ? ((h + 1 == heads) ? 0u : h + 1) : h;
                prmA[u] = head_tab[h];
                prmB[u] = head_tab[h2];
                float g[8], y[8];
                Store<T>::unpack(cd[u], g);
                codes_to_float(cq[u], y);
                float sA = 0.0f, sB = 0.0f;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const bool first = uint32_t(j) < nb[u];
                    const float yh = fmaf(y[j], first ? prmA[u].x : prmB[u].x, first ? prmA[u].y : prmB[u].y);
                    const float p = g[j] * yh;
                    sA += first ? p : 0.0f;
                    sB += first ? 0.0f : p;
                }
                pa[v] = sA;
                pb[v] = sB;
            }
        }
        tile_sync<TPT>();

        // 16 lanes per row: the row's own part of its first vector, then the vectors that start in it
        {
            const uint32_t lane16 = tid & 15u;
            for (uint32_t r = tid >> 4; r < nrows; r += TPT / 16) {
                const uint32_t start = r * cols;
                const uint32_t vs = start >> 3;
                const uint32_t ve = (start + cols - 1) >> 3;
                float s = 0.0f;
                if (lane16 == 0) s = (start & 7u) ? pb[vs] : pa[vs];
                for (uint32_t v = vs + 1 + lane16; v <= ve; v += 16) s += pa[v];
                s = lanes_sum<16>(s);
                if (lane16 == 0) rd[r] = s;
            }
        }
        tile_sync<TPT>();

        // keep only the packed inputs across the passes: the unpacked values are cheap to rebuild,
        // and holding them would halve the number of waves a SIMD can keep in flight
#pragma unroll
        for (int u = 0; u < kSmU; ++u) opaque(cq[u], cd[u]);
#pragma unroll
        for (int u = 0; u < kSmU; ++u) {
            const uint32_t v = u * TPT + tid;
            if (v < nvec) {
                const uint32_t le = v * kVec;
                const int64_t e = e0 + le;
                const uint32_t r2 = (r1[u] + 1 < nrows) ? r1[u] + 1 : r1[u];
                const float dA = rd[r1[u]], dB = rd[r2];
                float g[8], y[8], o[8];
                Store<T>::unpack(cd[u], g);
                codes_to_float(cq[u], y);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const bool first = uint32_t(j) < nb[u];
                    const float yh = fmaf(y[j], first ? prmA[u].x : prmB[u].x, first ? prmA[u].y : prmB[u].y);
                    o[j] = yh * (g[j] - (first ? dA : dB));
                }
                if (le + kVec <= nelem) {
                    Nt<T>::store(dx, e, Store<T>::pack(o));
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (le + j < nelem) Store<T>::store1(dx, e + j, o[j]);
                }
            }
        }
        tile_sync<TPT>();  // the next tile rewrites the partial sums
    }
}

}  // namespace mesa

using namespace mesa;

extern "C" MESA_EXPORT mesa_status mesa_softmax_bwd_q(const int8_t *yq, int64_t B, int64_t H, int64_t rows, int64_t cols,
                                                      const float *alpha, const float *beta, const void *dy, void *dx,
                                                      mesa_dtype dt, void *stream)
{
    if (!valid_dtype(dt) || B < 0 || H < 0 || rows < 0 || cols < 0) return MESA_ERR_INVALID_ARG;
    if (B == 0 || H == 0 || rows == 0 || cols == 0) return MESA_OK;
    if (!yq || !dy || !dx || !alpha || !beta || !aligned16(yq) || !aligned16(dy) || !aligned16(dx) || !aligned4(alpha) ||
        !aligned4(beta))
        return MESA_ERR_INVALID_ARG;
    if (H > kSmMaxHeads || rows >= (int64_t(1) << 31) || cols < kVec) return MESA_ERR_UNSUPPORTED;
    const long double tr = (long double)B * (long double)H * (long double)rows;
    if (tr >= 2147483648.0L) return MESA_ERR_UNSUPPORTED;
    const int64_t total_rows = B * H * rows;
    // rows per tile: a multiple of 8/gcd(cols, 8) so that every tile starts on a vector boundary.
    // Short rows: one wave per tile (2048 elements); long rows: the whole workgroup (8192 elements).
    int64_t gc = cols, b8 = 8;
    while (b8) { int64_t t = gc % b8; gc = b8; b8 = t; }
    const int64_t unit = 8 / gc;
    const bool wave_tiles = unit * cols <= int64_t(64) * kSmU * kVec;
    const int64_t cap = (wave_tiles ? 64 : kThreads) * int64_t(kSmU) * kVec;
    int64_t R = (cap / cols) / unit * unit;
    if (R < unit) return MESA_ERR_UNSUPPORTED;   // `unit` rows of this length do not fit one tile
    if (R > total_rows) R = ceil_div(total_rows, unit) * unit;
    const int64_t tiles = ceil_div(total_rows, R);
    const int64_t teams = wave_tiles ? kThreads / 64 : 1;
    const int64_t wgs = ceil_div(tiles, teams);
    const int grid = int(wgs < 2048 ? wgs : 2048);
    FastDiv dc = make_fastdiv(uint32_t(cols)), dr = make_fastdiv(uint32_t(rows)), dh = make_fastdiv(uint32_t(H));
    hipStream_t s = static_cast<hipStream_t>(stream);
#define MESA_LAUNCH_S(T, TPT_) \
    hipLaunchKernelGGL((k_softmax_bwd<T, TPT_>), dim3(grid), dim3(kThreads), 0, s, yq, dy, dx, total_rows, uint32_t(cols), \
                       uint32_t(R), tiles, dc, dr, dh, alpha, beta)
    if (dt == MESA_F16) { if (wave_tiles) MESA_LAUNCH_S(_Float16, 64); else MESA_LAUNCH_S(_Float16, kThreads); }
    else { if (wave_tiles) MESA_LAUNCH_S(float, 64); else MESA_LAUNCH_S(float, kThreads); }
#undef MESA_LAUNCH_S
    return launch_status();
}
