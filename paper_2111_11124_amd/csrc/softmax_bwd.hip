// softmax_bwd.hip -- softmax backward at the de-quantized attention map (Sec. 3.1 Eq. 2):
//   per row  d = sum_j dy_j*y_hat_j,  dx_j = y_hat_j*(dy_j - d),  y_hat = (q+128)*alpha_h/255 + beta_h.
//
// Rows of 197 or 49 elements start at odd byte offsets, so a wave (or, for long rows, a workgroup) takes a
// tile of R consecutive rows with R*cols a multiple of 8: the tile is then a run of whole 8-element vectors
// that start 16-byte aligned in dy / dx and 8-byte aligned in the codes, and is read and written flat with
// full-width accesses.  One HBM read of codes and dy, one write of dx.  Two kernels:
//   rows of up to 256 elements: k_softmax_bwd_rows, at the end of this file -- the tile staged through LDS, a
//   row per group of lanes;
//   longer rows: k_softmax_bwd -- codes and dy stay in registers between the two passes; only two partial
//   sums per vector (a vector touches at most two rows when cols >= 8) go through LDS, where 16 lanes per row
//   add them in a fixed order.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "api_util.hpp"
#include "common.hpp"
#include "softmax_rows.hpp"

namespace mesa {

constexpr int kSmU = 4;             // vectors per thread in a tile
constexpr int kSmMaxHeads = 1024;
constexpr int kSmWgPerCu = 3;       // occupancy the kernel's register budget is set for

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

// Four codes (the bytes of w, stored as x_bar - 128) as two binary16 pairs holding x_bar itself:
// 0x6400 | byte is 1024 + byte exactly, and the subtraction of 1024 is exact too.
__device__ __forceinline__ void codes_to_h2(uint32_t w, h2 &lo, h2 &hi)
{
    const h2 k1024 = {(_Float16)1024.0f, (_Float16)1024.0f};
    const uint32_t x = w ^ 0x80808080u;
    lo = as_h2(__builtin_amdgcn_perm(0x64646464u, x, 0x04010400u)) - k1024;   // bytes 0, 1
    hi = as_h2(__builtin_amdgcn_perm(0x64646464u, x, 0x04030402u)) - k1024;   // bytes 2, 3
}

// TPT threads (one wave, or the whole workgroup for long rows) own a tile of up to TPT*4 vectors.
template <typename T, int TPT>
__global__ __launch_bounds__(kThreads, kSmWgPerCu) void k_softmax_bwd(const int8_t *__restrict__ yq, const void *dy, void *dx,
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

    // Every tile has the same shape (R whole rows, a whole number of vectors), so where this thread's
    // vectors lie in their rows is the same in every tile: the row r1 a vector starts in, how many of
    // its elements belong to that row (nb; the rest to the next row), and -- for the binary16 fast
    // path -- bit masks of the halves that belong to the next row.
    constexpr bool kHalf = std::is_same<T, _Float16>::value;
    uint32_t r1[kSmU], nb[kSmU];
    uint32_t maskB[kSmU][4];
#pragma unroll
    for (int u = 0; u < kSmU; ++u) {
        const uint32_t le = (u * TPT + tid) * kVec;
        r1[u] = fastdiv(le, div_cols);
        nb[u] = (r1[u] + 1) * cols - le;
#pragma unroll
        for (int k = 0; k < 4; ++k)
            maskB[u][k] = (uint32_t(2 * k) >= nb[u] ? 0x0000FFFFu : 0u) | (uint32_t(2 * k + 1) >= nb[u] ? 0xFFFF0000u : 0u);
    }

    for (int64_t tile = int64_t(blockIdx.x) * kTeams + team; tile < tiles; tile += int64_t(gridDim.x) * kTeams) {
        const int64_t row0 = tile * R;
        const uint32_t nrows = uint32_t((total_rows - row0 < int64_t(R)) ? (total_rows - row0) : int64_t(R));
        const uint32_t nelem = nrows * cols;
        const uint32_t nvec = (nelem + kVec - 1) / kVec;
        const int64_t e0 = row0 * cols;

        u32x2 cq[kSmU];
        typename Store<T>::raw_t cd[kSmU];
        // (step, beta) of the head of row r1 and of the row after it; looked up again in the second pass
        // rather than held in registers across the reduction
        auto head_params = [&](int u, float2 &prmA, float2 &prmB) {
            const uint32_t grow = uint32_t(row0) + r1[u];
            const uint32_t slab = fastdiv(grow, div_rows);
            const uint32_t h = slab - fastdiv(slab, div_heads) * heads;
            const uint32_t h2 = (grow + 1 - slab * div_rows.d == div_rows.d) ? ((h + 1 == heads) ? 0u : h + 1) : h;
            prmA = head_tab[h];
            prmB = head_tab[h2];
        };
        // One head for the whole tile (all but the few tiles that straddle two attention maps): its
        // step and offset are uniform, and in binary16 the sums  sum dy*y_hat = step * sum dy*x_bar +
        // beta * sum dy  can be taken two elements at a time by dot instructions straight from the
        // packed dy and the codes (x_bar <= 255 is exact in binary16, the products and sums are binary32).
        const uint32_t slab_first = fastdiv(uint32_t(row0), div_rows);
        const uint32_t slab_last = fastdiv(uint32_t(row0) + nrows - 1, div_rows);
        const bool one_head = kHalf && slab_first == slab_last;
        const float2 prmT = head_tab[slab_first - fastdiv(slab_first, div_heads) * heads];
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
        if constexpr (kHalf) {
            if (one_head) {
                const h2 ones = {(_Float16)1.0f, (_Float16)1.0f};
#pragma unroll
                for (int u = 0; u < kSmU; ++u) {
                    const uint32_t v = u * TPT + tid;
                    if (v < nvec) {
                        float t1 = 0.0f, t2 = 0.0f, b1 = 0.0f, b2 = 0.0f;
#pragma unroll
                        for (int w = 0; w < 2; ++w) {
                            h2 ylo, yhi;
                            codes_to_h2(cq[u][w], ylo, yhi);
                            const uint32_t g0 = cd[u][2 * w], g1 = cd[u][2 * w + 1];
                            t1 = __builtin_amdgcn_fdot2(as_h2(g0), ylo, t1, false);
                            t1 = __builtin_amdgcn_fdot2(as_h2(g1), yhi, t1, false);
                            t2 = __builtin_amdgcn_fdot2(as_h2(g0), ones, t2, false);
                            t2 = __builtin_amdgcn_fdot2(as_h2(g1), ones, t2, false);
                            const h2 h0 = as_h2(g0 & maskB[u][2 * w]), h1 = as_h2(g1 & maskB[u][2 * w + 1]);
                            b1 = __builtin_amdgcn_fdot2(h0, ylo, b1, false);
                            b1 = __builtin_amdgcn_fdot2(h1, yhi, b1, false);
                            b2 = __builtin_amdgcn_fdot2(h0, ones, b2, false);
                            b2 = __builtin_amdgcn_fdot2(h1, ones, b2, false);
                        }
                        const float sT = fmaf(prmT.x, t1, prmT.y * t2), sB = fmaf(prmT.x, b1, prmT.y * b2);
                        pa[v] = sT - sB;
                        pb[v] = sB;
                    }
                }
            }
        }
        if (!one_head) {
#pragma unroll
        for (int u = 0; u < kSmU; ++u) {
            const uint32_t v = u * TPT + tid;
            if (v < nvec) {
                float2 prmA, prmB;
                head_params(u, prmA, prmB);
                float g[8], y[8];
                Store<T>::unpack(cd[u], g);
                codes_to_float(cq[u], y);
                float sA = 0.0f, sB = 0.0f;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const bool first = uint32_t(j) < nb[u];
                    const float yh = fmaf(y[j], first ? prmA.x : prmB.x, first ? prmA.y : prmB.y);
                    const float p = g[j] * yh;
                    sA += first ? p : 0.0f;
                    sB += first ? 0.0f : p;
                }
                pa[v] = sA;
                pb[v] = sB;
            }
        }
        }
        tile_sync<TPT>();

        // A group of lanes per row (8 when a row spans at most 8 vectors, else 16): the row's own part of
        // its first vector, then the vectors that start in it
        auto row_sums = [&](auto lanes) {
            constexpr uint32_t LPR = decltype(lanes)::value;
            const uint32_t ln = tid & (LPR - 1);
            for (uint32_t r = tid / LPR; r < nrows; r += TPT / LPR) {
                const uint32_t start = r * cols;
                const uint32_t vs = start >> 3;
                const uint32_t ve = (start + cols - 1) >> 3;
                float s = 0.0f;
                if (ln == 0) s = (start & 7u) ? pb[vs] : pa[vs];
                for (uint32_t v = vs + 1 + ln; v <= ve; v += LPR) s += pa[v];
                s = lanes_sum_dpp<LPR>(s);
                if (ln == 0) rd[r] = s;
            }
        };
        if (cols <= 56) row_sums(std::integral_constant<uint32_t, 8>());   // at most 8 vectors touch such a row
        else row_sums(std::integral_constant<uint32_t, 16>());
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
                float o[8];
                bool done = false;
                if constexpr (kHalf) {
                    if (one_head) {
                        // dy and x_bar enter the fused multiply-adds as binary16 operands
#pragma unroll
                        for (int w = 0; w < 2; ++w) {
                            h2 yq2[2];
                            codes_to_h2(cq[u][w], yq2[0], yq2[1]);
#pragma unroll
                            for (int c = 0; c < 2; ++c) {
                                const h2 g2 = as_h2(cd[u][2 * w + c]);
#pragma unroll
                                for (int i = 0; i < 2; ++i) {
                                    const int j = 4 * w + 2 * c + i;
                                    const float dsel = (uint32_t(j) < nb[u]) ? dA : dB;
                                    const float yh = fmaf(float(yq2[c][i]), prmT.x, prmT.y);
                                    o[j] = yh * fmaf(float(g2[i]), 1.0f, -dsel);
                                }
                            }
                        }
                        done = true;
                    }
                }
                if (!done) {
                    float2 prmA, prmB;
                    head_params(u, prmA, prmB);
                    float g[8], y[8];
                    Store<T>::unpack(cd[u], g);
                    codes_to_float(cq[u], y);
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const bool first = uint32_t(j) < nb[u];
                        const float yh = fmaf(y[j], first ? prmA.x : prmB.x, first ? prmA.y : prmB.y);
                        o[j] = yh * (g[j] - (first ? dA : dB));
                    }
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

// ---------------------------------------------------------------------------------------------
// Rows of at most 256 elements (the attention maps of the paper's models): a row per group of LPR lanes.
// A wave's tile of codes and dy goes through its LDS region flat, fetched one tile ahead; in the row phase a lane
// holds its EPL slots of dy and y_hat in registers, the row's d = sum dy*y_hat is a reduction inside the group,
// and dx is written back over dy in LDS, from where it leaves as aligned vectors.  dx may be dy (in place): a
// tile's dy is in LDS before any of its dx is stored, and tiles do not overlap.
// ---------------------------------------------------------------------------------------------
constexpr int kSbRowWaves = 4;      // waves per SIMD the row kernel's register budget is set for

template <typename T, int LPR, int EPL, bool TIGHT>
__global__ __launch_bounds__(kThreads, kSbRowWaves) void k_softmax_bwd_rows(const int8_t *__restrict__ yq, const void *dy, void *dx,
                                                                           int64_t total_rows, uint32_t cols, uint32_t R,
                                                                           int64_t tiles, FastDiv div_rows, FastDiv div_heads,
                                                                           const float *__restrict__ alpha,
                                                                           const float *__restrict__ beta, uint32_t tab_bytes,
                                                                           uint32_t wave_bytes)
{
    constexpr int kB = Store<T>::kBytes;
    constexpr int RPP = 64 / LPR;                        // rows per pass
    constexpr int kWaves = kThreads / 64;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const uint32_t heads = div_heads.d;
    float2 *head_tab = reinterpret_cast<float2 *>(smem);              // y_hat = s * q + off with q the signed code
    for (uint32_t h = threadIdx.x; h < heads; h += kThreads) {
        const float s = alpha[h] / 255.0f;
        head_tab[h] = make_float2(s, fmaf(128.0f, s, beta[h]));
    }
    __syncthreads();

    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint32_t sub = lane / LPR, l = lane % LPR;
    const uint32_t tile_cap = R * cols;                  // elements of a whole tile, a multiple of 8
    unsigned char *gs = smem + tab_bytes + wave * wave_bytes;         // dy, then dx
    unsigned char *cs = gs + tile_cap * kB;                           // codes

    typename Store<T>::raw_t raw[kSrFlat];
    u32x2 rawq[kSrFlat];
    auto fetch = [&](int64_t t) {
        const int64_t row0 = t * R;
        const uint32_t nrows = uint32_t((total_rows - row0 < int64_t(R)) ? (total_rows - row0) : int64_t(R));
        const uint32_t nfull = nrows * cols / kVec;
#pragma unroll
        for (int u = 0; u < kSrFlat; ++u) {
            const uint32_t v = u * 64 + lane;
            if (v < nfull) {
                raw[u] = Nt<T>::load(dy, row0 * cols + v * kVec);
                rawq[u] = nt_load<u32x2>(yq + row0 * cols + v * kVec);
            }
        }
    };
    const int64_t tile_step = int64_t(gridDim.x) * kWaves;
    int64_t tile = int64_t(blockIdx.x) * kWaves + wave;
    if (tile < tiles) fetch(tile);
    for (; tile < tiles; tile += tile_step) {
        const int64_t row0 = tile * R;
        const uint32_t nrows = uint32_t((total_rows - row0 < int64_t(R)) ? (total_rows - row0) : int64_t(R));
        const uint32_t nelem = nrows * cols;
        const int64_t e0 = row0 * cols;                  // a multiple of 8
        const uint32_t nfull = nelem / kVec, tail = nelem % kVec;    // a tail: only at the end of the whole tensor
        if (lane < tail) {
            const uint32_t le = nfull * kVec + lane;
            LdsElem<T>::put(gs + le * kB, Store<T>::load1(dy, e0 + le));
            cs[le] = uint8_t(yq[e0 + le]);
        }
#pragma unroll
        for (int u = 0; u < kSrFlat; ++u) {
            const uint32_t v = u * 64 + lane;
            if (v < nfull) {
                Store<T>::store(gs, int64_t(v) * kVec, raw[u]);
                *reinterpret_cast<u32x2 *>(cs + v * kVec) = rawq[u];
            }
        }
        team_sync<64>();
        if (tile + tile_step < tiles) fetch(tile + tile_step);

        for (uint32_t p0 = 0; p0 < nrows; p0 += RPP) {
            const uint32_t r = p0 + sub;
            const bool live = r < nrows;
            const uint32_t rr = live ? r : p0;                        // groups without a row repeat the pass's first
            const uint32_t eb = rr * cols + l;
            unsigned char *gp = gs + eb * kB;
            const unsigned char *cp = cs + eb;
            const uint32_t grow = uint32_t(row0) + rr;
            const uint32_t slab = fastdiv(grow, div_rows);
            const float2 prm = head_tab[slab - fastdiv(slab, div_heads) * heads];
            float g[EPL], yh[EPL];
            float d = 0.0f;
#pragma unroll
            for (int k = 0; k < EPL; ++k) {
                const bool valid = (TIGHT && k < EPL - 1) || l + k * LPR < cols;
                const float gv = LdsElem<T>::get(gp + k * LPR * kB);
                const float qv = float(int(*reinterpret_cast<const int8_t *>(cp + k * LPR)));
                g[k] = valid ? gv : 0.0f;                             // unused slots add nothing
                yh[k] = fmaf(qv, prm.x, prm.y);
                d = fmaf(g[k], yh[k], d);
            }
            d = lanes_sum_dpp<LPR>(d);
            if (live) {
#pragma unroll
                for (int k = 0; k < EPL; ++k) {
                    const bool valid = (TIGHT && k < EPL - 1) || l + k * LPR < cols;
                    if (valid) LdsElem<T>::put(gp + k * LPR * kB, yh[k] * (g[k] - d));
                }
            }
        }
        team_sync<64>();

#pragma unroll
        for (int u = 0; u < kSrFlat; ++u) {
            const uint32_t v = u * 64 + lane;
            if (v < nfull) Nt<T>::store(dx, e0 + v * kVec, Store<T>::load(gs, int64_t(v) * kVec));
        }
        if (lane < tail) {
            const uint32_t le = nfull * kVec + lane;
            Store<T>::store1(dx, e0 + le, LdsElem<T>::get(gs + le * kB));   // exact: the value is already of type T
        }
        team_sync<64>();   // the next tile rewrites the region
    }
}

// Rows the tiled kernels cannot take (eight rows of an odd length above 1024 do not fit a tile, more than
// kSmMaxHeads heads, rows shorter than a vector next to many heads): one workgroup per row, the row read twice --
// once for d = sum_j dy_j * y_hat_j (per-thread sums in a fixed order, then the wave's lanes, then the four waves),
// once more for dx_j = y_hat_j * (dy_j - d); the second read comes from the caches.  A row starts wherever the one
// before it ended: the elements up to the first 16-byte boundary of dy and those behind the last one go one by one,
// the vectors between them whole.  Any length.  dx may alias dy: a thread writes only the elements it has just read,
// and every sum is complete before the first write.
template <typename T>
__global__ __launch_bounds__(kThreads) void k_softmax_bwd_plain(const int8_t *__restrict__ yq, const void *dy, void *dx, int64_t total_rows,
                                                                uint32_t cols, uint32_t rows, uint32_t heads,
                                                                const float *__restrict__ alpha, const float *__restrict__ beta)
{
    __shared__ float part[kThreads / 64];
    for (int64_t row = blockIdx.x; row < total_rows; row += gridDim.x) {
        const uint32_t h = uint32_t((row / rows) % heads);
        const float s = alpha[h] / 255.0f, b = beta[h];                  // y_hat = s * x_bar + beta, x_bar = code + 128
        const int64_t e0 = row * int64_t(cols);
        const uint32_t lead = uint32_t((8 - (e0 & 7)) & 7);
        const uint32_t head = lead < cols ? lead : cols;                  // elements before the first whole vector
        const uint32_t nvec = (cols - head) / kVec;
        const uint32_t tail0 = head + nvec * kVec;                        // first element behind the last whole vector
        // the edge elements: thread t takes head element t or tail element t - 8
        const uint32_t edge = threadIdx.x < 8 ? threadIdx.x : tail0 + (threadIdx.x - 8);
        const bool has_edge = threadIdx.x < 8 ? threadIdx.x < head : (threadIdx.x < 16 && edge < cols);
        float d = 0.0f;
        if (has_edge) d = Store<T>::load1(dy, e0 + edge) * fmaf(code_to_float(yq[e0 + edge]), s, b);
        for (uint32_t v = threadIdx.x; v < nvec; v += kThreads) {
            const int64_t e = e0 + head + int64_t(v) * kVec;
            float g[8], y[8];
            Store<T>::unpack(Store<T>::load(dy, e), g);
            codes_to_float(*reinterpret_cast<const u32x2 *>(yq + e), y);
#pragma unroll
            for (int k = 0; k < 8; ++k) d = fmaf(g[k], fmaf(y[k], s, b), d);
        }
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) d += __shfl_xor(d, m);
        if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = d;
        __syncthreads();
        d = (part[0] + part[1]) + (part[2] + part[3]);
        if (has_edge) {
            const float yh = fmaf(code_to_float(yq[e0 + edge]), s, b);
            Store<T>::store1(dx, e0 + edge, yh * (Store<T>::load1(dy, e0 + edge) - d));
        }
        for (uint32_t v = threadIdx.x; v < nvec; v += kThreads) {
            const int64_t e = e0 + head + int64_t(v) * kVec;
            float g[8], y[8], o[8];
            Store<T>::unpack(Store<T>::load(dy, e), g);
            codes_to_float(*reinterpret_cast<const u32x2 *>(yq + e), y);
#pragma unroll
            for (int k = 0; k < 8; ++k) o[k] = fmaf(y[k], s, b) * (g[k] - d);
            Store<T>::store(dx, e, Store<T>::pack(o));
        }
        __syncthreads();                                   // the next row's sums reuse `part`
    }
}

struct SbPlan {
    bool ok;
    SrShape sh;
    int grid;
    uint32_t tab_bytes, wave_bytes;
    size_t lds;
};

static SbPlan sb_plan(int64_t total_rows, int64_t H, int64_t cols, int elem_bytes)
{
    SbPlan p{};
    if (cols > kSrMaxCols) return p;
    p.sh = sr_shape(total_rows, cols);
    p.tab_bytes = uint32_t((H * 8 + 15) / 16 * 16);
    p.wave_bytes = uint32_t((p.sh.R * cols * (elem_bytes + 1) + 15) / 16 * 16);
    p.lds = size_t(p.tab_bytes) + size_t(kThreads / 64) * p.wave_bytes + kSrSlack;
    p.ok = p.lds <= 64 * 1024;
    if (!p.ok) return p;
    // one tile per wave: many short workgroups, launched in order, sweep the tensor as one compact window -- measured 0.73
    // against 0.68 of the HBM peak for one resident round of workgroups striding over the tiles (119 M elements)
    const int64_t wgs = ceil_div(p.sh.tiles, kThreads / 64);
    p.grid = int(wgs < (int64_t(1) << 22) ? wgs : (int64_t(1) << 22));
    return p;
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
    if (rows >= (int64_t(1) << 31) || cols >= (int64_t(1) << 31) || H >= (int64_t(1) << 31)) return MESA_ERR_UNSUPPORTED;
    const long double tr = (long double)B * (long double)H * (long double)rows;
    if (tr >= 2147483648.0L) return MESA_ERR_UNSUPPORTED;
    const int64_t total_rows = B * H * rows;
    auto plain = [&]() {
        hipStream_t sp = static_cast<hipStream_t>(stream);
#define MESA_LAUNCH_SP(T) \
    hipLaunchKernelGGL((k_softmax_bwd_plain<T>), dim3(unsigned(total_rows < (int64_t(1) << 20) ? total_rows : (int64_t(1) << 20))), \
                       dim3(kThreads), 0, sp, yq, dy, dx, total_rows, uint32_t(cols), uint32_t(rows), uint32_t(H), alpha, beta)
        MESA_FOR_DTYPE(dt, MESA_LAUNCH_SP);
#undef MESA_LAUNCH_SP
        return launch_status();
    };
    if (H > kSmMaxHeads) return plain();
    const SbPlan rp = sb_plan(total_rows, H, cols, dtype_bytes(dt));
    if (rp.ok) {
        FastDiv drr = make_fastdiv(uint32_t(rows)), dhh = make_fastdiv(uint32_t(H));
        hipStream_t sr = static_cast<hipStream_t>(stream);
#define MESA_LAUNCH_SB(T, LPR_, EPL_, TIGHT_) \
    hipLaunchKernelGGL((k_softmax_bwd_rows<T, LPR_, EPL_, TIGHT_>), dim3(rp.grid), dim3(kThreads), rp.lds, sr, yq, dy, dx, total_rows, \
                       uint32_t(cols), uint32_t(rp.sh.R), rp.sh.tiles, drr, dhh, alpha, beta, rp.tab_bytes, rp.wave_bytes)
#define MESA_LAUNCH_SB_C(T, LPR_, EPL_) \
    do { if (rp.sh.tight) MESA_LAUNCH_SB(T, LPR_, EPL_, true); else MESA_LAUNCH_SB(T, LPR_, EPL_, false); } while (0)
#define MESA_LAUNCH_SB_T(T) \
    do { \
        if (rp.sh.lpr == 16) MESA_LAUNCH_SB_C(T, 16, 16); \
        else if (rp.sh.epl == 25) MESA_LAUNCH_SB_C(T, 8, 25); \
        else if (rp.sh.epl == 13) MESA_LAUNCH_SB_C(T, 8, 13); \
        else if (rp.sh.epl == 16) MESA_LAUNCH_SB_C(T, 8, 16); \
        else if (rp.sh.epl == 8) MESA_LAUNCH_SB_C(T, 8, 8); \
        else MESA_LAUNCH_SB_C(T, 8, 7); \
    } while (0)
        MESA_FOR_DTYPE(dt, MESA_LAUNCH_SB_T);
#undef MESA_LAUNCH_SB_T
#undef MESA_LAUNCH_SB_C
#undef MESA_LAUNCH_SB
        return launch_status();
    }
    if (cols < kVec) return plain();
    // rows per tile: a multiple of 8/gcd(cols, 8) so that every tile starts on a vector boundary.
    // Short rows: one wave per tile (2048 elements); long rows: the whole workgroup (8192 elements).
    int64_t gc = cols, b8 = 8;
    while (b8) { int64_t t = gc % b8; gc = b8; b8 = t; }
    const int64_t unit = 8 / gc;
    const bool wave_tiles = unit * cols <= int64_t(64) * kSmU * kVec;
    const int64_t cap = (wave_tiles ? 64 : kThreads) * int64_t(kSmU) * kVec;
    int64_t R = (cap / cols) / unit * unit;
    if (R < unit) return plain();                // `unit` rows of this length do not fit one tile
    if (R > total_rows) R = ceil_div(total_rows, unit) * unit;
    const int64_t tiles = ceil_div(total_rows, R);
    const int64_t teams = wave_tiles ? kThreads / 64 : 1;
    const int64_t wgs = ceil_div(tiles, teams);
    // about four tiles per workgroup, at least one resident round of workgroups (three per CU at this register budget):
    // at 2^31 elements 768 / 12288 / 49152 / 262144 workgroups gave 0.665 / 0.669 / 0.724 / 0.685 of the HBM peak
    const int64_t resident = 256 * kSmWgPerCu;
    int64_t want = ceil_div(wgs, 4);
    if (want < resident) want = resident;
    const int grid = int(wgs < want ? wgs : want);
    FastDiv dc = make_fastdiv(uint32_t(cols)), dr = make_fastdiv(uint32_t(rows)), dh = make_fastdiv(uint32_t(H));
    hipStream_t s = static_cast<hipStream_t>(stream);
#define MESA_LAUNCH_S(T, TPT_) \
    hipLaunchKernelGGL((k_softmax_bwd<T, TPT_>), dim3(grid), dim3(kThreads), 0, s, yq, dy, dx, total_rows, uint32_t(cols), \
                       uint32_t(R), tiles, dc, dr, dh, alpha, beta)
#define MESA_LAUNCH_S_T(T) do { if (wave_tiles) MESA_LAUNCH_S(T, 64); else MESA_LAUNCH_S(T, kThreads); } while (0)
    MESA_FOR_DTYPE(dt, MESA_LAUNCH_S_T);
#undef MESA_LAUNCH_S_T
#undef MESA_LAUNCH_S
    return launch_status();
}
