// softmax_fwd.hip -- a Mesa softmax layer's forward in one pass over the logits (Sec. 3.1: the forward output
// is computed exactly; the output is what the layer saves, compressed -- Sec. 3.2 Eq. 3-4, 6-7):
//   per row  y_j = exp(s_j - max s) / sum_k exp(s_k - max s),
//   then for the stored y: codes with the running estimates as they are on entry and this batch's
//   per-head extrema, from which the estimates are moved afterwards (the single-pass forward).
//
// Tiling as in the backward kernel: rows of 197 or 49 elements start at odd byte offsets, so a team (one
// wave, or the workgroup for long rows) takes R consecutive rows with R*cols a multiple of 8 -- a run of
// whole, aligned 8-element vectors, read and written flat.  A vector touches at most two rows; its two
// partial maxima, then its two partial sums, go through LDS, where a group of lanes per row combines
// them.  The exponentials stay in registers between the passes.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "api_util.hpp"
#include "common.hpp"
#include "quantize.hpp"

namespace mesa {

constexpr int kSfU = 4;             // vectors per thread in a tile
constexpr int kSfMaxHeads = 1024;
constexpr int kSfWaves = 3;         // waves per SIMD the register budget is set for

template <int TPT> __device__ __forceinline__ void team_sync()
{
    if (TPT == kThreads) {
        __syncthreads();
    } else {   // the team is one wave: order its own LDS traffic
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
}

template <int WIDTH, bool MAX> __device__ __forceinline__ float lanes_combine(float v)
{
#pragma unroll
    for (int off = WIDTH / 2; off > 0; off >>= 1) {
        const float o = __shfl_xor(v, off, 64);
        v = MAX ? vmax(v, o) : v + o;
    }
    return v;
}

template <typename T, int TPT, bool SR>
__global__ __launch_bounds__(kThreads, kSfWaves) void k_softmax_fwd(const void *__restrict__ s_in, void *__restrict__ y,
                                                                  int8_t *__restrict__ q, int64_t total_rows, uint32_t cols,
                                                                  uint32_t R, int64_t tiles, FastDiv div_cols, FastDiv div_rows,
                                                                  FastDiv div_heads, const float *__restrict__ alpha,
                                                                  const float *__restrict__ beta, uint64_t seed, uint64_t offset,
                                                                  float *__restrict__ part)
{
    constexpr int kTileVec = TPT * kSfU;
    constexpr int kTeams = kThreads / TPT;
    __shared__ float2 head_tab[kSfMaxHeads];   // (255 / alpha, beta) per head
    __shared__ int lmn[kSfMaxHeads], lmx[kSfMaxHeads];
    __shared__ float PA[kTeams][kTileVec], PB[kTeams][kTileVec], rowD[kTeams][kTileVec];

    const uint32_t heads = div_heads.d;
    for (uint32_t h = threadIdx.x; h < heads; h += kThreads) {
        const float a = alpha[h];
        head_tab[h] = make_float2(a > 0.0f ? 255.0f / a : 0.0f, beta[h]);
        lmn[h] = order_key(__builtin_inff());
        lmx[h] = order_key(-__builtin_inff());
    }
    __syncthreads();

    const uint32_t team = threadIdx.x / TPT;
    const uint32_t tid = threadIdx.x % TPT;
    float *pa = PA[team], *pb = PB[team], *rd = rowD[team];

    // where this thread's vectors lie in their rows is the same in every tile: the row r1 a vector starts
    // in and how many of its elements belong to that row (the rest belong to the next one)
    uint32_t r1[kSfU], nb[kSfU];
#pragma unroll
    for (int u = 0; u < kSfU; ++u) {
        const uint32_t le = (u * TPT + tid) * kVec;
        r1[u] = fastdiv(le, div_cols);
        nb[u] = (r1[u] + 1) * cols - le;
    }

    for (int64_t tile = int64_t(blockIdx.x) * kTeams + team; tile < tiles; tile += int64_t(gridDim.x) * kTeams) {
        const int64_t row0 = tile * R;
        const uint32_t nrows = uint32_t((total_rows - row0 < int64_t(R)) ? (total_rows - row0) : int64_t(R));
        const uint32_t nelem = nrows * cols;
        const uint32_t nvec = (nelem + kVec - 1) / kVec;
        const int64_t e0 = row0 * cols;

        // a group of lanes per row combines the row's own part of its first vector with the vectors that start in it
        auto row_combine = [&](auto lanes, auto is_max) {
            constexpr uint32_t LPR = decltype(lanes)::value;
            constexpr bool MAX = decltype(is_max)::value;
            const uint32_t ln = tid & (LPR - 1);
            for (uint32_t r = tid / LPR; r < nrows; r += TPT / LPR) {
                const uint32_t start = r * cols;
                const uint32_t vs = start >> 3;
                const uint32_t ve = (start + cols - 1) >> 3;
                float acc = MAX ? -__builtin_inff() : 0.0f;
                if (ln == 0) acc = (start & 7u) ? pb[vs] : pa[vs];
                for (uint32_t v = vs + 1 + ln; v <= ve; v += LPR) acc = MAX ? vmax(acc, pa[v]) : acc + pa[v];
                acc = lanes_combine<LPR, MAX>(acc);
                if (ln == 0) rd[r] = MAX ? acc : 1.0f / acc;
            }
        };
        auto rows_of = [&](auto is_max) {
            if (cols <= 56) row_combine(std::integral_constant<uint32_t, 8>(), is_max);   // at most 8 vectors touch such a row
            else row_combine(std::integral_constant<uint32_t, 16>(), is_max);
        };

        float ev[kSfU][8];
        // pass 1: the logits, and each vector's two partial maxima
#pragma unroll
        for (int u = 0; u < kSfU; ++u) {
            const uint32_t v = u * TPT + tid;
            if (v < nvec) {
                const uint32_t le = v * kVec;
                const int64_t e = e0 + le;
                if (le + kVec <= nelem) {
                    Store<T>::unpack(Nt<T>::load(s_in, e), ev[u]);
                } else {   // ragged end of the whole tensor
#pragma unroll
                    for (int j = 0; j < 8; ++j) ev[u][j] = le + j < nelem ? Store<T>::load1(s_in, e + j) : -__builtin_inff();
                }
                float mA = -__builtin_inff(), mB = -__builtin_inff();
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    if (uint32_t(j) < nb[u]) mA = vmax(mA, ev[u][j]);
                    else mB = vmax(mB, ev[u][j]);
                }
                pa[v] = mA;
                pb[v] = mB;
            }
        }
        team_sync<TPT>();
        rows_of(std::true_type());
        team_sync<TPT>();

        // pass 2: exponentials (kept), and each vector's two partial sums
#pragma unroll
        for (int u = 0; u < kSfU; ++u) {
            const uint32_t v = u * TPT + tid;
            if (v < nvec) {
                const uint32_t r2 = (r1[u] + 1 < nrows) ? r1[u] + 1 : r1[u];
                const float mA = rd[r1[u]], mB = rd[r2];
                float sA = 0.0f, sB = 0.0f;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const bool first = uint32_t(j) < nb[u];
                    const float t = (ev[u][j] - (first ? mA : mB)) * 1.4426950408889634f;
                    const float ex = __builtin_amdgcn_exp2f(t);   // 0 for the padding beyond the tensor's end
                    ev[u][j] = ex;
                    sA += first ? ex : 0.0f;
                    sB += first ? 0.0f : ex;
                }
                pa[v] = sA;
                pb[v] = sB;
            }
        }
        team_sync<TPT>();
        rows_of(std::false_type());   // leaves 1 / sum
        team_sync<TPT>();

        // pass 3: y, rounded to its storage type; from the stored value the code and the extrema
        const uint32_t slab_first = fastdiv(uint32_t(row0), div_rows);
        const uint32_t slab_last = fastdiv(uint32_t(row0) + nrows - 1, div_rows);
        const bool one_head = slab_first == slab_last;     // uniform in the team
        const uint32_t head_first = slab_first - fastdiv(slab_first, div_heads) * heads;
        const float2 prmT = head_tab[head_first];
        float tmn = __builtin_inff(), tmx = -__builtin_inff();   // this thread's extrema in a one-head tile
#pragma unroll
        for (int u = 0; u < kSfU; ++u) {
            const uint32_t v = u * TPT + tid;
            if (v < nvec) {
                const uint32_t le = v * kVec;
                const int64_t e = e0 + le;
                const uint32_t r2 = (r1[u] + 1 < nrows) ? r1[u] + 1 : r1[u];
                const float iA = rd[r1[u]], iB = rd[r2];
                float yv[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) yv[j] = ev[u][j] * ((uint32_t(j) < nb[u]) ? iA : iB);
                const typename Store<T>::raw_t raw = Store<T>::pack(yv);
                float f[8];
                Store<T>::unpack(raw, f);                  // y as stored
                float bits[8], w[8];
                if (SR) sr_bits(seed, offset + uint64_t(e >> 3), bits);
                uint32_t hA = head_first, hB = head_first;
                if (one_head) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) w[j] = quantize_one<SR>(f[j], prmT.x, prmT.y, SR ? bits[j] : 0.0f);
                } else {   // heads of the row the vector starts in and of the next row
                    const uint32_t grow = uint32_t(row0) + r1[u];
                    const uint32_t slab = fastdiv(grow, div_rows);
                    hA = slab - fastdiv(slab, div_heads) * heads;
                    hB = (grow + 1 - slab * div_rows.d == div_rows.d) ? ((hA + 1 == heads) ? 0u : hA + 1) : hA;
                    const float2 pA = head_tab[hA], pB = head_tab[hB];
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const bool first = uint32_t(j) < nb[u];
                        w[j] = quantize_one<SR>(f[j], first ? pA.x : pB.x, first ? pA.y : pB.y, SR ? bits[j] : 0.0f);
                    }
                }
                // extrema of the stored values: per part of the vector where two heads may meet, else of the whole vector
                float mnA = __builtin_inff(), mxA = -__builtin_inff(), mnB = __builtin_inff(), mxB = -__builtin_inff();
                if (le + kVec <= nelem) {
                    Nt<T>::store(y, e, raw);
                    nt_store<u32x2>(q + e, pack_codes(w));
                    if (one_head) {
#pragma unroll
                        for (int j = 0; j < 8; ++j) { tmn = vmin(tmn, f[j]); tmx = vmax(tmx, f[j]); }
                    } else {
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            if (uint32_t(j) < nb[u]) { mnA = vmin(mnA, f[j]); mxA = vmax(mxA, f[j]); }
                            else { mnB = vmin(mnB, f[j]); mxB = vmax(mxB, f[j]); }
                        }
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (le + j < nelem) {
                            Store<T>::store1(y, e + j, f[j]);
                            q[e + j] = int8_t(int(clamp_code(w[j])) - 128);
                            if (uint32_t(j) < nb[u]) { mnA = vmin(mnA, f[j]); mxA = vmax(mxA, f[j]); }
                            else { mnB = vmin(mnB, f[j]); mxB = vmax(mxB, f[j]); }
                        }
                    if (one_head) {
                        tmn = vmin(tmn, vmin(mnA, mnB));
                        tmx = vmax(tmx, vmax(mxA, mxB));
                    }
                }
                if (!one_head) {   // the few tiles that straddle two attention maps: straight to the heads' slots
                    if (mnA <= mxA) { atomicMin(&lmn[hA], order_key(mnA)); atomicMax(&lmx[hA], order_key(mxA)); }
                    if (mnB <= mxB) { atomicMin(&lmn[hB], order_key(mnB)); atomicMax(&lmx[hB], order_key(mxB)); }
                }
            }
        }
        if (one_head) {   // one pair of LDS atomics per wave
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) {
                tmn = vmin(tmn, __shfl_xor(tmn, off, 64));
                tmx = vmax(tmx, __shfl_xor(tmx, off, 64));
            }
            if ((threadIdx.x & 63) == 0 && tmn <= tmx) {
                atomicMin(&lmn[head_first], order_key(tmn));
                atomicMax(&lmx[head_first], order_key(tmx));
            }
        }
        team_sync<TPT>();   // the next tile rewrites the partial results
    }
    __syncthreads();
    float *out = part + int64_t(blockIdx.x) * 2 * heads;
    for (uint32_t h = threadIdx.x; h < heads; h += kThreads) {
        out[h] = order_val(lmn[h]);
        out[heads + h] = order_val(lmx[h]);
    }
}

// tiles, grid and workspace of k_softmax_fwd
struct SfPlan {
    bool ok, wave_tiles;
    int64_t R, tiles;
    int grid;
};

static SfPlan sf_plan(int64_t total_rows, int64_t cols)
{
    SfPlan p{};
    // rows per tile: a multiple of 8/gcd(cols, 8) so that every tile starts on a vector boundary.
    // Short rows: one wave per tile (2048 elements); long rows: the whole workgroup (8192 elements).
    int64_t gc = cols, b8 = 8;
    while (b8) { int64_t t = gc % b8; gc = b8; b8 = t; }
    const int64_t unit = 8 / gc;
    p.wave_tiles = unit * cols <= int64_t(64) * kSfU * kVec;
    const int64_t cap = (p.wave_tiles ? 64 : kThreads) * int64_t(kSfU) * kVec;
    p.R = (cap / cols) / unit * unit;
    p.ok = p.R >= unit;                                    // else `unit` rows of this length do not fit one tile
    if (!p.ok) return p;
    if (p.R > total_rows) p.R = ceil_div(total_rows, unit) * unit;
    p.tiles = ceil_div(total_rows, p.R);
    const int64_t wgs = ceil_div(p.tiles, p.wave_tiles ? kThreads / 64 : 1);
    const int64_t resident = 256 * kSfWaves;               // one resident round of workgroups, striding over the tiles
    p.grid = int(wgs < resident ? wgs : resident);
    return p;
}

size_t softmax_fwd_ws_bytes(int64_t total_rows, int64_t H, int64_t cols)
{
    if (total_rows <= 0 || H <= 0 || cols < kVec || H > kSfMaxHeads || total_rows >= (int64_t(1) << 31)) return 16;
    const SfPlan p = sf_plan(total_rows, cols);
    if (!p.ok) return 16;
    return size_t(p.grid) * 2 * size_t(H) * sizeof(float) + 16;
}

}  // namespace mesa

using namespace mesa;

extern "C" MESA_EXPORT mesa_status mesa_softmax_fwd_q(const void *s_in, int64_t B, int64_t H, int64_t rows, int64_t cols, float *alpha,
                                                      float *beta, float lambda, void *y, int8_t *q, mesa_round mode, uint64_t seed,
                                                      uint64_t offset, void *ws, size_t ws_bytes, mesa_dtype dt, void *stream)
{
    if (!valid_dtype(dt) || B < 0 || H < 0 || rows < 0 || cols < 0) return MESA_ERR_INVALID_ARG;
    if (mode != MESA_ROUND_NEAREST_EVEN && mode != MESA_ROUND_STOCHASTIC) return MESA_ERR_INVALID_ARG;
    if (!(lambda >= 0.0f && lambda <= 1.0f)) return MESA_ERR_INVALID_ARG;
    if (B == 0 || H == 0 || rows == 0 || cols == 0) return MESA_OK;
    if (!s_in || !y || !q || !alpha || !beta || !aligned16(s_in) || !aligned16(y) || !aligned16(q) || !aligned4(alpha) ||
        !aligned4(beta) || y == s_in)
        return MESA_ERR_INVALID_ARG;
    if (H > kSfMaxHeads || rows >= (int64_t(1) << 31) || cols < kVec) return MESA_ERR_UNSUPPORTED;
    const long double tr = (long double)B * (long double)H * (long double)rows;
    if (tr >= 2147483648.0L) return MESA_ERR_UNSUPPORTED;
    const int64_t total_rows = B * H * rows;
    const SfPlan p = sf_plan(total_rows, cols);
    if (!p.ok) return MESA_ERR_UNSUPPORTED;
    if (!ws || !aligned16(ws) || ws_bytes < softmax_fwd_ws_bytes(total_rows, H, cols)) return MESA_ERR_WORKSPACE;
    FastDiv dc = make_fastdiv(uint32_t(cols)), dr = make_fastdiv(uint32_t(rows)), dh = make_fastdiv(uint32_t(H));
    hipStream_t s = static_cast<hipStream_t>(stream);
    float *part = static_cast<float *>(ws);
    const bool sr = mode == MESA_ROUND_STOCHASTIC;
#define MESA_LAUNCH_SF(T, TPT_, SR_) \
    hipLaunchKernelGGL((k_softmax_fwd<T, TPT_, SR_>), dim3(p.grid), dim3(kThreads), 0, s, s_in, y, q, total_rows, uint32_t(cols), \
                       uint32_t(p.R), p.tiles, dc, dr, dh, alpha, beta, seed, offset, part)
#define MESA_LAUNCH_SF_T(T) \
    do { \
        if (p.wave_tiles) { if (sr) MESA_LAUNCH_SF(T, 64, true); else MESA_LAUNCH_SF(T, 64, false); } \
        else { if (sr) MESA_LAUNCH_SF(T, kThreads, true); else MESA_LAUNCH_SF(T, kThreads, false); } \
    } while (0)
    MESA_FOR_DTYPE(dt, MESA_LAUNCH_SF_T);
#undef MESA_LAUNCH_SF_T
#undef MESA_LAUNCH_SF
    launch_ema_finalize(part, p.grid, uint32_t(H), alpha, beta, lambda, 0, 0, 0.0f, s);
    return launch_status();
}
