// softmax_fwd.hip -- a Mesa softmax layer's forward in one pass over the logits (Sec. 3.1: the forward output
// is computed exactly; the output is what the layer saves, compressed -- Sec. 3.2 Eq. 3-4, 6-7):
//   per row  y_j = exp(s_j - max s) / sum_k exp(s_k - max s),
//   then for the stored y: codes with the running estimates as they are on entry and this batch's
//   per-head extrema, from which the estimates are moved afterwards (the single-pass forward).
//
// Three kernels.  Rows of up to 256 elements (the attention maps of the paper's models: 197, 49): k_softmax_fwd_rows,
// further down -- tiles staged flat through LDS, a row per group of lanes.  Longer rows of 8k elements, up to 4096:
// k_softmax_fwd_wave, after it -- a row per group of lanes, in registers.  Other long rows: k_softmax_fwd, tiled as
// the backward kernel: rows start at odd byte offsets, so a team (one wave, or the workgroup for long rows) takes
// R consecutive rows with R*cols a multiple of 8 -- a run of whole, aligned 8-element vectors, read and written
// flat.  A vector touches at most two rows; its two partial maxima, then its two partial sums, go through LDS,
// where a group of lanes per row combines them.  The exponentials stay in registers between the passes.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "api_util.hpp"
#include "common.hpp"
#include "quantize.hpp"
#include "softmax_rows.hpp"

namespace mesa {

constexpr int kSfU = 4;             // vectors per thread in a tile
constexpr int kSfMaxHeads = 1024;
constexpr int kSfWaves = 3;         // waves per SIMD the register budget is set for

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

// ---------------------------------------------------------------------------------------------
// Short rows (at most 256 elements): a row per group of LPR lanes.
//
// A wave owns a tile of R consecutive rows, R * cols a multiple of 8 as above.  Flat phase: the tile's
// aligned 8-element vectors are read from memory and copied to the wave's LDS region as they lie; the random
// bits of stochastic rounding are generated per vector (one Philox block covers 8 consecutive elements) and laid
// out next to them, 16 bits per element in element order.  Row phase: 64 / LPR rows at a time, lane l of a
// row's group takes elements l, l + LPR, ... into registers (EPL slots); maximum and sum are reductions inside
// the group; y is rounded to its storage type and written back over the logits, its code next to it.  Flat
// phase: the finished vectors of y and of the codes leave as aligned 16- and 8-byte stores.  A lane's extrema
// stay in registers as long as its rows belong to one head.
// ---------------------------------------------------------------------------------------------
constexpr int kSfRowWaves = 4;      // waves per SIMD the row kernel's register budget is set for

// TIGHT: cols > LPR * (EPL - 1), so only the last slot of a lane can lie beyond the row's end
template <typename T, int LPR, int EPL, bool TIGHT, bool SR>
__global__ __launch_bounds__(kThreads, kSfRowWaves) void k_softmax_fwd_rows(const void *__restrict__ s_in, void *__restrict__ y,
                                                                  int8_t *__restrict__ q, int64_t total_rows, uint32_t cols,
                                                                  uint32_t R, int64_t tiles, FastDiv div_rows, FastDiv div_heads,
                                                                  const float *__restrict__ alpha, const float *__restrict__ beta,
                                                                  uint64_t seed, uint64_t offset, float *__restrict__ part,
                                                                  uint32_t tab_bytes, uint32_t wave_bytes)
{
    constexpr int kB = Store<T>::kBytes;
    constexpr int RPP = 64 / LPR;                        // rows per pass
    constexpr int kWaves = kThreads / 64;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const uint32_t heads = div_heads.d;
    float2 *head_tab = reinterpret_cast<float2 *>(smem);              // (255 / alpha, beta) per head
    int *lmn = reinterpret_cast<int *>(smem + heads * sizeof(float2));
    int *lmx = lmn + heads;
    for (uint32_t h = threadIdx.x; h < heads; h += kThreads) {
        const float a = alpha[h];
        head_tab[h] = make_float2(a > 0.0f ? 255.0f / a : 0.0f, beta[h]);
        lmn[h] = order_key(__builtin_inff());
        lmx[h] = order_key(-__builtin_inff());
    }
    __syncthreads();

    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint32_t sub = lane / LPR, l = lane % LPR;
    const uint32_t tile_cap = R * cols;                  // elements of a whole tile, a multiple of 8
    unsigned char *xs = smem + tab_bytes + wave * wave_bytes;         // logits, then y
    unsigned char *ns = xs + tile_cap * kB;                           // 16 random bits per element
    unsigned char *qs = ns + (SR ? tile_cap * 2 : 0);                 // codes

    uint32_t cur_h = 0;
    float mn = __builtin_inff(), mx = -__builtin_inff();              // extrema of this lane's elements of head cur_h
    auto flush = [&]() {                                              // a whole lane group at a time
        const float a = lanes_extreme_dpp<LPR, false>(mn), b = lanes_extreme_dpp<LPR, true>(mx);
        if (l == 0 && a <= b) {
            atomicMin(&lmn[cur_h], order_key(a));
            atomicMax(&lmx[cur_h], order_key(b));
        }
    };

    // The whole vectors of a tile are fetched one tile ahead: the loads are issued before the row phase of
    // the tile before and have arrived when it ends.
    typename Store<T>::raw_t raw[kSrFlat];
    auto fetch = [&](int64_t t) {
        const int64_t row0 = t * R;
        const uint32_t nrows = uint32_t((total_rows - row0 < int64_t(R)) ? (total_rows - row0) : int64_t(R));
        const uint32_t nfull = nrows * cols / kVec;
#pragma unroll
        for (int u = 0; u < kSrFlat; ++u) {
            const uint32_t v = u * 64 + lane;
            if (v < nfull) raw[u] = Nt<T>::load(s_in, row0 * cols + v * kVec);
        }
    };
    const int64_t tile_step = int64_t(gridDim.x) * kWaves;
    int64_t tile = int64_t(blockIdx.x) * kWaves + wave;
    if (tile < tiles) fetch(tile);
    for (; tile < tiles; tile += tile_step) {
        const int64_t row0 = tile * R;
        const uint32_t nrows = uint32_t((total_rows - row0 < int64_t(R)) ? (total_rows - row0) : int64_t(R));
        const uint32_t nelem = nrows * cols;
        const uint32_t nvec = (nelem + kVec - 1) / kVec;
        const int64_t e0 = row0 * cols;                  // a multiple of 8

        // flat: random bits and the fetched logits -> LDS
        const uint32_t nfull = nelem / kVec, tail = nelem % kVec;    // a tail: only at the end of the whole tensor
        if (lane < tail) LdsElem<T>::put(xs + (nfull * kVec + lane) * kB, Store<T>::load1(s_in, e0 + nfull * kVec + lane));
        if (SR) {
#pragma unroll 1   // one block at a time: four interleaved generators would not fit the register budget
            for (int u = 0; u < kSrFlat; ++u) {
                const uint32_t v = u * 64 + lane;
                if (v < nvec) {
                    const uint64_t counter = offset + uint64_t(e0 >> 3) + v;
                    uint32_t w[4];
                    philox4x32_10(uint32_t(counter), uint32_t(counter >> 32), uint32_t(seed), uint32_t(seed >> 32), w);
                    const u32x4 w4 = {w[0], w[1], w[2], w[3]};
                    *reinterpret_cast<u32x4 *>(ns + v * 16) = w4;     // element e's bits: halfword e of the block
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kSrFlat; ++u) {
            const uint32_t v = u * 64 + lane;
            if (v < nfull) Store<T>::store(xs, int64_t(v) * kVec, raw[u]);
        }
        team_sync<64>();
        if (tile + tile_step < tiles) fetch(tile + tile_step);

        // rows
        for (uint32_t p0 = 0; p0 < nrows; p0 += RPP) {
            const uint32_t r = p0 + sub;
            const bool live = r < nrows;
            const uint32_t eb = (live ? r : p0) * cols + l;           // groups without a row repeat the pass's first
            // slot k is a constant distance from the lane's first element: one address register per array
            unsigned char *xp = xs + eb * kB;
            const unsigned char *np = ns + eb * 2;
            unsigned char *qp = qs + eb;
            float x[EPL];
#pragma unroll
            for (int k = 0; k < EPL; ++k) {
                const float v = LdsElem<T>::get(xp + k * LPR * kB);
                const bool valid = (TIGHT && k < EPL - 1) || l + k * LPR < cols;
                x[k] = valid ? v : -__builtin_inff();
            }
            // the random bits are read before anything is written back: reads after a write to the same
            // array would each wait for it
            uint32_t bits[EPL];
            if (SR) {
#pragma unroll
                for (int k = 0; k < EPL; ++k) bits[k] = *reinterpret_cast<const uint16_t *>(np + k * LPR * 2);   // unused slots: discarded
            }
            float m = x[0];
#pragma unroll
            for (int k = 1; k < EPL; ++k) m = vmax(m, x[k]);
            m = lanes_extreme_dpp<LPR, true>(m);
            const float ml = m * 1.4426950408889634f;
            float sum = 0.0f;
#pragma unroll
            for (int k = 0; k < EPL; ++k) {
                x[k] = __builtin_amdgcn_exp2f(__builtin_fmaf(x[k], 1.4426950408889634f, -ml));   // 0 in unused slots
                sum += x[k];
            }
            sum = lanes_sum_dpp<LPR>(sum);
            const float inv = 1.0f / sum;
            if (live) {
                const uint32_t grow = uint32_t(row0) + r;
                const uint32_t slab = fastdiv(grow, div_rows);
                const uint32_t h = slab - fastdiv(slab, div_heads) * heads;
                if (h != cur_h) {
                    flush();
                    cur_h = h;
                    mn = __builtin_inff();
                    mx = -__builtin_inff();
                }
                const float2 prm = head_tab[h];
#pragma unroll
                for (int k = 0; k < EPL; ++k) {
                    const bool valid = (TIGHT && k < EPL - 1) || l + k * LPR < cols;
                    if (valid) {
                        const float f = LdsElem<T>::put(xp + k * LPR * kB, x[k] * inv);   // y as stored
                        const float w = quantize_one<SR>(f, prm.x, prm.y, SR ? float(bits[k]) : 0.0f);
                        qp[k * LPR] = (unsigned char)(__builtin_amdgcn_cvt_pk_u8_f32(w, 0, 0u) ^ 0x80u);   // saturates to [0, 255]
                        mn = vmin(mn, f);
                        mx = vmax(mx, f);
                    }
                }
            }
        }
        team_sync<64>();

        // flat: LDS -> memory
#pragma unroll
        for (int u = 0; u < kSrFlat; ++u) {
            const uint32_t v = u * 64 + lane;
            if (v < nfull) {
                const uint32_t le = v * kVec;
                Nt<T>::store(y, e0 + le, Store<T>::load(xs, int64_t(le)));
                nt_store<u32x2>(q + e0 + le, *reinterpret_cast<const u32x2 *>(qs + le));
            }
        }
        if (lane < tail) {
            const uint32_t le = nfull * kVec + lane;
            Store<T>::store1(y, e0 + le, LdsElem<T>::get(xs + le * kB));   // exact: the value is already of type T
            q[e0 + le] = int8_t(qs[le]);
        }
        team_sync<64>();   // the next tile rewrites the region
    }
    flush();
    __syncthreads();
    float *out = part + int64_t(blockIdx.x) * 2 * heads;
    for (uint32_t h = threadIdx.x; h < heads; h += kThreads) {
        out[h] = order_val(lmn[h]);
        out[heads + h] = order_val(lmx[h]);
    }
}

// ---------------------------------------------------------------------------------------------
// Rows of 8k elements, 256 < cols <= 4096 (long sequences): a row per group of LPR lanes (a wave, or half or a quarter
// of one where that fills the lanes better).  Such rows start on vector boundaries, so a lane holds NV whole vectors of
// ONE row (vector u*LPR + its index in the group), all requested before the first is used; maximum and sum are
// reductions inside the group -- no LDS traffic, no barrier.  The exponentials stay in registers between the passes.
// A wave walks blocks of 64/LPR consecutive rows a grid stride apart (the entry point picks LPR < 64 only when the rows
// per attention map are a multiple of 64/LPR, so that a block lies in one head) and keeps the extrema of the stored
// values in registers for as long as its rows belong to one head (one pair of LDS atomics per wave and head).
// ---------------------------------------------------------------------------------------------
constexpr int kSwMaxCols = 4096;

template <typename T, int LPR, int NV, bool SR>
__global__ __launch_bounds__(kThreads, NV <= 4 ? 4 : 3) void k_softmax_fwd_wave(const void *__restrict__ s_in, void *__restrict__ y,
                                                                              int8_t *__restrict__ q, int64_t total_rows, uint32_t cols,
                                                                              FastDiv div_rows, FastDiv div_heads,
                                                                              const float *__restrict__ alpha, const float *__restrict__ beta,
                                                                              uint64_t seed, uint64_t offset, float *__restrict__ part)
{
    constexpr int RPW = 64 / LPR;              // rows a wave takes at a time
    __shared__ float2 head_tab[kSfMaxHeads];   // (255 / alpha, beta) per head
    __shared__ int lmn[kSfMaxHeads], lmx[kSfMaxHeads];
    const uint32_t heads = div_heads.d;
    for (uint32_t h = threadIdx.x; h < heads; h += kThreads) {
        const float a = alpha[h];
        head_tab[h] = make_float2(a > 0.0f ? 255.0f / a : 0.0f, beta[h]);
        lmn[h] = order_key(__builtin_inff());
        lmx[h] = order_key(-__builtin_inff());
    }
    __syncthreads();

    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t sub = lane / LPR, lr = lane % LPR;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t nvec = cols >> 3;
    constexpr uint32_t kNone = 0xFFFFFFFFu;
    uint32_t cur = kNone;                                        // the head whose extrema tmn, tmx hold
    float tmn = __builtin_inff(), tmx = -__builtin_inff();
    auto flush = [&]() {
        tmn = -lanes_combine<64, true>(-tmn);
        tmx = lanes_combine<64, true>(tmx);
        if (lane == 0 && tmn <= tmx) {
            atomicMin(&lmn[cur], order_key(tmn));
            atomicMax(&lmx[cur], order_key(tmx));
        }
        tmn = __builtin_inff();
        tmx = -__builtin_inff();
    };

    const int64_t blocks = total_rows / RPW;                     // total_rows is a multiple of RPW
    for (int64_t blk = int64_t(blockIdx.x) * (kThreads / 64) + wave; blk < blocks; blk += int64_t(gridDim.x) * (kThreads / 64)) {
        const int64_t row0 = blk * RPW;
        const uint32_t slab = fastdiv(uint32_t(row0), div_rows);
        const uint32_t head = slab - fastdiv(slab, div_heads) * heads;
        if (head != cur) {
            if (cur != kNone) flush();
            cur = head;
        }
        const float2 prm = head_tab[head];
        const int64_t e0 = (row0 + sub) * int64_t(cols);

        typename Store<T>::raw_t raw[NV];
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const uint32_t v = u * LPR + lr;
            if (v < nvec) raw[u] = Nt<T>::load(s_in, e0 + int64_t(v) * kVec);
        }
        float ev[NV][8];
        float m = -__builtin_inff();
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const uint32_t v = u * LPR + lr;
            if (v < nvec) {
                Store<T>::unpack(raw[u], ev[u]);
#pragma unroll
                for (int j = 0; j < 8; ++j) m = vmax(m, ev[u][j]);
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) ev[u][j] = -__builtin_inff();   // exponential 0
            }
        }
        m = lanes_combine<LPR, true>(m);
        float sum = 0.0f;
#pragma unroll
        for (int u = 0; u < NV; ++u)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float ex = __builtin_amdgcn_exp2f((ev[u][j] - m) * 1.4426950408889634f);
                ev[u][j] = ex;
                sum += ex;
            }
        sum = lanes_combine<LPR, false>(sum);
        const float inv = 1.0f / sum;

        // y, rounded to its storage type; from the stored value the code and the extrema
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const uint32_t v = u * LPR + lr;
            if (v < nvec) {
                const int64_t e = e0 + int64_t(v) * kVec;
                float yv[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) yv[j] = ev[u][j] * inv;
                const typename Store<T>::raw_t out = Store<T>::pack(yv);
                float f[8], bits[8], w[8];
                Store<T>::unpack(out, f);                  // y as stored
                if (SR) sr_bits(seed, offset + uint64_t(e >> 3), bits);
#pragma unroll
                for (int j = 0; j < 8; ++j) w[j] = quantize_one<SR>(f[j], prm.x, prm.y, SR ? bits[j] : 0.0f);
                Nt<T>::store(y, e, out);
                nt_store<u32x2>(q + e, pack_codes(w));
#pragma unroll
                for (int j = 0; j < 8; ++j) { tmn = vmin(tmn, f[j]); tmx = vmax(tmx, f[j]); }
            }
        }
    }
    if (cur != kNone) flush();
    __syncthreads();
    float *out = part + int64_t(blockIdx.x) * 2 * heads;
    for (uint32_t h = threadIdx.x; h < heads; h += kThreads) {
        out[h] = order_val(lmn[h]);
        out[heads + h] = order_val(lmx[h]);
    }
}

static bool sw_fits(int64_t cols) { return cols % kVec == 0 && cols > kSrMaxCols && cols <= kSwMaxCols; }

// lanes per row and vectors per lane: the smallest product that holds the row's vectors, among the shapes built
struct SwPlan {
    int lpr, nv, grid;
};
static SwPlan sw_plan(int64_t total_rows, int64_t rows, int64_t cols)
{
    const int64_t nvec = cols / kVec;
    SwPlan p{};
    if (nvec <= 48 && rows % 4 == 0) { p.lpr = 16; p.nv = 3; }
    else if (nvec <= 64 && rows % 2 == 0) { p.lpr = 32; p.nv = 2; }
    else if (nvec > 64 && nvec <= 96 && rows % 2 == 0) { p.lpr = 32; p.nv = 3; }
    else if (nvec <= 128) { p.lpr = 64; p.nv = 2; }
    else if (nvec <= 192) { p.lpr = 64; p.nv = 3; }
    else if (nvec <= 256) { p.lpr = 64; p.nv = 4; }
    else { p.lpr = 64; p.nv = 8; }
    // one resident round: four workgroups per CU, two where a lane holds eight vectors
    const int64_t wgs = ceil_div(total_rows / (64 / p.lpr), kThreads / 64), resident = 256 * (p.nv <= 4 ? 4 : 3);
    p.grid = int(wgs < resident ? wgs : resident);
    return p;
}
// the largest grid any shape of the plan may take for these rows (what the workspace is sized for)
static int sw_grid_bound(int64_t total_rows)
{
    const int64_t wgs = ceil_div(total_rows, kThreads / 64);
    return int(wgs < 1024 ? wgs : 1024);
}

struct SrPlan {
    bool ok, tight;
    int lpr, epl, grid;
    int64_t R, tiles;
    uint32_t tab_bytes, wave_bytes;
    size_t lds;
};

static SrPlan sr_plan(int64_t total_rows, int64_t H, int64_t cols, int elem_bytes, bool sr)
{
    SrPlan p{};
    if (cols > kSrMaxCols) return p;
    const SrShape sh = sr_shape(total_rows, cols);
    p.lpr = sh.lpr; p.epl = sh.epl; p.tight = sh.tight; p.R = sh.R; p.tiles = sh.tiles;
    p.tab_bytes = uint32_t((H * 16 + 15) / 16 * 16);
    p.wave_bytes = uint32_t((p.R * cols * (elem_bytes + (sr ? 2 : 0) + 1) + 15) / 16 * 16);
    p.lds = size_t(p.tab_bytes) + size_t(kThreads / 64) * p.wave_bytes + kSrSlack;
    p.ok = p.lds <= 64 * 1024;
    if (!p.ok) return p;
    int64_t per_cu = int64_t(160 * 1024) / int64_t(p.lds);
    if (per_cu > kSfRowWaves) per_cu = kSfRowWaves;
    const int64_t wgs = ceil_div(p.tiles, kThreads / 64), resident = 256 * per_cu;
    p.grid = int(wgs < resident ? wgs : resident);
    return p;
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

// ---------------------------------------------------------------------------------------------
// Rows no kernel above takes (odd lengths too long for a tile, rows shorter than a vector that have no row plan, more
// heads than the tables hold): y by a plain kernel -- one workgroup per row, the row read three times --, then the
// single-pass quantizer on the stored y, which is how the call is defined.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kThreads) void k_softmax_fwd_plain_y(const void *__restrict__ s_in, void *__restrict__ y, int64_t total_rows,
                                                                  uint32_t cols)
{
    __shared__ float red[kThreads / 64];
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    auto block_combine = [&](float v, auto is_max) {   // the same value in every thread; waves in a fixed order
        constexpr bool MAX = decltype(is_max)::value;
        v = lanes_combine<64, MAX>(v);
        if (lane == 0) red[wave] = v;
        __syncthreads();
        float r = red[0];
#pragma unroll
        for (int w = 1; w < kThreads / 64; ++w) r = MAX ? vmax(r, red[w]) : r + red[w];
        __syncthreads();
        return r;
    };
    for (int64_t row = blockIdx.x; row < total_rows; row += gridDim.x) {
        const int64_t e0 = row * int64_t(cols);
        float m = -__builtin_inff();
        for (uint32_t c = threadIdx.x; c < cols; c += kThreads) m = vmax(m, Store<T>::load1(s_in, e0 + c));
        m = block_combine(m, std::true_type());
        float sum = 0.0f;
        for (uint32_t c = threadIdx.x; c < cols; c += kThreads)
            sum += __builtin_amdgcn_exp2f((Store<T>::load1(s_in, e0 + c) - m) * 1.4426950408889634f);
        sum = block_combine(sum, std::false_type());
        const float inv = 1.0f / sum;
        for (uint32_t c = threadIdx.x; c < cols; c += kThreads)
            Store<T>::store1(y, e0 + c, __builtin_amdgcn_exp2f((Store<T>::load1(s_in, e0 + c) - m) * 1.4426950408889634f) * inv);
    }
}

// which kernel family takes the call; two_step: none of the single-pass kernels
struct SfRoute {
    bool two_step, wave_rows;
    SrPlan rp;
    SfPlan p;
};
static SfRoute sf_route(int64_t total_rows, int64_t H, int64_t cols, int elem_bytes, bool sr)
{
    SfRoute r{};
    if (H > kSfMaxHeads) { r.two_step = true; return r; }
    r.rp = sr_plan(total_rows, H, cols, elem_bytes, sr);
    if (r.rp.ok) return r;
    r.wave_rows = sw_fits(cols);
    if (r.wave_rows) return r;
    if (cols < kVec) { r.two_step = true; return r; }
    r.p = sf_plan(total_rows, cols);
    r.two_step = !r.p.ok;
    return r;
}

// enough for whichever kernel, storage type and rounding mode the call will use
size_t softmax_fwd_ws_bytes(int64_t total_rows, int64_t H, int64_t cols)
{
    if (total_rows <= 0 || H <= 0 || cols <= 0 || total_rows >= (int64_t(1) << 31)) return 16;
    int grid = 0;
    bool two_step = false;
    for (int eb = 2; eb <= 4; eb += 2)
        for (int sr = 0; sr < 2; ++sr) {
            const SfRoute r = sf_route(total_rows, H, cols, eb, sr != 0);
            two_step = two_step || r.two_step;
            if (r.rp.ok && r.rp.grid > grid) grid = r.rp.grid;
            if (r.p.ok && r.p.grid > grid) grid = r.p.grid;
            if (r.wave_rows && sw_grid_bound(total_rows) > grid) grid = sw_grid_bound(total_rows);
        }
    size_t need = grid == 0 ? 16 : size_t(grid) * 2 * size_t(H) * sizeof(float) + 16;
    if (two_step) {
        const size_t b = update_ws_bound(total_rows * cols, H);
        if (b > need) need = b;
    }
    return need;
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
    if (rows >= (int64_t(1) << 31) || cols >= (int64_t(1) << 31)) return MESA_ERR_UNSUPPORTED;
    const long double tr = (long double)B * (long double)H * (long double)rows;
    if (tr >= 2147483648.0L) return MESA_ERR_UNSUPPORTED;
    const int64_t total_rows = B * H * rows;
    const bool sr = mode == MESA_ROUND_STOCHASTIC;
    const SfRoute route = sf_route(total_rows, H, cols, dtype_bytes(dt), sr);
    const SrPlan &rp = route.rp;
    const SfPlan &p = route.p;
    const bool wave_rows = route.wave_rows;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (route.two_step) {
        // everything the second step would refuse is refused here, before anything is written
        const mesa_layout L = {B, H, rows * cols};
        const mesa_status st = check_layout(L);
        if (st != MESA_OK) return st;
        if (!ws || !aligned16(ws) || ws_bytes < update_ws_bytes(L.outer, L.groups, L.inner)) return MESA_ERR_WORKSPACE;
        const unsigned grid = unsigned(total_rows < (int64_t(1) << 20) ? total_rows : (int64_t(1) << 20));
#define MESA_LAUNCH_SP(T) hipLaunchKernelGGL((k_softmax_fwd_plain_y<T>), dim3(grid), dim3(kThreads), 0, s, s_in, y, total_rows, uint32_t(cols))
        MESA_FOR_DTYPE(dt, MESA_LAUNCH_SP);
#undef MESA_LAUNCH_SP
        if (launch_status() != MESA_OK) return MESA_ERR_LAUNCH;
        return mesa_quantize_update_fused(y, dt, L, alpha, beta, lambda, q, mode, seed, offset, ws, ws_bytes, stream);
    }
    if (!ws || !aligned16(ws) || ws_bytes < softmax_fwd_ws_bytes(total_rows, H, cols)) return MESA_ERR_WORKSPACE;
    FastDiv dc = make_fastdiv(uint32_t(cols)), dr = make_fastdiv(uint32_t(rows)), dh = make_fastdiv(uint32_t(H));
    float *part = static_cast<float *>(ws);
    if (rp.ok) {
#define MESA_LAUNCH_SR(T, LPR_, EPL_, TIGHT_, SR_) \
    hipLaunchKernelGGL((k_softmax_fwd_rows<T, LPR_, EPL_, TIGHT_, SR_>), dim3(rp.grid), dim3(kThreads), rp.lds, s, s_in, y, q, total_rows, \
                       uint32_t(cols), uint32_t(rp.R), rp.tiles, dr, dh, alpha, beta, seed, offset, part, rp.tab_bytes, rp.wave_bytes)
#define MESA_LAUNCH_SR_M(T, LPR_, EPL_, TIGHT_) \
    do { if (sr) MESA_LAUNCH_SR(T, LPR_, EPL_, TIGHT_, true); else MESA_LAUNCH_SR(T, LPR_, EPL_, TIGHT_, false); } while (0)
#define MESA_LAUNCH_SR_C(T, LPR_, EPL_) \
    do { if (rp.tight) MESA_LAUNCH_SR_M(T, LPR_, EPL_, true); else MESA_LAUNCH_SR_M(T, LPR_, EPL_, false); } while (0)
#define MESA_LAUNCH_SR_T(T) \
    do { \
        if (rp.lpr == 16) MESA_LAUNCH_SR_C(T, 16, 16); \
        else if (rp.epl == 25) MESA_LAUNCH_SR_C(T, 8, 25); \
        else if (rp.epl == 13) MESA_LAUNCH_SR_C(T, 8, 13); \
        else if (rp.epl == 16) MESA_LAUNCH_SR_C(T, 8, 16); \
        else if (rp.epl == 8) MESA_LAUNCH_SR_C(T, 8, 8); \
        else MESA_LAUNCH_SR_C(T, 8, 7); \
    } while (0)
        MESA_FOR_DTYPE(dt, MESA_LAUNCH_SR_T);
#undef MESA_LAUNCH_SR_T
#undef MESA_LAUNCH_SR_C
#undef MESA_LAUNCH_SR_M
#undef MESA_LAUNCH_SR
        if (launch_status() != MESA_OK) return MESA_ERR_LAUNCH;   // the consumer must not run on a workspace nobody wrote
        launch_ema_finalize(part, rp.grid, uint32_t(H), alpha, beta, lambda, 0, 0, 0.0f, s);
        return launch_status();
    }
    if (wave_rows) {
        const SwPlan wp = sw_plan(total_rows, rows, cols);
#define MESA_LAUNCH_SW(T, LPR_, NV_, SR_) \
    hipLaunchKernelGGL((k_softmax_fwd_wave<T, LPR_, NV_, SR_>), dim3(wp.grid), dim3(kThreads), 0, s, s_in, y, q, total_rows, uint32_t(cols), \
                       dr, dh, alpha, beta, seed, offset, part)
#define MESA_LAUNCH_SW_M(T, LPR_, NV_) \
    do { if (sr) MESA_LAUNCH_SW(T, LPR_, NV_, true); else MESA_LAUNCH_SW(T, LPR_, NV_, false); } while (0)
#define MESA_LAUNCH_SW_T(T) \
    do { \
        if (wp.lpr == 16) MESA_LAUNCH_SW_M(T, 16, 3); \
        else if (wp.lpr == 32 && wp.nv == 2) MESA_LAUNCH_SW_M(T, 32, 2); \
        else if (wp.lpr == 32) MESA_LAUNCH_SW_M(T, 32, 3); \
        else if (wp.nv == 2) MESA_LAUNCH_SW_M(T, 64, 2); \
        else if (wp.nv == 3) MESA_LAUNCH_SW_M(T, 64, 3); \
        else if (wp.nv == 4) MESA_LAUNCH_SW_M(T, 64, 4); \
        else MESA_LAUNCH_SW_M(T, 64, 8); \
    } while (0)
        MESA_FOR_DTYPE(dt, MESA_LAUNCH_SW_T);
#undef MESA_LAUNCH_SW_T
#undef MESA_LAUNCH_SW_M
#undef MESA_LAUNCH_SW
        if (launch_status() != MESA_OK) return MESA_ERR_LAUNCH;
        launch_ema_finalize(part, wp.grid, uint32_t(H), alpha, beta, lambda, 0, 0, 0.0f, s);
        return launch_status();
    }
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
    if (launch_status() != MESA_OK) return MESA_ERR_LAUNCH;
    launch_ema_finalize(part, p.grid, uint32_t(H), alpha, beta, lambda, 0, 0, 0.0f, s);
    return launch_status();
}
