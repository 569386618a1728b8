// linear_dw.hip -- Linear weight gradient at the de-quantized input (Sec. 3.1 Eq. 2 for y = x W^T):
//   dW[n,k] = sum_m dy[m,n]*x_hat[m,k],  x_hat[m,k] = (q[m,k]+128)*s_g(k) + beta_g(k)   (Sec. 3.2 Eq. 5)
// evaluated in the factored form
//   dW[n,k] = s_g(k) * P[n,k] + (beta_g(k) + 128 s_g(k)) * S0[n],   P = dy^T q,  S0[n] = sum_m dy[m,n]
// so that the matrix cores contract dy with the signed 8-bit codes themselves (exact in binary16,
// and centred, so P does not cancel against S0) and the per-column affine map is applied once to
// the finished sums.
//
// binary16 path, gfx950.  Both operands are row-major in the contraction index m, which is the
// layout the MFMA operands do NOT want (a lane holds 8 consecutive contraction values of one
// row).  gfx950's LDS transpose reads solve exactly this: the dy and code tiles are copied to
// LDS as they lie in memory, and ds_read_b64_tr_b16 / ds_read_b64_tr_b8 deliver, per lane, the
// column of four binary16 / eight int8 values it needs (within 16 lanes, lanes 4k..4k+3 -- resp.
// 2k, 2k+1 -- supply row k and lane i receives column i).  A workgroup of four waves owns a
// BN x BK tile of dW (each wave a quarter, as 32x32x16 MFMA tiles) for one slice of m; slices
// are combined in a fixed order by a second kernel that also applies the affine map.
// Workgroups are numbered so that those sharing a slice of m run on the same XCD (same L2).
#include <hip/hip_runtime.h>

#include <type_traits>

#include "api_util.hpp"
#include "common.hpp"

namespace mesa {

typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));
typedef short v4s __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef float v16f __attribute__((ext_vector_type(16)));

#define MESA_LDS3(T, p) ((__attribute__((address_space(3))) T *)(p))

constexpr int kDwBM = 32;        // contraction rows per LDS stage
constexpr int kDwXcd = 8;
constexpr int kDwPF = 3;         // stages prefetched into registers ahead of the one being multiplied

// BN x BK tile of dW per workgroup, WGN x WGK waves, each wave (BN/WGN) x (BK/WGK) as 32x32 MFMA tiles
template <int BN, int BK, int WGN, int WGK> struct DwCfg {
    static constexpr int NW = WGN * WGK;
    static constexpr int THREADS = NW * 64;
    static constexpr int WN = BN / WGN, WK = BK / WGK;  // wave tile
    static constexpr int TI = WN / 32, TJ = WK / 32;    // MFMA tiles per wave
    static constexpr int PA = BN * 2 + 64;              // LDS row pitch of the dy tile, bytes
    static constexpr int PB = BK + 32;                  // LDS row pitch of the code tile, bytes
    static constexpr int A_STAGE = kDwBM * PA;
    static constexpr int B_STAGE = kDwBM * PB;
    static constexpr int STAGE = A_STAGE + B_STAGE;
    static constexpr int A_CPR = BN / 8;                // 16-byte chunks per tile row
    static constexpr int B_CPR = BK / 16;
    static constexpr int A_TOTAL = kDwBM * A_CPR, B_TOTAL = kDwBM * B_CPR;
    static constexpr int A_CHUNKS = (A_TOTAL + THREADS - 1) / THREADS;
    static constexpr int B_CHUNKS = (B_TOTAL + THREADS - 1) / THREADS;
    static_assert(WN % 64 == 0 && WK % 32 == 0, "wave tile: an even number of 32-row MFMA tiles by whole 32-column tiles");
    static_assert(2 * STAGE <= 64 * 1024, "two stages must fit the default dynamic LDS limit");
};

// eight signed codes (bytes) -> eight binary16 values q: 0x6400 | (byte ^ 0x80) is 1152 + q exactly
__device__ __forceinline__ v8h codes_to_half8(v2i raw)
{
    v8h out;
    const h2 k1152 = {(_Float16)1152.0f, (_Float16)1152.0f};
#pragma unroll
    for (int w = 0; w < 2; ++w) {
        const uint32_t x = uint32_t(raw[w]) ^ 0x80808080u;
        const h2 a = as_h2(__builtin_amdgcn_perm(0x64646464u, x, 0x04010400u)) - k1152;   // bytes 0, 1
        const h2 b = as_h2(__builtin_amdgcn_perm(0x64646464u, x, 0x04030402u)) - k1152;   // bytes 2, 3
        out[4 * w + 0] = a.x; out[4 * w + 1] = a.y; out[4 * w + 2] = b.x; out[4 * w + 3] = b.y;
    }
    return out;
}

// P[split][n][k] = sum over the slice's m of dy[m][n] * q[m][k]   (q the signed code)
// S0[split][n]   = sum over the slice's m of dy[m][n]
template <int BN, int BK, int WGN, int WGK>
__global__ __launch_bounds__(WGN * WGK * 64, 1) void k_dw_f16(const int8_t *__restrict__ xq, const _Float16 *__restrict__ dy,
                                                              int64_t M, int K, int N, int tiles_n, int tiles_k, int splits,
                                                              int64_t rows_per_split, float *__restrict__ P,
                                                              float *__restrict__ S0)
{
    using C = DwCfg<BN, BK, WGN, WGK>;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int total = gridDim.x;                          // a multiple of 8
    const int logical = int(blockIdx.x % kDwXcd) * (total / kDwXcd) + int(blockIdx.x / kDwXcd);
    const int ntiles = tiles_n * tiles_k;
    if (logical >= ntiles * splits) return;               // padding workgroups; uniform, before any barrier
    const int split = logical / ntiles;
    const int t = logical - split * ntiles;
    const int tn = t / tiles_k, tk = t - tn * tiles_k;
    const int n0 = tn * BN, kk0 = tk * BK;
    const int64_t m_begin = int64_t(split) * rows_per_split;
    const int64_t m_end = (m_begin + rows_per_split < M) ? m_begin + rows_per_split : M;
    const int nstages = (m_end > m_begin) ? int((m_end - m_begin + kDwBM - 1) / kDwBM) : 0;

    const int wn = wave / WGK, wk = wave % WGK;
    const int blk = lane >> 4, sl = lane & 15;
    // byte offsets of this lane's transpose-read addresses inside a stage
    const int a_off = ((blk >> 1) * 8 + (sl >> 2)) * C::PA + (wn * C::WN + (blk & 1) * 16 + (sl & 3) * 4) * 2;
    const int b_off = C::A_STAGE + ((blk >> 1) * 8 + (sl >> 1)) * C::PB + wk * C::WK + (blk & 1) * 16 + (sl & 1) * 8;

    v16f acc[C::TI][C::TJ];
#pragma unroll
    for (int i = 0; i < C::TI; ++i)
#pragma unroll
        for (int j = 0; j < C::TJ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
    float s0[C::TI];
#pragma unroll
    for (int i = 0; i < C::TI; ++i) s0[i] = 0.0f;
    const bool do_s0 = (tk == 0) && (wk == 0);   // the waves whose row sums are written out

    // global -> register prefetch ring: stage s+1 .. s+kDwPF are in flight while stage s is multiplied,
    // enough bytes per CU to cover the latency of L2 / memory-side-cache hits at the rate MFMA consumes them.
    // Every load is unconditional from a clamped, always valid address; what lies outside the tile or
    // past the end of the slice is zeroed by a select, so the steady-state loop has no branches.
    u32x4 ring_a[kDwPF][C::A_CHUNKS], ring_b[kDwPF][C::B_CHUNKS];
    const _Float16 *pa[C::A_CHUNKS];
    const int8_t *pb[C::B_CHUNKS];
    int row_a[C::A_CHUNKS], row_b[C::B_CHUNKS], lds_a[C::A_CHUNKS], lds_b[C::B_CHUNKS];
    bool ok_a[C::A_CHUNKS], ok_b[C::B_CHUNKS];
#pragma unroll
    for (int i = 0; i < C::A_CHUNKS; ++i) {
        const int c = i * C::THREADS + tid;
        const int row = (c / C::A_CPR) % kDwBM, cc = c % C::A_CPR;
        const int n = n0 + cc * 8;
        ok_a[i] = c < C::A_TOTAL && n < N;
        row_a[i] = row;
        pa[i] = dy + (ok_a[i] ? n : 0);
        lds_a[i] = row * C::PA + cc * 16;
    }
#pragma unroll
    for (int i = 0; i < C::B_CHUNKS; ++i) {
        const int c = i * C::THREADS + tid;
        const int row = (c / C::B_CPR) % kDwBM, cc = c % C::B_CPR;
        const int kk = kk0 + cc * 16;
        ok_b[i] = c < C::B_TOTAL && kk < K;
        row_b[i] = row;
        pb[i] = xq + (ok_b[i] ? kk : 0);
        lds_b[i] = C::A_STAGE + row * C::PB + cc * 16;
    }
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    const int64_t m_last = (m_end > m_begin) ? m_end - 1 : 0;

    // EDGE = false: every row of the stage lies inside the slice (no row clamping, no row select).
    // The zeroing select is applied when the registers are written to LDS, not at the load, so that
    // nothing waits on a load before its stage is due.
    auto load_stage = [&](int64_t m_stage, u32x4 *ra, u32x4 *rb, auto edge) {
        constexpr bool EDGE = decltype(edge)::value;
#pragma unroll
        for (int i = 0; i < C::A_CHUNKS; ++i) {
            int64_t m = m_stage + row_a[i];
            if (EDGE) m = m < m_end ? m : m_last;
            ra[i] = *reinterpret_cast<const u32x4 *>(pa[i] + m * N);
        }
#pragma unroll
        for (int i = 0; i < C::B_CHUNKS; ++i) {
            int64_t m = m_stage + row_b[i];
            if (EDGE) m = m < m_end ? m : m_last;
            rb[i] = *reinterpret_cast<const u32x4 *>(pb[i] + m * K);
        }
    };
    auto store_stage = [&](unsigned char *st, int64_t m_stage, const u32x4 *ra, const u32x4 *rb, auto edge) {
        constexpr bool EDGE = decltype(edge)::value;
#pragma unroll
        for (int i = 0; i < C::A_CHUNKS; ++i)
            if (C::A_TOTAL % C::THREADS == 0 || i * C::THREADS + tid < C::A_TOTAL) {
                const bool ok = ok_a[i] && (!EDGE || m_stage + row_a[i] < m_end);
                *reinterpret_cast<u32x4 *>(st + lds_a[i]) = ok ? ra[i] : zero4;
            }
#pragma unroll
        for (int i = 0; i < C::B_CHUNKS; ++i)
            if (C::B_TOTAL % C::THREADS == 0 || i * C::THREADS + tid < C::B_TOTAL) {
                const bool ok = ok_b[i] && (!EDGE || m_stage + row_b[i] < m_end);
                *reinterpret_cast<u32x4 *>(st + lds_b[i]) = ok ? rb[i] : zero4;
            }
    };
    const std::true_type edge_yes;
    const std::false_type edge_no;

    // ---- software pipeline -------------------------------------------------------------------
    // A stage holds two contraction steps of 16 rows.  While the MFMAs of one step run, the wave
    // reads (and converts) the fragments of the next step, so LDS latency and the int8 -> binary16
    // conversion sit in the shadow of the matrix cores; the workgroup barrier falls between the two
    // MFMA batches of a stage, after this wave's last LDS read of the stage and its LDS writes of the
    // next one.  The sched_group_barrier calls spell the interleaving out for the scheduler.
    auto read_a = [&](const unsigned char *st, int ks, v8h af[C::TI]) {
#pragma unroll
        for (int i = 0; i < C::TI; ++i) {
            const unsigned char *p = st + a_off + ks * 16 * C::PA + i * 64;
            v4h lo = __builtin_bit_cast(v4h, __builtin_amdgcn_ds_read_tr16_b64_v4i16(MESA_LDS3(v4s, p)));
            v4h hi = __builtin_bit_cast(v4h, __builtin_amdgcn_ds_read_tr16_b64_v4i16(MESA_LDS3(v4s, p + 4 * C::PA)));
            af[i] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        }
    };
    auto read_b = [&](const unsigned char *st, int ks, v2i braw[C::TJ]) {
#pragma unroll
        for (int j = 0; j < C::TJ; ++j)
            braw[j] = __builtin_amdgcn_ds_read_tr8_b64_v2i32(MESA_LDS3(v2i, st + b_off + ks * 16 * C::PB + j * 32));
    };
    // One contraction step on the matrix cores, in two halves.  First half: the row sums of the dy
    // fragments (every wave keeps them -- 16 dot instructions hidden under the MFMAs -- and only the
    // owners write them out) and the MFMAs of the upper fragment rows.  Second half: the remaining
    // MFMAs, with the conversion of the NEXT step's code fragments in their shadow; by then the LDS
    // reads issued before the first half have long returned, so the in-order instruction stream
    // never waits on them while the matrix core idles.
    auto mfma_half = [&](const v8h af[C::TI], const v8h bf[C::TJ], int half) {
#pragma unroll
        for (int i = half * (C::TI / 2); i < (half + 1) * (C::TI / 2); ++i)
#pragma unroll
            for (int j = 0; j < C::TJ; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bf[j], acc[i][j], 0, 0, 0);
    };
    auto row_sums = [&](const v8h af[C::TI]) {
        const h2 ones = {(_Float16)1.0f, (_Float16)1.0f};
#pragma unroll
        for (int i = 0; i < C::TI; ++i)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                h2 pr = {af[i][2 * k], af[i][2 * k + 1]};
                s0[i] = __builtin_amdgcn_fdot2(pr, ones, s0[i], false);
            }
    };
    constexpr int kHalfMfma = (C::TI / 2) * C::TJ;
    auto pace = [&](auto valu_per_mfma) {   // one MFMA, then a few VALU instructions, repeated
#pragma unroll
        for (int r = 0; r < kHalfMfma; ++r) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, decltype(valu_per_mfma)::value, 0);
        }
    };
    const std::integral_constant<int, 2> few;
    const std::integral_constant<int, 5> many;

    if (nstages > 0) {
        load_stage(m_begin, ring_a[0], ring_b[0], edge_yes);
        store_stage(smem, m_begin, ring_a[0], ring_b[0], edge_yes);
    }
#pragma unroll
    for (int d = 0; d < kDwPF; ++d)
        if (d + 1 < nstages) load_stage(m_begin + int64_t(d + 1) * kDwBM, ring_a[d], ring_b[d], edge_yes);
    __syncthreads();

    v8h af0[C::TI], af1[C::TI], bf0[C::TJ], bf1[C::TJ];
    v2i braw[C::TJ];
    if (nstages > 0) {
        read_a(smem, 0, af0);
        read_b(smem, 0, braw);
#pragma unroll
        for (int j = 0; j < C::TJ; ++j) bf0[j] = codes_to_half8(braw[j]);
    }

    // One stage.  STEADY: stage s+1+kDwPF exists and lies wholly inside the slice, so nothing here
    // is conditional.  Otherwise the same steps with their guards (the last kDwPF+1 stages).
    auto stage = [&](int s, u32x4 *ra, u32x4 *rb, auto steady) {
        constexpr bool STEADY = decltype(steady)::value;
        unsigned char *cur = smem + (s & 1) * C::STAGE;
        unsigned char *nxt = smem + ((s + 1) & 1) * C::STAGE;
        const bool more = STEADY || s + 1 < nstages;
        // step 0 of stage s on the matrix cores; step 1's fragments on their way
        read_a(cur, 1, af1);
        read_b(cur, 1, braw);
        row_sums(af0);
        mfma_half(af0, bf0, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, C::TI * 2 + C::TJ, 0);
        pace(few);
        __builtin_amdgcn_sched_barrier(0);
        mfma_half(af0, bf0, 1);
#pragma unroll
        for (int j = 0; j < C::TJ; ++j) bf1[j] = codes_to_half8(braw[j]);
        pace(many);
        __builtin_amdgcn_sched_barrier(0);
        if (STEADY) store_stage(nxt, m_begin + int64_t(s + 1) * kDwBM, ra, rb, edge_no);
        else if (more) store_stage(nxt, m_begin + int64_t(s + 1) * kDwBM, ra, rb, edge_yes);
        if (STEADY) load_stage(m_begin + int64_t(s + 1 + kDwPF) * kDwBM, ra, rb, edge_no);
        else if (s + 1 + kDwPF < nstages) load_stage(m_begin + int64_t(s + 1 + kDwPF) * kDwBM, ra, rb, edge_yes);
        __syncthreads();
        // step 1 of stage s; step 0 of stage s+1 on its way
        if (more) {
            read_a(nxt, 0, af0);
            read_b(nxt, 0, braw);
        }
        row_sums(af1);
        mfma_half(af1, bf1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, C::TI * 2 + C::TJ, 0);
        pace(few);
        __builtin_amdgcn_sched_barrier(0);
        mfma_half(af1, bf1, 1);
        if (more) {
#pragma unroll
            for (int j = 0; j < C::TJ; ++j) bf0[j] = codes_to_half8(braw[j]);
        }
        pace(many);
        __builtin_amdgcn_sched_barrier(0);
    };

    // The stage loop is unrolled by the ring length so that every ring slot is a fixed set of
    // registers: stage s+1 sits in slot s % kDwPF, goes to LDS after the first step of stage s, and
    // the slot is refilled at once with stage s+1+kDwPF.
    // steady while (s + 1 + kDwPF) * 32 + 32 <= rows of the slice
    const int full_stages = int((m_end - m_begin) / kDwBM);            // stages with all 32 rows inside
    const int steady_end = full_stages - 1 - kDwPF > 0 ? ((full_stages - 1 - kDwPF) / kDwPF) * kDwPF : 0;
    int sbase = 0;
    for (; sbase < steady_end; sbase += kDwPF) {
#pragma unroll
        for (int d = 0; d < kDwPF; ++d) stage(sbase + d, ring_a[d], ring_b[d], edge_yes /* steady */);
    }
    for (; sbase < nstages; sbase += kDwPF) {
#pragma unroll
        for (int d = 0; d < kDwPF; ++d)
            if (sbase + d < nstages) stage(sbase + d, ring_a[d], ring_b[d], edge_no /* guarded */);
    }

    // partial sums of this slice: lane l, register v of a 32x32 tile -> row 8*(v/4) + 4*(l/32) + v%4, column l%32
    float *Ps = P + int64_t(split) * N * K;
    const int col_l = lane & 31, row_l = (lane >> 5) * 4;
#pragma unroll
    for (int i = 0; i < C::TI; ++i)
#pragma unroll
        for (int j = 0; j < C::TJ; ++j) {
            const int kk = kk0 + wk * C::WK + j * 32 + col_l;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int n = n0 + wn * C::WN + i * 32 + (v >> 2) * 8 + row_l + (v & 3);
                if (n < N && kk < K) Ps[int64_t(n) * K + kk] = acc[i][j][v];
            }
        }
    if (do_s0) {
#pragma unroll
        for (int i = 0; i < C::TI; ++i) {
            float tot = s0[i] + __shfl_xor(s0[i], 32, 64);   // the two halves of the contraction slots
            const int n = n0 + wn * C::WN + i * 32 + col_l;
            if (lane < 32 && n < N) S0[int64_t(split) * N + n] = tot;
        }
    }
}

// binary32 path: 32x32x2 MFMA, operands straight from global memory (a lane needs a single value
// per operand, so no transposition is involved).  Kept simple: it serves the fp32 configuration,
// which is far too small to be a throughput case.
constexpr int kDw32BN = 128, kDw32BK = 128;

__global__ __launch_bounds__(kThreads) void k_dw_f32(const int8_t *__restrict__ xq, const float *__restrict__ dy, int64_t M,
                                                     int K, int N, int tiles_n, int tiles_k, int splits, int64_t rows_per_split,
                                                     float *__restrict__ P, float *__restrict__ S0)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int total = gridDim.x;
    const int logical = int(blockIdx.x % kDwXcd) * (total / kDwXcd) + int(blockIdx.x / kDwXcd);
    const int ntiles = tiles_n * tiles_k;
    if (logical >= ntiles * splits) return;
    const int split = logical / ntiles;
    const int t = logical - split * ntiles;
    const int tn = t / tiles_k, tk = t - tn * tiles_k;
    const int n = tn * kDw32BN + wave * 32 + (lane & 31);     // this lane's row of dW as an A operand
    const int kkb = tk * kDw32BK + (lane & 31);               // its column (plus 32*j) as a B operand
    const int64_t m_begin = int64_t(split) * rows_per_split;
    const int64_t m_end = (m_begin + rows_per_split < M) ? m_begin + rows_per_split : M;

    v16f acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.0f;
    float s0 = 0.0f;
    for (int64_t m2 = m_begin; m2 < m_end; m2 += 2) {
        const int64_t m = m2 + (lane >> 5);
        const bool mv = m < m_end;
        const float a = (mv && n < N) ? dy[m * N + n] : 0.0f;
        s0 += a;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int kk = kkb + 32 * j;
            const float b = (mv && kk < K) ? float(int(xq[m * K + kk])) : 0.0f;
            acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[j], 0, 0, 0);
        }
    }
    float *Ps = P + int64_t(split) * N * K;
    const int row_l = (lane >> 5) * 4;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int kk = kkb + 32 * j;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int nn = tn * kDw32BN + wave * 32 + (v >> 2) * 8 + row_l + (v & 3);
            if (nn < N && kk < K) Ps[int64_t(nn) * K + kk] = acc[j][v];
        }
    }
    if (tk == 0) {
        float tot = s0 + __shfl_xor(s0, 32, 64);
        if (lane < 32 && n < N) S0[int64_t(split) * N + n] = tot;
    }
}

// With q the signed code, x_hat = s_g*q + (beta_g + 128 s_g), so
// dW = s_g(k) * sum_slices P + (beta_g(k) + 128 s_g(k)) * sum_slices S0;  db = sum_slices S0.  Four columns per thread.
__global__ __launch_bounds__(kThreads) void k_dw_reduce(const float *__restrict__ P, const float *__restrict__ S0, int splits,
                                                        int N, int K, FastDiv div_k4, FastDiv div_per,
                                                        const float *__restrict__ alpha, const float *__restrict__ beta,
                                                        float *__restrict__ dW, float *__restrict__ db)
{
    const int64_t idx = int64_t(blockIdx.x) * kThreads + threadIdx.x;
    const int64_t nvec = int64_t(N) * (K / 4);
    if (idx >= nvec) return;
    const uint32_t n = fastdiv(uint32_t(idx), div_k4);
    const uint32_t kk = (uint32_t(idx) - n * div_k4.d) * 4;
    float4 s1 = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    float s0 = 0.0f;
    for (int sp = 0; sp < splits; ++sp) {
        const float4 p = *reinterpret_cast<const float4 *>(P + (int64_t(sp) * N + n) * K + kk);
        s1.x += p.x; s1.y += p.y; s1.z += p.z; s1.w += p.w;
        s0 += S0[int64_t(sp) * N + n];
    }
    float o[4] = {s1.x, s1.y, s1.z, s1.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t g = fastdiv(kk + j, div_per);
        const float sg = alpha[g] / 255.0f;
        o[j] = fmaf(sg, o[j], fmaf(128.0f, sg, beta[g]) * s0);
    }
    *reinterpret_cast<float4 *>(dW + int64_t(n) * K + kk) = make_float4(o[0], o[1], o[2], o[3]);
    if (db && kk == 0) db[n] = s0;
}

struct DwPlan {
    int variant;   // 0: 256x256 tile, 8 waves; 1: 256x128 tile, 4 waves; 2: binary32
    int bn, bk, tiles_n, tiles_k, splits, grid;
    int64_t rows_per_split;
};

static DwPlan dw_plan(int64_t M, int64_t K, int64_t N, mesa_dtype dt)
{
    DwPlan p;
    if (dt == MESA_F16) {
        p.variant = (K % 256 == 0 || K > 1024) ? 0 : 1;
        p.bn = 256;
        p.bk = p.variant == 0 ? 256 : 128;
    } else {
        p.variant = 2;
        p.bn = kDw32BN;
        p.bk = kDw32BK;
    }
    p.tiles_n = int(ceil_div(N, p.bn));
    p.tiles_k = int(ceil_div(K, p.bk));
    const int64_t tiles = int64_t(p.tiles_n) * p.tiles_k;
    // one workgroup per CU and round; slices of at least 256 contraction rows
    int64_t splits = 256 / tiles;
    if (splits < 1) splits = 1;
    int64_t max_splits = M / 256;
    if (max_splits < 1) max_splits = 1;
    if (splits > max_splits) splits = max_splits;
    if (splits > 64) splits = 64;
    int64_t rps = ceil_div(ceil_div(M > 0 ? M : 1, splits), kDwBM) * kDwBM;
    splits = ceil_div(M > 0 ? M : 1, rps);
    p.splits = int(splits);
    p.rows_per_split = rps;
    p.grid = int(ceil_div(tiles * splits, kDwXcd) * kDwXcd);
    return p;
}

size_t linear_dw_ws_bytes(int64_t M, int64_t K, int64_t N, mesa_dtype dt)
{
    if (K <= 0 || N <= 0 || M < 0) return 16;
    DwPlan p = dw_plan(M, K, N, dt);
    return size_t(p.splits) * (size_t(N) * size_t(K) + size_t(N)) * sizeof(float) + 16;
}

}  // namespace mesa

using namespace mesa;

extern "C" MESA_EXPORT mesa_status mesa_linear_dw_q(const int8_t *xq, int64_t M, int64_t K, int64_t G, const float *alpha,
                                                    const float *beta, const void *dy, int64_t N_out, mesa_dtype dt, float *dW,
                                                    float *db, void *ws, size_t ws_bytes, void *stream)
{
    if (!valid_dtype(dt) || M < 0 || K < 0 || G < 0 || N_out < 0) return MESA_ERR_INVALID_ARG;
    if (K == 0 || N_out == 0) return MESA_OK;
    if (G == 0 || K % G != 0) return MESA_ERR_INVALID_ARG;
    if (!alpha || !beta || !dW || !aligned4(alpha) || !aligned4(beta) || !aligned16(dW) || (db && !aligned4(db)))
        return MESA_ERR_INVALID_ARG;
    if (M > 0 && (!xq || !dy || !aligned16(xq) || !aligned16(dy))) return MESA_ERR_INVALID_ARG;
    if (K % 16 != 0 || N_out % 8 != 0 || K >= (int64_t(1) << 30) || N_out >= (int64_t(1) << 30) ||
        (long double)K * (long double)N_out >= 17179869184.0L /* 2^34 */)
        return MESA_ERR_UNSUPPORTED;
    if ((long double)K * (long double)N_out / 4 >= 2147483648.0L) return MESA_ERR_UNSUPPORTED;
    if (!ws || !aligned16(ws) || ws_bytes < linear_dw_ws_bytes(M, K, N_out, dt)) return MESA_ERR_WORKSPACE;
    DwPlan p = dw_plan(M, K, N_out, dt);
    hipStream_t s = static_cast<hipStream_t>(stream);
    float *P = static_cast<float *>(ws);
    float *S0 = P + size_t(p.splits) * size_t(N_out) * size_t(K);
    const int Ki = int(K), Ni = int(N_out);
    if (dt == MESA_F16) {
        const _Float16 *dyh = static_cast<const _Float16 *>(dy);
        if (p.variant == 0) {
            using C = DwCfg<256, 256, 2, 2>;
            hipLaunchKernelGGL((k_dw_f16<256, 256, 2, 2>), dim3(p.grid), dim3(C::THREADS), 2 * C::STAGE, s, xq, dyh, M, Ki, Ni,
                               p.tiles_n, p.tiles_k, p.splits, p.rows_per_split, P, S0);
        } else {
            using C = DwCfg<256, 128, 2, 2>;
            hipLaunchKernelGGL((k_dw_f16<256, 128, 2, 2>), dim3(p.grid), dim3(C::THREADS), 2 * C::STAGE, s, xq, dyh, M, Ki, Ni,
                               p.tiles_n, p.tiles_k, p.splits, p.rows_per_split, P, S0);
        }
    } else {
        hipLaunchKernelGGL(k_dw_f32, dim3(p.grid), dim3(kThreads), 0, s, xq, static_cast<const float *>(dy), M, Ki, Ni,
                           p.tiles_n, p.tiles_k, p.splits, p.rows_per_split, P, S0);
    }
    const int64_t nvec = N_out * (K / 4);
    FastDiv dk4 = make_fastdiv(uint32_t(K / 4)), dper = make_fastdiv(uint32_t(K / G));
    hipLaunchKernelGGL(k_dw_reduce, dim3(unsigned(ceil_div(nvec, kThreads))), dim3(kThreads), 0, s, P, S0, p.splits, Ni, Ki, dk4,
                       dper, alpha, beta, dW, db);
    return launch_status();
}
