// linear_dw.hip -- Linear weight gradient at the de-quantized input (Sec. 3.1 Eq. 2 for y = x W^T):
//   dW[n,k] = sum_m dy[m,n]*x_hat[m,k],  x_hat[m,k] = (q[m,k]+128)*s_g(k) + beta_g(k)   (Sec. 3.2 Eq. 5)
// evaluated in the factored form
//   dW[n,k] = s_g(k) * P[n,k] + (beta_g(k) + 128 s_g(k)) * S0[n],   P = dy^T q,  S0[n] = sum_m dy[m,n]
// so that the matrix cores contract dy with the signed 8-bit codes themselves (exact in binary16,
// and centred, so P does not cancel against S0) and the per-column affine map is applied once to
// the finished sums.
//
// (bfloat16 dy: the same kernel with bfloat16 matrix-core operands; there the contracted value is
// x_bar = q + 128 itself, c = 0 in  dW = s_g (dy^T (x_bar - c)) + (beta_g + c s_g) S0.)
//
// 16-bit path, gfx950.  Both operands are row-major in the contraction index m, which is the
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
typedef __bf16 v8b __attribute__((ext_vector_type(8)));
typedef __bf16 v2b __attribute__((ext_vector_type(2)));
typedef short v4s __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef float v16f __attribute__((ext_vector_type(16)));

#define MESA_LDS3(T, p) ((__attribute__((address_space(3))) T *)(p))

constexpr int kDwBM = 32;        // contraction rows per LDS stage
constexpr int kDwXcd = 8;
constexpr int kDwPF = 3;         // stages prefetched into registers ahead of the one being multiplied

// BN x BK tile of dW per workgroup, WGN x WGK waves, each wave (BN/WGN) x (BK/WGK) as 32x32 MFMA tiles
template <int BN, int BK, int WGN, int WGK> struct DwCfg {
    static constexpr int PF = BN * BK <= 128 * 128 ? 2 * kDwPF : kDwPF;   // small tiles: less per stage, so more stages in flight
    static constexpr int NW = WGN * WGK;
    static constexpr int THREADS = NW * 64;
    static constexpr int WN = BN / WGN, WK = BK / WGK;  // wave tile
    static constexpr int TI = WN / 32, TJ = WK / 32;    // MFMA tiles per wave
    static constexpr int TIS = TI / WGK;                // dy fragments whose row sums this wave keeps
    static constexpr int PA = BN * 2 + 64;              // LDS row pitch of the dy tile, bytes
    static constexpr int PB = BK + 32;                  // LDS row pitch of the code tile, bytes
    static constexpr int A_STAGE = kDwBM * PA;
    static constexpr int B_STAGE = kDwBM * PB;
    static constexpr int STAGE = A_STAGE + B_STAGE;
    static constexpr int A_CPR = BN / 8;                // 16-byte chunks per tile row
    static constexpr int B_CPR = BK / 16;
    static constexpr int A_TOTAL = kDwBM * A_CPR, B_TOTAL = kDwBM * B_CPR;
    static constexpr int A_CHUNKS = A_TOTAL / THREADS;  // chunks a thread moves per stage
    static constexpr int RA = THREADS / A_CPR;          // dy: rows between a thread's successive chunks (same column)
    static constexpr int TPR_B = THREADS / kDwBM;       // codes: threads per row, each taking every TPR_B-th chunk of it
    static constexpr int B_CHUNKS = B_CPR / TPR_B;
    static_assert(A_TOTAL % THREADS == 0 && THREADS % A_CPR == 0 && THREADS % kDwBM == 0 && B_CPR % TPR_B == 0,
                  "every thread moves the same number of chunks, at fixed strides");
    static_assert(TI % WGK == 0, "the row sums are shared out among the waves of a row");
    static_assert(WN % 64 == 0 && WK % 32 == 0, "wave tile: an even number of 32-row MFMA tiles by whole 32-column tiles");
    static_assert(2 * STAGE <= 64 * 1024, "two stages must fit the default dynamic LDS limit");
};

// four signed codes (the bytes of x) -> four binary16 values 1024 + x_bar: 0x6400 | (byte ^ 0x80), exactly.
// The constant rides along in the contraction (dy^T (x_bar + 1024) = dy^T x_bar + 1024 S0) and is taken out
// with the row sums afterwards: three instructions per four codes instead of five, at the price of four bits
// of the binary32 sums (the products are at most 14 times larger than with the centred code).
__device__ __forceinline__ v4s codes_to_half4(int raw)
{
    const uint32_t x = uint32_t(raw) ^ 0x80808080u;
    const v2i w = {int(__builtin_amdgcn_perm(0x64646464u, x, 0x04010400u)),    // bytes 0, 1
                   int(__builtin_amdgcn_perm(0x64646464u, x, 0x04030402u))};   // bytes 2, 3
    return __builtin_bit_cast(v4s, w);
}

// four signed codes -> four bfloat16 values q + 128 (bfloat16 has no spare mantissa bit for the exponent trick
// above, and its eight significant bits hold 0..255 exactly): byte -> binary32 -> upper halves
__device__ __forceinline__ v4s codes_to_bf4(int raw)
{
    const uint32_t x = uint32_t(raw) ^ 0x80808080u;
    const uint32_t f0 = __float_as_uint(float(x & 0xFFu)), f1 = __float_as_uint(float((x >> 8) & 0xFFu));
    const uint32_t f2 = __float_as_uint(float((x >> 16) & 0xFFu)), f3 = __float_as_uint(float(x >> 24));
    const v2i w = {int(__builtin_amdgcn_perm(f1, f0, 0x07060302u)), int(__builtin_amdgcn_perm(f3, f2, 0x07060302u))};
    return __builtin_bit_cast(v4s, w);
}

// What the operand type decides: how codes become matrix-core operands and which value of the code is
// contracted (kCentre: the offset c in "operand = x_bar - c"), the row sums of dy, and the MFMA itself.
template <typename E> struct DwElem;
template <> struct DwElem<_Float16> {
    static constexpr float kCentre = -1024.0f;
    __device__ static __forceinline__ v4s convert(int raw) { return codes_to_half4(raw); }
    __device__ static __forceinline__ float dot_ones(uint32_t pair, float acc)
    {
        const h2 ones = {(_Float16)1.0f, (_Float16)1.0f};
        return __builtin_amdgcn_fdot2(as_h2(pair), ones, acc, false);
    }
    __device__ static __forceinline__ v16f mfma(v4s a0, v4s a1, v4s b0, v4s b1, v16f c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7)),
                                                      __builtin_bit_cast(v8h, __builtin_shufflevector(b0, b1, 0, 1, 2, 3, 4, 5, 6, 7)),
                                                      c, 0, 0, 0);
    }
};
template <> struct DwElem<__bf16> {
    static constexpr float kCentre = 0.0f;
    __device__ static __forceinline__ v4s convert(int raw) { return codes_to_bf4(raw); }
    __device__ static __forceinline__ float dot_ones(uint32_t pair, float acc)
    {
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(v2b, pair), __builtin_bit_cast(v2b, 0x3F803F80u), acc, false);
    }
    __device__ static __forceinline__ v16f mfma(v4s a0, v4s a1, v4s b0, v4s b1, v16f c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8b, __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7)),
                                                       __builtin_bit_cast(v8b, __builtin_shufflevector(b0, b1, 0, 1, 2, 3, 4, 5, 6, 7)),
                                                       c, 0, 0, 0);
    }
};

// P[split][n][k] = sum over the slice's m of dy[m][n] * (x_bar[m][k] - kCentre)   (x_bar - 128 is the signed code)
// S0[split][n]   = sum over the slice's m of dy[m][n]
template <typename E, int BN, int BK, int WGN, int WGK>
__global__ __launch_bounds__(WGN * WGK * 64, 1) void k_dw_f16(const int8_t *__restrict__ xq, const E *__restrict__ dy,
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

    const int wn = wave / WGK, wk = wave % WGK;
    const int blk = lane >> 4, sl = lane & 15;
    // byte offsets of this lane's transpose-read addresses inside a stage
    const int a_off = ((blk >> 1) * 8 + (sl >> 2)) * C::PA + (wn * C::WN + (blk & 1) * 16 + (sl & 3) * 4) * 2;
    // The WGK waves that hold the same dy rows visit the wave tile's 32-row blocks in rotated order:
    // fragment i of wave wk is block a_block(i), so that "the first TIS fragments" -- a compile-time
    // set -- is a different quarter or half of the rows in each of them, and each row sum is
    // accumulated by exactly one wave.
    int a_base[WGK];
#pragma unroll
    for (int g = 0; g < WGK; ++g) a_base[g] = a_off + ((g + wk) % WGK) * C::TIS * 64;
    auto a_block = [&](int i) { return ((i / C::TIS + wk) % WGK) * C::TIS + i % C::TIS; };
    const int b_off = C::A_STAGE + ((blk >> 1) * 8 + (sl >> 1)) * C::PB + wk * C::WK + (blk & 1) * 16 + (sl & 1) * 8;

    v16f acc[C::TI][C::TJ];
#pragma unroll
    for (int i = 0; i < C::TI; ++i)
#pragma unroll
        for (int j = 0; j < C::TJ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
    float s0[C::TIS];
#pragma unroll
    for (int i = 0; i < C::TIS; ++i) s0[i] = 0.0f;
    const bool do_s0 = (tk == 0);   // the workgroups whose row sums are written out

    // global -> register prefetch ring: stage s+1 .. s+kDwPF are in flight while stage s is multiplied,
    // enough bytes per CU to cover the latency of L2 / memory-side-cache hits at the rate MFMA consumes them.
    // Of dy a thread moves the same 16-byte column chunk of rows row0, row0 + RA, row0 + 2 RA, ... of
    // every stage, so one 32-bit offset serves all its loads (the row of the item and the stage go into
    // the uniform base address) and one LDS address all its writes; of the codes it moves every
    // TPR_B-th chunk of one row (an offset per chunk, since each may be clamped).  Columns outside N or K
    // are read from column 0 instead and left as they are: row n of the product depends on column n
    // of dy only and column k on column k of the codes, and those rows and columns are never written.
    u32x4 ring_a[C::PF][C::A_CHUNKS], ring_b[C::PF][C::B_CHUNKS];
    const int row0_a = tid / C::A_CPR, col_a = n0 + (tid % C::A_CPR) * 8;
    const int row_b = tid / C::TPR_B, cb = tid % C::TPR_B;
    const uint32_t voff_a = (uint32_t(row0_a) * uint32_t(N) + uint32_t(col_a < N ? col_a : 0)) * 2u;   // bytes
    uint32_t voff_b[C::B_CHUNKS];
#pragma unroll
    for (int i = 0; i < C::B_CHUNKS; ++i) {
        const int col_b = kk0 + (cb + i * C::TPR_B) * 16;
        voff_b[i] = uint32_t(row_b) * uint32_t(K) + uint32_t(col_b < K ? col_b : 0);
    }
    const int lds_a0 = row0_a * C::PA + (tid % C::A_CPR) * 16;
    const int lds_b0 = C::A_STAGE + row_b * C::PB + cb * 16;
    const char *dy_bytes = reinterpret_cast<const char *>(dy);
    const char *xq_bytes = reinterpret_cast<const char *>(xq);
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    const int64_t len = m_end - m_begin;
    const int nfull = int(len / kDwBM);                  // stages with all their rows inside the slice
    const int64_t m_cap = M - kDwBM;                     // last row a whole stage may start at

    constexpr int kMove = C::A_CHUNKS + C::B_CHUNKS;     // 16-byte chunks a thread moves per stage
    // Whole stages are loaded without any per-lane guard.  A stage that starts beyond the tensor's
    // last whole stage (only ever a prefetch that is never used) is moved back to it: one scalar min.
    auto load_item = [&](int t, int64_t m_stage, u32x4 *ra, u32x4 *rb) {
        if (t < C::A_CHUNKS) {
            const char *base = dy_bytes + (m_stage + t * C::RA) * int64_t(N) * 2;     // uniform
            ra[t] = *reinterpret_cast<const u32x4 *>(base + voff_a);
        } else {
            const int i = t - C::A_CHUNKS;
            const char *base = xq_bytes + m_stage * int64_t(K);
            rb[i] = *reinterpret_cast<const u32x4 *>(base + voff_b[i]);
        }
    };
    auto store_item = [&](int t, unsigned char *st, const u32x4 *ra, const u32x4 *rb) {
        if (t < C::A_CHUNKS) *reinterpret_cast<u32x4 *>(st + lds_a0 + t * C::RA * C::PA) = ra[t];
        else *reinterpret_cast<u32x4 *>(st + lds_b0 + (t - C::A_CHUNKS) * C::TPR_B * 16) = rb[t - C::A_CHUNKS];
    };
    auto stage_start = [&](int s) {
        const int64_t m = m_begin + int64_t(s) * kDwBM;
        return m < m_cap ? m : m_cap;
    };

    // ---- software pipeline -------------------------------------------------------------------
    // A stage holds two contraction steps of 16 rows.  With one wave per SIMD the instruction
    // stream is issued in order, so the matrix core idles behind any burst of other instructions:
    // each step is therefore written as kNM slices -- one MFMA followed by that slice's share of
    // everything else -- fenced by scheduling barriers so that the program order is the issue order.
    // "Everything else" is, per step: the LDS reads of the next step's fragments (codes first), the
    // LDS writes of the next stage (first step) or the global loads that refill the ring slot just
    // freed (second step), this wave's share of the row sums of dy, and -- in the second half, when
    // the codes have arrived from LDS -- their conversion to binary16.  The workgroup barrier falls
    // between the two steps: after this wave's last read of the current buffer and its writes to
    // the other one.
    // Nothing in a step is conditional.  The last stages of a slice therefore also write to LDS,
    // read, convert and prefetch stages that do not exist: all of it lands in registers and LDS
    // buffers that nobody uses afterwards.
    constexpr int kNM = C::TI * C::TJ;                       // MFMAs per step
    constexpr int kNR = C::TI * 2 + C::TJ;                   // LDS reads per step
    constexpr int kND = C::TIS * 4;                          // dot instructions per step
    constexpr int kNC = C::TJ * 2;                           // conversions (four codes each) per step
    v4s afr[2][C::TI][2], bfr[2][C::TJ][2];                  // fragments of the step in flight and the next (raw 16-bit lanes)
    v2i braw[C::TJ];
    auto read_item = [&](int t, const unsigned char *st, int ks, int set) {
        if (t < C::TJ) {
            braw[t] = __builtin_amdgcn_ds_read_tr8_b64_v2i32(MESA_LDS3(v2i, st + b_off + ks * 16 * C::PB + t * 32));
        } else {
            const int i = (t - C::TJ) >> 1, h = (t - C::TJ) & 1;
            const unsigned char *p = st + a_base[i / C::TIS] + ks * 16 * C::PA + (i % C::TIS) * 64 + h * 4 * C::PA;
            afr[set][i][h] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(MESA_LDS3(v4s, p));
        }
    };
    auto dot_item = [&](int d, int set) {
        const int i = d >> 2, k = d & 3;
        s0[i] = DwElem<E>::dot_ones(uint32_t(__builtin_bit_cast(v2i, afr[set][i][k >> 1])[k & 1]), s0[i]);
    };
    auto conv_item = [&](int c, int set) { bfr[set][c >> 1][c & 1] = DwElem<E>::convert(braw[c >> 1][c & 1]); };
    auto mfma_item = [&](int r, int set) {
        const int i = r / C::TJ, j = r % C::TJ;
        acc[i][j] = DwElem<E>::mfma(afr[set][i][0], afr[set][i][1], bfr[set][j][0], bfr[set][j][1], acc[i][j]);
    };

    // One step.  PH = 0: multiplies fragment set 0 (step 0 of stage s), fetches step 1 into set 1 and
    // writes stage s+1 (ring slot ra/rb) to the other LDS buffer.  PH = 1: multiplies set 1, fetches
    // step 0 of stage s+1 into set 0 and refills the ring slot with stage s+1+kDwPF.
    auto step = [&](auto phase, int s, u32x4 *ra, u32x4 *rb) {
        constexpr int PH = decltype(phase)::value;
        const unsigned char *cur = smem + (s & 1) * C::STAGE;
        unsigned char *nxt = smem + ((s + 1) & 1) * C::STAGE;
        const int64_t m_fill = stage_start(s + 1 + C::PF);
#pragma unroll
        for (int r = 0; r < kNM; ++r) {
            mfma_item(r, PH);
            // LDS reads: the code fragments in the first TJ slices (one each), the dy fragments over the rest
            constexpr int kRA = kNR - C::TJ, kSA = kNM - C::TJ;
            if (r < C::TJ) {
                if (PH == 0) read_item(r, cur, 1, 1);
                else read_item(r, nxt, 0, 0);
            } else {
#pragma unroll
                for (int t = C::TJ + (r - C::TJ) * kRA / kSA; t < C::TJ + (r + 1 - C::TJ) * kRA / kSA; ++t) {
                    if (PH == 0) read_item(t, cur, 1, 1);
                    else read_item(t, nxt, 0, 0);
                }
            }
#pragma unroll
            for (int t = r * kMove / kNM; t < (r + 1) * kMove / kNM; ++t) {
                if (PH == 0) store_item(t, nxt, ra, rb);
                else load_item(t, m_fill, ra, rb);
            }
            // conversions: fragment j's codes were requested in slice j; its two conversions run kLat slices
            // later at the earliest, one per slice where the step is long enough, and the row sums take the
            // slices the conversions leave free
            constexpr int kLat = kNM >= 16 ? 4 : kNM / 2;
            constexpr int kSC = kNM - kLat;                  // slices that carry conversions
            if (r >= kLat) {
#pragma unroll
                for (int c = (r - kLat) * kNC / kSC; c < (r + 1 - kLat) * kNC / kSC; ++c) conv_item(c, 1 - PH);
            }
            if (kNC >= kSC) {   // conversions everywhere behind kLat: the dots go wherever they fall evenly
#pragma unroll
                for (int d = r * kND / kNM; d < (r + 1) * kND / kNM; ++d) dot_item(d, PH);
            } else {            // slices without a conversion (the first kLat, and the tail) take the dots
                constexpr int kFree = (kLat + (kSC - kNC)) > 0 ? kLat + (kSC - kNC) : 1;
                const int f = r < kLat ? r : (r >= kLat + kNC ? r - kNC : -1);
                if (f >= 0) {
#pragma unroll
                    for (int d = f * kND / kFree; d < (f + 1) * kND / kFree; ++d) dot_item(d, PH);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    const std::integral_constant<int, 0> ph0;
    const std::integral_constant<int, 1> ph1;
    auto stage = [&](int s, u32x4 *ra, u32x4 *rb) {
        step(ph0, s, ra, rb);
        __syncthreads();
        step(ph1, s, ra, rb);
    };

    if (nfull > 0) {
        // (the scheduling barriers keep the ring loads in slot order: the waits inside the loop are
        // counted from the youngest load, and the loop head must see the same order on every path)
#pragma unroll
        for (int t = 0; t < kMove; ++t) load_item(t, m_begin, ring_a[0], ring_b[0]);
#pragma unroll
        for (int t = 0; t < kMove; ++t) store_item(t, smem, ring_a[0], ring_b[0]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int d = 0; d < C::PF; ++d) {
#pragma unroll
            for (int t = 0; t < kMove; ++t) load_item(t, stage_start(d + 1), ring_a[d], ring_b[d]);
            __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();
#pragma unroll
        for (int t = 0; t < kNR; ++t) read_item(t, smem, 0, 0);
#pragma unroll
        for (int c = 0; c < kNC; ++c) conv_item(c, 0);

        // The stage loop is unrolled by the ring length so that every ring slot is a fixed set of
        // registers: stage s+1 sits in slot s % kDwPF, goes to LDS during the first step of stage s,
        // and the slot is refilled during the second step with stage s+1+kDwPF.
        // The loop body is kDwPF whole stages with no way out of its middle, and the stages left over
        // are separate copies behind it.  (Leaving the loop from the inside makes every exit a
        // predecessor of the loop's latch: the compiler then has to assume at the loop head that ANY
        // slot may hold the youngest loads, waits for the whole ring before the first slot's LDS
        // writes -- a third of all stages then run with no prefetch distance at all -- and copies
        // fragment registers at the latch.)
        int sbase = 0;
        for (; sbase + C::PF <= nfull; sbase += C::PF) {
#pragma unroll
            for (int d = 0; d < C::PF; ++d) stage(sbase + d, ring_a[d], ring_b[d]);
        }
#pragma unroll
        for (int d = 0; d < C::PF - 1; ++d) {
            if (sbase + d < nfull) stage(sbase + d, ring_a[d], ring_b[d]);
        }
    }
    // The rows left over when the slice is not a whole number of stages (only the slice that ends
    // the tensor can be): one stage outside the pipeline, with every row checked.
    if (len > int64_t(nfull) * kDwBM) {
        const int64_t m0 = m_begin + int64_t(nfull) * kDwBM;
        const int64_t m_last = m_end - 1;
        __syncthreads();   // the pipeline's last LDS reads are done
#pragma unroll
        for (int i = 0; i < C::A_CHUNKS; ++i) {
            const int64_t m = m0 + row0_a + i * C::RA;
            const char *base = dy_bytes + ((m < m_end ? m : m_last) - row0_a) * int64_t(N) * 2;
            const u32x4 v = *reinterpret_cast<const u32x4 *>(base + voff_a);
            *reinterpret_cast<u32x4 *>(smem + lds_a0 + i * C::RA * C::PA) = m < m_end ? v : zero4;
        }
#pragma unroll
        for (int i = 0; i < C::B_CHUNKS; ++i) {
            const int64_t m = m0 + row_b;
            const char *base = xq_bytes + ((m < m_end ? m : m_last) - row_b) * int64_t(K);
            const u32x4 v = *reinterpret_cast<const u32x4 *>(base + voff_b[i]);
            *reinterpret_cast<u32x4 *>(smem + lds_b0 + i * C::TPR_B * 16) = m < m_end ? v : zero4;
        }
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
            for (int t = 0; t < kNR; ++t) read_item(t, smem, ks, 0);
#pragma unroll
            for (int c = 0; c < kNC; ++c) conv_item(c, 0);
#pragma unroll
            for (int d = 0; d < kND; ++d) dot_item(d, 0);
#pragma unroll
            for (int r = 0; r < kNM; ++r) mfma_item(r, 0);
        }
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
                const int n = n0 + wn * C::WN + a_block(i) * 32 + (v >> 2) * 8 + row_l + (v & 3);
                if (n < N && kk < K) Ps[int64_t(n) * K + kk] = acc[i][j][v];
            }
        }
    if (do_s0) {
#pragma unroll
        for (int i = 0; i < C::TIS; ++i) {
            float tot = s0[i] + __shfl_xor(s0[i], 32, 64);   // the two halves of the contraction slots
            const int n = n0 + wn * C::WN + a_block(i) * 32 + col_l;
            if (lane < 32 && n < N) S0[int64_t(split) * N + n] = tot;
        }
    }
}

// The plain path: 32x32x2 binary32 MFMA, operands straight from global memory, one element at a time (a lane
// needs a single value per operand, so no transposition and no alignment is involved).  Kept simple: it serves
// binary32 tensors (the binary32 configuration is far too small to be a throughput case) and, for the 16-bit
// types, widths that the vector loads of the kernel above cannot take (K not a multiple of 16, N not of 8).
constexpr int kDw32BN = 128, kDw32BK = 128;

template <typename T>
__global__ __launch_bounds__(kThreads) void k_dw_f32(const int8_t *__restrict__ xq, const void *__restrict__ dy, int64_t M,
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
        const float a = (mv && n < N) ? Store<T>::load1(dy, m * N + n) : 0.0f;
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

// With the contracted operand u = x_bar - c, x_hat = s_g*u + (beta_g + c s_g), so
// dW = s_g(k) * sum_slices P + (beta_g(k) + c s_g(k)) * sum_slices S0;  db = sum_slices S0.  Four columns per thread.
__global__ __launch_bounds__(kThreads) void k_dw_reduce(const float *__restrict__ P, const float *__restrict__ S0, int splits,
                                                        int N, int K, FastDiv div_k4, FastDiv div_per,
                                                        const float *__restrict__ alpha, const float *__restrict__ beta,
                                                        float centre, float *__restrict__ dW, float *__restrict__ db)
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
        o[j] = fmaf(sg, o[j], fmaf(centre, sg, beta[g]) * s0);
    }
    *reinterpret_cast<float4 *>(dW + int64_t(n) * K + kk) = make_float4(o[0], o[1], o[2], o[3]);
    if (db && kk == 0) db[n] = s0;
}

// Small matrices with many slices (the narrow layers of a windowed transformer: 96 x 96 outputs, 128 slices): too few
// outputs to hide 128 dependent loads per thread behind other threads' -- eight threads share an output vector, each adds
// every eighth slice in order, and the eight partial sums are added in a fixed order.
__global__ __launch_bounds__(kThreads) void k_dw_reduce_few(const float *__restrict__ P, const float *__restrict__ S0, int splits,
                                                            int N, int K, FastDiv div_k4, FastDiv div_per,
                                                            const float *__restrict__ alpha, const float *__restrict__ beta,
                                                            float centre, float *__restrict__ dW, float *__restrict__ db)
{
    __shared__ float4 part1[8][32];
    __shared__ float part0[8][32];
    const int vl = threadIdx.x & 31, sl = threadIdx.x >> 5;
    const int64_t idx = int64_t(blockIdx.x) * 32 + vl;
    const int64_t nvec = int64_t(N) * (K / 4);
    const bool live = idx < nvec;
    const uint32_t n = live ? fastdiv(uint32_t(idx), div_k4) : 0u;
    const uint32_t kk = live ? (uint32_t(idx) - n * div_k4.d) * 4 : 0u;
    float4 s1 = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    float s0 = 0.0f;
    if (live) {
        for (int sp = sl; sp < splits; sp += 8) {
            const float4 p = *reinterpret_cast<const float4 *>(P + (int64_t(sp) * N + n) * K + kk);
            s1.x += p.x; s1.y += p.y; s1.z += p.z; s1.w += p.w;
            s0 += S0[int64_t(sp) * N + n];
        }
    }
    part1[sl][vl] = s1;
    part0[sl][vl] = s0;
    __syncthreads();
    if (sl != 0 || !live) return;
    float o[4], t0;
    {
        float4 q[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) q[i] = part1[i][vl];
        o[0] = ((q[0].x + q[1].x) + (q[2].x + q[3].x)) + ((q[4].x + q[5].x) + (q[6].x + q[7].x));
        o[1] = ((q[0].y + q[1].y) + (q[2].y + q[3].y)) + ((q[4].y + q[5].y) + (q[6].y + q[7].y));
        o[2] = ((q[0].z + q[1].z) + (q[2].z + q[3].z)) + ((q[4].z + q[5].z) + (q[6].z + q[7].z));
        o[3] = ((q[0].w + q[1].w) + (q[2].w + q[3].w)) + ((q[4].w + q[5].w) + (q[6].w + q[7].w));
        t0 = ((part0[0][vl] + part0[1][vl]) + (part0[2][vl] + part0[3][vl])) + ((part0[4][vl] + part0[5][vl]) + (part0[6][vl] + part0[7][vl]));
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t g = fastdiv(kk + j, div_per);
        const float sg = alpha[g] / 255.0f;
        o[j] = fmaf(sg, o[j], fmaf(centre, sg, beta[g]) * t0);
    }
    *reinterpret_cast<float4 *>(dW + int64_t(n) * K + kk) = make_float4(o[0], o[1], o[2], o[3]);
    if (db && kk == 0) db[n] = t0;
}

// the same for any K: one output per thread
__global__ __launch_bounds__(kThreads) void k_dw_reduce_any(const float *__restrict__ P, const float *__restrict__ S0, int splits,
                                                            int N, int K, FastDiv div_k, FastDiv div_per,
                                                            const float *__restrict__ alpha, const float *__restrict__ beta,
                                                            float centre, float *__restrict__ dW, float *__restrict__ db)
{
    const int64_t idx = int64_t(blockIdx.x) * kThreads + threadIdx.x;
    if (idx >= int64_t(N) * K) return;
    const uint32_t n = fastdiv(uint32_t(idx), div_k);
    const uint32_t kk = uint32_t(idx) - n * div_k.d;
    float s1 = 0.0f, s0 = 0.0f;
    for (int sp = 0; sp < splits; ++sp) {
        s1 += P[(int64_t(sp) * N + n) * K + kk];
        s0 += S0[int64_t(sp) * N + n];
    }
    const uint32_t g = fastdiv(kk, div_per);
    const float sg = alpha[g] / 255.0f;
    dW[idx] = fmaf(sg, s1, fmaf(centre, sg, beta[g]) * s0);
    if (db && kk == 0) db[n] = s0;
}

struct DwPlan {
    int variant;   // 16-bit tiles (n x k): 0: 256 x 256, 1: 256 x 128, 3: 128 x 128; 2: the plain path
    int bn, bk, tiles_n, tiles_k, splits, grid;
    int64_t rows_per_split;
};

static DwPlan dw_plan(int64_t M, int64_t K, int64_t N, mesa_dtype dt)
{
    DwPlan p;
    if (dt != MESA_F32 && K % 16 == 0 && N % 8 == 0) {
        // 256-wide k tiles unless they would waste much of the last one.  (A 128 x 384 tile for K = 384 was
        // measured too: no faster per MFMA, and its 21 slices instead of 14 cost more partial-sum traffic.)
        if (K % 256 == 0 || K > 1024) { p.variant = 0; p.bn = 256; p.bk = 256; }
        else if ((K <= 128 || N <= 128) && N % 256 != 0 && N % 256 <= 128) { p.variant = 3; p.bn = 128; p.bk = 128; }   // narrow K or N: no empty half tile in N
        else { p.variant = 1; p.bn = 256; p.bk = 128; }
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
    if (splits > 256) splits = 256;   // one workgroup per CU also where there is a single tile
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
    // a thread's byte offsets inside a stage of 32 rows are 32-bit (32*K and 64*N_out), the reduction indexes N_out*K/4 in 32 bits
    if (K >= (int64_t(1) << 26) || N_out >= (int64_t(1) << 25) || (long double)K * (long double)N_out >= 2147483648.0L)
        return MESA_ERR_UNSUPPORTED;
    if (!ws || !aligned16(ws) || ws_bytes < linear_dw_ws_bytes(M, K, N_out, dt)) return MESA_ERR_WORKSPACE;
    DwPlan p = dw_plan(M, K, N_out, dt);
    hipStream_t s = static_cast<hipStream_t>(stream);
    float *P = static_cast<float *>(ws);
    float *S0 = P + size_t(p.splits) * size_t(N_out) * size_t(K);
    const int Ki = int(K), Ni = int(N_out);
    float centre = 128.0f;
#define MESA_LAUNCH_DW(E, BN_, BK_) \
    do { \
        using C = DwCfg<BN_, BK_, 2, 2>; \
        hipLaunchKernelGGL((k_dw_f16<E, BN_, BK_, 2, 2>), dim3(p.grid), dim3(C::THREADS), 2 * C::STAGE, s, xq, \
                           static_cast<const E *>(dy), M, Ki, Ni, p.tiles_n, p.tiles_k, p.splits, p.rows_per_split, P, S0); \
        centre = DwElem<E>::kCentre; \
    } while (0)
    if (p.variant == 2) {   // the plain path contracts with the signed code
#define MESA_LAUNCH_DW_PLAIN(T) \
    hipLaunchKernelGGL((k_dw_f32<T>), dim3(p.grid), dim3(kThreads), 0, s, xq, dy, M, Ki, Ni, p.tiles_n, p.tiles_k, p.splits, \
                       p.rows_per_split, P, S0)
        MESA_FOR_DTYPE(dt, MESA_LAUNCH_DW_PLAIN);
#undef MESA_LAUNCH_DW_PLAIN
    } else if (dt == MESA_F16) {
        if (p.variant == 0) MESA_LAUNCH_DW(_Float16, 256, 256); else if (p.variant == 1) MESA_LAUNCH_DW(_Float16, 256, 128); else MESA_LAUNCH_DW(_Float16, 128, 128);
    } else {
        if (p.variant == 0) MESA_LAUNCH_DW(__bf16, 256, 256); else if (p.variant == 1) MESA_LAUNCH_DW(__bf16, 256, 128); else MESA_LAUNCH_DW(__bf16, 128, 128);
    }
    if (launch_status() != MESA_OK) return MESA_ERR_LAUNCH;   // the reduction must not run on partial sums nobody wrote
    FastDiv dper = make_fastdiv(uint32_t(K / G));
    if (K % 4 == 0) {
        const int64_t nvec = N_out * (K / 4);
        FastDiv dk4 = make_fastdiv(uint32_t(K / 4));
        if (nvec <= 65536 && p.splits >= 16)
            hipLaunchKernelGGL(k_dw_reduce_few, dim3(unsigned(ceil_div(nvec, 32))), dim3(kThreads), 0, s, P, S0, p.splits, Ni, Ki, dk4,
                               dper, alpha, beta, centre, dW, db);
        else
            hipLaunchKernelGGL(k_dw_reduce, dim3(unsigned(ceil_div(nvec, kThreads))), dim3(kThreads), 0, s, P, S0, p.splits, Ni, Ki, dk4,
                               dper, alpha, beta, centre, dW, db);
    } else {
        FastDiv dk = make_fastdiv(uint32_t(K));
        hipLaunchKernelGGL(k_dw_reduce_any, dim3(unsigned(ceil_div(N_out * K, kThreads))), dim3(kThreads), 0, s, P, S0, p.splits, Ni,
                           Ki, dk, dper, alpha, beta, centre, dW, db);
    }
#undef MESA_LAUNCH_DW
    return launch_status();
}
