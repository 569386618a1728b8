// attn_matmul_bwd.hip -- backward of the two matrix products of self-attention at head-wise
// de-quantized operands (Sec. 3.1 Eq. 2 with G_l the gradient of a matrix product; Sec. 3.2: the
// operands of the products are saved as 8-bit codes with one (alpha, beta) pair per head):
//   O = A V           dA[i,j] = sum_d dO[i,d]*V_hat[j,d]           dV[j,d] = sum_i A_hat[i,j]*dO[i,d]
//   S = scale Q K^T   dQ[i,d] = scale*sum_j dS[i,j]*K_hat[j,d]     dK[j,d] = scale*sum_i dS[i,j]*Q_hat[i,d]
//
// All four are one batched product  C[r,c] = sum_t P(r,t)*Q(t,c)  per (sample, head), where P and Q are
// strided views of the tensors and exactly one of them is coded.  As in the weight gradient, the matrix
// cores contract with the signed codes themselves (exact in binary16) and the head's affine map is
// applied to the finished sums:  x_hat = s*(q+128) + beta  gives
//   C = s * sum_t P*q  +  (beta + 128 s) * sum_t P        (Q coded; symmetric when P is),
// the plain sums coming from one more MFMA against a fragment of ones.
//
// The sequence length of a vision transformer is odd (197), so rows of the attention-shaped tensors
// start at odd offsets and nothing here can be loaded in ALIGNED vectors: operand tiles of 64 x 32 are
// staged into LDS with element-aligned 8-element loads along each operand's unit-stride index (whole
// vectors inside the extents, single elements and zero fill at the edges, so any extents work) and
// kept in the operand's own orientation; where that is not the orientation the MFMA wants, the
// fragments come from the LDS transpose reads.  The next stage's loads are in flight while a stage
// is multiplied.  binary16 or bfloat16 tensors (every kernel here takes the number type as a parameter);
// binary32 tensors through one plain kernel (k_bmm_q_f32).
//
// That general kernel (k_bmm_q) serves every shape; dedicated kernels take the shapes that matter: k_attn_da,
// k_attn_tn, k_attn_nn for sequences one workgroup per head (or per 32 rows) can hold, odd lengths included, and
// k_attn_da_cols, k_attn_tn_cols, k_attn_nn_rows for sequences of any length whose rows are aligned (N a multiple of 8
// or 16): long ones, and short ones too -- a pitch of N elements with N a multiple of 32 puts the first three kernels'
// lanes on the same LDS banks.
#include <hip/hip_runtime.h>
#include <type_traits>

#include "api_util.hpp"
#include "common.hpp"

namespace mesa {

typedef _Float16 bm_v8h __attribute__((ext_vector_type(8)));
typedef _Float16 bm_v2h __attribute__((ext_vector_type(2)));
typedef _Float16 bm_v4h __attribute__((ext_vector_type(4)));
typedef short bm_v4s __attribute__((ext_vector_type(4)));
typedef int bm_v2i __attribute__((ext_vector_type(2)));
typedef float bm_v16f __attribute__((ext_vector_type(16)));
typedef float bm_v4f __attribute__((ext_vector_type(4)));
typedef unsigned bm_v4u __attribute__((ext_vector_type(4)));

#define BM_LDS3(T, p) ((__attribute__((address_space(3))) T *)(p))

constexpr int kBmTile = 64;     // output tile of a workgroup (rows and columns)
constexpr int kBmT = 32;        // contraction extent per stage
constexpr int kBmParts = kBmT / 32;   // 8-element vectors per thread, operand and stage

// eight signed codes (bytes) -> eight binary16 values q: 0x6400 | (byte ^ 0x80) is 1152 + q exactly
__device__ __forceinline__ bm_v8h bm_codes_to_half8(bm_v2i raw)
{
    bm_v8h out;
    const h2 k1152 = {(_Float16)1152.0f, (_Float16)1152.0f};
#pragma unroll
    for (int w = 0; w < 2; ++w) {
        const uint32_t x = uint32_t(raw[w]) ^ 0x80808080u;
        const h2 lo = as_h2(__builtin_amdgcn_perm(0x64646464u, x, 0x04010400u)) - k1152;   // bytes 0, 1
        const h2 hi = as_h2(__builtin_amdgcn_perm(0x64646464u, x, 0x04030402u)) - k1152;   // bytes 2, 3
        out[4 * w + 0] = lo.x; out[4 * w + 1] = lo.y; out[4 * w + 2] = hi.x; out[4 * w + 3] = hi.y;
    }
    return out;
}

// What the 16-bit number type decides in the general kernel: how codes become matrix-core operands and which
// value of the code is contracted (kCentre: c in "operand = x_bar - c"; bfloat16 has no spare mantissa bit for
// the exponent trick and takes x_bar = q + 128 itself, byte -> binary32 -> upper half), the fragment of ones,
// the MFMA and the rounding of a result.  Operands travel as raw 16-bit lanes (bm_v8h as a container).
typedef __bf16 bm_v8b __attribute__((ext_vector_type(8)));
template <typename ET> struct BmNum;
template <> struct BmNum<_Float16> {
    static constexpr float kCentre = 128.0f;
    static constexpr uint16_t kOne = 0x3C00u;
    __device__ static __forceinline__ bm_v8h codes8(bm_v2i raw) { return bm_codes_to_half8(raw); }
    __device__ static __forceinline__ bm_v16f mfma(bm_v8h a, bm_v8h b, bm_v16f c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
    __device__ static __forceinline__ _Float16 round(float v) { return (_Float16)v; }
    // eight codes gathered two to a register (bits 0-7 and 16-23): 0x6400 | (byte ^ 0x80) is 1024 + x_bar, minus 1152
    __device__ static __forceinline__ bm_v8h gathered(bm_v4u u)
    {
#pragma unroll
        for (int k = 0; k < 4; ++k) u[k] = (u[k] ^ 0x00800080u) | 0x64006400u;
        bm_v8h f = __builtin_bit_cast(bm_v8h, u);
#pragma unroll
        for (int k = 0; k < 8; ++k) f[k] = f[k] - (_Float16)1152.0f;
        return f;
    }
    // acc + the two values of a register pair
    __device__ static __forceinline__ float dot_ones(_Float16 a, _Float16 b, float acc)
    {
        return __builtin_amdgcn_fdot2(bm_v2h{a, b}, bm_v2h{(_Float16)1.0f, (_Float16)1.0f}, acc, false);
    }
};
template <> struct BmNum<__bf16> {
    static constexpr float kCentre = 0.0f;
    static constexpr uint16_t kOne = 0x3F80u;
    __device__ static __forceinline__ bm_v8h codes8(bm_v2i raw)
    {
        bm_v4u out;
#pragma unroll
        for (int w = 0; w < 2; ++w) {
            const uint32_t x = uint32_t(raw[w]) ^ 0x80808080u;
            const uint32_t f0 = __float_as_uint(float(x & 0xFFu)), f1 = __float_as_uint(float((x >> 8) & 0xFFu));
            const uint32_t f2 = __float_as_uint(float((x >> 16) & 0xFFu)), f3 = __float_as_uint(float(x >> 24));
            out[2 * w] = __builtin_amdgcn_perm(f1, f0, 0x07060302u);
            out[2 * w + 1] = __builtin_amdgcn_perm(f3, f2, 0x07060302u);
        }
        return __builtin_bit_cast(bm_v8h, out);
    }
    __device__ static __forceinline__ bm_v16f mfma(bm_v8h a, bm_v8h b, bm_v16f c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bm_v8b, a), __builtin_bit_cast(bm_v8b, b), c, 0, 0, 0);
    }
    __device__ static __forceinline__ _Float16 round(float v)   // the bits of the bfloat16, in the 16-bit container
    {
        return __builtin_bit_cast(_Float16, __bf16(v));
    }
    __device__ static __forceinline__ bm_v8h gathered(bm_v4u u)
    {
        bm_v4u out;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t x = u[k] ^ 0x00800080u;
            out[k] = __builtin_amdgcn_perm(__float_as_uint(float((x >> 16) & 0xFFu)), __float_as_uint(float(x & 0xFFu)), 0x07060302u);
        }
        return __builtin_bit_cast(bm_v8h, out);
    }
    __device__ static __forceinline__ float dot_ones(_Float16 a, _Float16 b, float acc)
    {
        typedef __bf16 v2b __attribute__((ext_vector_type(2)));
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(v2b, bm_v2h{a, b}), __builtin_bit_cast(v2b, 0x3F803F80u), acc, false);
    }
};

struct BmmArgs {
    const _Float16 *x;          // the plain operand (16-bit container: binary16 or bfloat16 bits)
    const int8_t *y;            // the coded operand
    _Float16 *c;                // output, row-major R x Cn per batch
    int64_t x_batch, y_batch, c_batch;   // elements per (sample, head)
    int R, Cn, Tn;              // output rows, output columns, contraction extent
    int64_t p_rs, p_ts;         // element strides of the view P(r, t)
    int64_t q_ts, q_cs;         // element strides of the view Q(t, c)
    int tiles_r, tiles_c;
    int64_t batch0;             // first (sample, head) of this launch
    int head0;                  // and its head: batch0 % heads
    int heads;
    float scale;
    const float *alpha, *beta;  // of the coded operand, per head
};

// ---- staging: global -> registers -> LDS ---------------------------------------------------------
// A 64 x kBmT operand tile per stage is kBmParts * 256 vectors of eight elements along the operand's
// unit-stride index (vector idx = tid + 256 * part), each loaded with one element-aligned 16-byte
// (binary16) or 8-byte (codes) load and stored to LDS as it is, in the operand's own orientation:
//   TFAST  (unit stride along the contraction index t):  idx -> (line = idx / (kBmT/8), t = 8 * (idx % (kBmT/8)) ..+7),
//          LDS rows are lines ([line][t]) and an MFMA fragment is a plain 16- or 8-byte read;
//   !TFAST (unit stride along the row / column index):   idx -> (t = idx/8, lines 8*(idx%8) ..+7),
//          LDS rows are contraction steps ([t][line]) and the fragment comes from gfx950's transposing
//          LDS reads (ds_read_b64_tr_b16 / _b8: within 16 lanes, the lanes 4k..4k+3 -- 2k, 2k+1 for bytes --
//          supply row k, and lane i receives column i).
// `line` is the row of P or the column of Q.  Codes stay bytes in LDS and become binary16 (the signed
// code itself, exact) in the fragment.  Row pitches are padded so that neither access conflicts.
template <bool CODED> struct BmRaw;
template <> struct BmRaw<false> { u32x4 w; };   // eight binary16
template <> struct BmRaw<true> { u32x2 w; };    // eight codes

template <bool CODED> struct BmElem;
template <> struct BmElem<false> {
    typedef _Float16 type;
    static constexpr int kBytes = 2;
};
template <> struct BmElem<true> {
    typedef int8_t type;
    static constexpr int kBytes = 1;
};

// Edges.  Rows of P / columns of Q beyond the extents produce output rows / columns that are never
// written, so they may hold any finite data; contraction steps t >= Tn must contribute nothing, so both
// operands hold zeros there (never stale LDS contents: 0 x NaN would poison a sum).  Every load is an
// unconditional whole-vector load from coordinates clamped into the tensor (no branch, no merge with
// other values: nothing waits on a load before its stage is due); a vector that was moved back to stay
// inside the extent is written to LDS at the position it really came from (element by element: the
// slots overlap the neighbouring vector's, with the same values), and zeros are written where required.
template <bool CODED, bool TFAST> struct BmOperand {
    typedef typename BmElem<CODED>::type E;
    static constexpr int kEb = BmElem<CODED>::kBytes;
    // bytes per LDS row: [line][t]: kBmT elements + 8 of padding; [t][line]: 64 elements + 32 of padding
    static constexpr int kPitch = TFAST ? (kBmT + 8) * kEb : (kBmTile + 32) * kEb;
    static constexpr int kBytes = TFAST ? kBmTile * kPitch : kBmT * kPitch;
    typedef decltype(BmRaw<CODED>::w) W;

    // tile-relative coordinates of vector idx: (line, t) of its first element
    __device__ static __forceinline__ void coord(int idx, int &line, int &t)
    {
        if (TFAST) { line = idx / (kBmT / 8); t = (idx % (kBmT / 8)) * 8; }
        else { t = idx / 8; line = (idx % 8) * 8; }
    }
    // lines >= 8 and tn >= 8 (checked by the entry points)
    __device__ static __forceinline__ BmRaw<CODED> load(const E *base, int64_t line_stride, int64_t t_stride, int line0, int t0,
                                                        int lines, int tn, int idx)
    {
        int line, t;
        coord(idx, line, t);
        line += line0;
        t += t0;
        BmRaw<CODED> v;
        if (TFAST) {
            line = line < lines ? line : lines - 1;
            t = t + 8 <= tn ? t : tn - 8;
            __builtin_memcpy(&v.w, base + int64_t(line) * line_stride + t, 8 * kEb);       // t_stride == 1
        } else {
            t = t < tn ? t : tn - 1;
            line = line + 8 <= lines ? line : lines - 8;
            __builtin_memcpy(&v.w, base + int64_t(t) * t_stride + line, 8 * kEb);          // line_stride == 1
        }
        return v;
    }
    __device__ static __forceinline__ void store(unsigned char *lds, const BmRaw<CODED> &v, int line0, int t0, int lines, int tn,
                                                 int idx)
    {
        int line, t;
        coord(idx, line, t);
        if (line0 + kBmTile <= lines && t0 + kBmT <= tn) {   // uniform: the whole tile lies inside the extents
            *reinterpret_cast<W *>(lds + (TFAST ? line * kPitch + t * kEb : t * kPitch + line * kEb)) = v.w;
            return;
        }
        E e[8];
        __builtin_memcpy(e, &v.w, 8 * kEb);
        W zero;
#pragma unroll
        for (int k = 0; k < int(sizeof(W) / 4); ++k) zero[k] = 0u;
        if (TFAST) {
            unsigned char *row = lds + line * kPitch;
            const int tg = t0 + t;                                   // global contraction index of slot t
            if (tg + 8 <= tn) {
                *reinterpret_cast<W *>(row + t * kEb) = v.w;
            } else if (tg < tn) {                                    // the vector was moved back to tn - 8
                const int tc = tn - 8 - t0;                          // tile-relative slot of its first element (>= -7)
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if (tc + i >= t) reinterpret_cast<E *>(row)[tc + i] = e[i];
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (tg + j >= tn) reinterpret_cast<E *>(row)[t + j] = E(0);
            } else {
                *reinterpret_cast<W *>(row + t * kEb) = zero;
            }
        } else {
            unsigned char *row = lds + t * kPitch;
            const bool t_ok = t0 + t < tn;
            const int lg = line0 + line;
            if (lg + 8 <= lines || lg >= lines) {                    // whole vector inside, or wholly outside (anything will do)
                *reinterpret_cast<W *>(row + line * kEb) = t_ok ? v.w : zero;
            } else {                                                 // moved back to lines - 8
                const int lc = lines - 8 - line0;
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if (lc + i >= line) reinterpret_cast<E *>(row)[lc + i] = t_ok ? e[i] : E(0);
            }
        }
    }
    // the MFMA operand of a wave's 32 lines starting at l0, contraction slots 16*ks ..+15: lane l holds line
    // l%32 and the eight slots 8*(l/32) ..+7
    template <typename ET> __device__ static __forceinline__ bm_v8h frag(const unsigned char *lds, int l0, int ks, int lane)
    {
        if (TFAST) {
            const unsigned char *p = lds + (l0 + (lane & 31)) * kPitch + (ks * 16 + (lane >> 5) * 8) * kEb;
            if (CODED) return BmNum<ET>::codes8(*reinterpret_cast<const bm_v2i *>(p));
            return *reinterpret_cast<const bm_v8h *>(p);
        }
        const int blk = lane >> 4, sl = lane & 15;
        if (CODED) {
            const unsigned char *p = lds + (ks * 16 + (blk >> 1) * 8 + (sl >> 1)) * kPitch + l0 + (blk & 1) * 16 + (sl & 1) * 8;
            return BmNum<ET>::codes8(__builtin_amdgcn_ds_read_tr8_b64_v2i32(BM_LDS3(bm_v2i, p)));
        }
        const unsigned char *p = lds + (ks * 16 + (blk >> 1) * 8 + (sl >> 2)) * kPitch + (l0 + (blk & 1) * 16 + (sl & 3) * 4) * 2;
        const bm_v4h lo = __builtin_bit_cast(bm_v4h, __builtin_amdgcn_ds_read_tr16_b64_v4i16(BM_LDS3(bm_v4s, p)));
        const bm_v4h hi = __builtin_bit_cast(bm_v4h, __builtin_amdgcn_ds_read_tr16_b64_v4i16(BM_LDS3(bm_v4s, p + 4 * kPitch)));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
};

// P_CODED: P is the coded operand (else Q).  P_TFAST / Q_TFAST: the contraction index is the unit-stride
// index of that operand in memory.  ET: _Float16 or __bf16 (the tensors' 16-bit type; BmmArgs carries them as
// 16-bit containers).
template <bool P_CODED, bool P_TFAST, bool Q_TFAST, typename ET>
__global__ __launch_bounds__(kThreads, 6) void k_bmm_q(BmmArgs a)
{
    typedef BmOperand<P_CODED, P_TFAST> OP;
    typedef BmOperand<!P_CODED, Q_TFAST> OQ;
    __shared__ __attribute__((aligned(16))) unsigned char LP[OP::kBytes];
    __shared__ __attribute__((aligned(16))) unsigned char LQ[OQ::kBytes];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // grid: x = column tile, y = row tile, z = (sample, head) in pieces of at most 65535 (32-bit, uniform arithmetic only)
    const uint32_t b = blockIdx.z;
    const int r0 = int(blockIdx.y) * kBmTile, c0 = int(blockIdx.x) * kBmTile;
    const uint32_t h = (b + uint32_t(a.head0)) % uint32_t(a.heads);

    const _Float16 *xb = a.x + int64_t(b) * a.x_batch + a.batch0 * a.x_batch;
    const int8_t *yb = a.y + int64_t(b) * a.y_batch + a.batch0 * a.y_batch;
    auto load_p = [&](int t0, int part) {
        if constexpr (P_CODED) return OP::load(yb, a.p_rs, a.p_ts, r0, t0, a.R, a.Tn, tid + part * kThreads);
        else return OP::load(xb, a.p_rs, a.p_ts, r0, t0, a.R, a.Tn, tid + part * kThreads);
    };
    auto load_q = [&](int t0, int part) {
        if constexpr (P_CODED) return OQ::load(xb, a.q_cs, a.q_ts, c0, t0, a.Cn, a.Tn, tid + part * kThreads);
        else return OQ::load(yb, a.q_cs, a.q_ts, c0, t0, a.Cn, a.Tn, tid + part * kThreads);
    };

    const int wr = wave >> 1, wc = wave & 1;            // 2 x 2 waves, a 32 x 32 MFMA tile each
    bm_v16f acc, acc1;
#pragma unroll
    for (int v = 0; v < 16; ++v) { acc[v] = 0.0f; acc1[v] = 0.0f; }
    bm_v8h ones;
#pragma unroll
    for (int j = 0; j < 8; ++j) ones[j] = __builtin_bit_cast(_Float16, BmNum<ET>::kOne);

    BmRaw<P_CODED> pv[kBmParts];
    BmRaw<!P_CODED> qv[kBmParts];
#pragma unroll
    for (int k = 0; k < kBmParts; ++k) { pv[k] = load_p(0, k); qv[k] = load_q(0, k); }
    for (int t0 = 0; t0 < a.Tn; t0 += kBmT) {
        __syncthreads();   // the previous stage's fragments have been read
#pragma unroll
        for (int k = 0; k < kBmParts; ++k) {
            OP::store(LP, pv[k], r0, t0, a.R, a.Tn, tid + k * kThreads);
            OQ::store(LQ, qv[k], c0, t0, a.Cn, a.Tn, tid + k * kThreads);
        }
        __syncthreads();
        if (t0 + kBmT < a.Tn) {   // the next stage's loads fly while this one is multiplied
#pragma unroll
            for (int k = 0; k < kBmParts; ++k) { pv[k] = load_p(t0 + kBmT, k); qv[k] = load_q(t0 + kBmT, k); }
        }
#pragma unroll
        for (int ks = 0; ks < kBmT / 16; ++ks) {
            const bm_v8h fa = OP::template frag<ET>(LP, wr * 32, ks, lane);
            const bm_v8h fb = OQ::template frag<ET>(LQ, wc * 32, ks, lane);
            acc = BmNum<ET>::mfma(fa, fb, acc);
            acc1 = BmNum<ET>::mfma(P_CODED ? ones : fa, P_CODED ? fb : ones, acc1);
        }
    }

    // lane l, register v of a 32 x 32 tile: row 8*(v/4) + 4*(l/32) + v%4, column l%32
    const float s = a.alpha[h] / 255.0f;
    const float off = fmaf(BmNum<ET>::kCentre, s, a.beta[h]);
    const int col = c0 + wc * 32 + (lane & 31);
    const int row_l = r0 + wr * 32 + (lane >> 5) * 4;
    // R * Cn < 2^31 (checked by the entry points): 32-bit offsets from the batch's base
    _Float16 *cb = a.c + (int64_t(b) + a.batch0) * a.c_batch;
    const uint32_t o0 = uint32_t(row_l) * uint32_t(a.Cn) + uint32_t(col);
    if (col < a.Cn) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int dr = (v >> 2) * 8 + (v & 3);
            if (row_l + dr < a.R) cb[o0 + uint32_t(dr) * uint32_t(a.Cn)] = BmNum<ET>::round(a.scale * fmaf(s, acc[v], off * acc1[v]));
        }
    }
}

template <bool P_CODED, bool P_TFAST, bool Q_TFAST, typename ET = _Float16>
static void launch_bmm(BmmArgs a, int64_t batches, hipStream_t s)
{
    a.tiles_r = int(ceil_div(a.R, kBmTile));
    a.tiles_c = int(ceil_div(a.Cn, kBmTile));
    // the z extent of a grid is limited to 65535: more (sample, head) pairs than that go in several launches
    for (int64_t b0 = 0; b0 < batches; b0 += 65535) {
        a.batch0 = b0;
        a.head0 = int(b0 % a.heads);
        const int64_t nb = batches - b0 < 65535 ? batches - b0 : 65535;
        hipLaunchKernelGGL((k_bmm_q<P_CODED, P_TFAST, Q_TFAST, ET>), dim3(unsigned(a.tiles_c), unsigned(a.tiles_r), unsigned(nb)),
                           dim3(kThreads), 0, s, a);
    }
}

// The plain kernel: 32x32x2 binary32 MFMA with operands straight from global memory, one element at a time (a lane
// needs one value per operand and step: lane l holds row / column l%32 at contraction slot l/32).  Kept simple: it
// serves binary32 tensors (the binary32 configuration is far too small to be a throughput case) and, for the 16-bit
// types, extents shorter than one load vector.  T: the tensors' element type (BmmArgs' pointers are reinterpreted).
template <bool P_CODED, typename T>
__global__ __launch_bounds__(kThreads) void k_bmm_q_f32(BmmArgs a)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t b = blockIdx.z;
    const int r = int(blockIdx.y) * kBmTile + (wave >> 1) * 32 + (lane & 31);
    const int c = int(blockIdx.x) * kBmTile + (wave & 1) * 32 + (lane & 31);
    const uint32_t h = (b + uint32_t(a.head0)) % uint32_t(a.heads);
    const int64_t xb0 = (int64_t(b) + a.batch0) * a.x_batch;
    const int8_t *yb = a.y + (int64_t(b) + a.batch0) * a.y_batch;
    const bool r_ok = r < a.R, c_ok = c < a.Cn;
    bm_v16f acc, acc1;
#pragma unroll
    for (int v = 0; v < 16; ++v) { acc[v] = 0.0f; acc1[v] = 0.0f; }
    for (int t0 = 0; t0 < a.Tn; t0 += 2) {
        const int t = t0 + (lane >> 5);
        const bool t_ok = t < a.Tn;
        float pa = 0.0f, qb = 0.0f;
        const int64_t po = int64_t(r) * a.p_rs + int64_t(t) * a.p_ts, qo = int64_t(t) * a.q_ts + int64_t(c) * a.q_cs;
        if (t_ok && r_ok) pa = P_CODED ? float(int(yb[po])) : Store<T>::load1(a.x, xb0 + po);
        if (t_ok && c_ok) qb = P_CODED ? Store<T>::load1(a.x, xb0 + qo) : float(int(yb[qo]));
        const float one = t_ok ? 1.0f : 0.0f;
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(pa, qb, acc, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(P_CODED ? one : pa, P_CODED ? qb : one, acc1, 0, 0, 0);   // sums of the plain operand
    }
    const float s = a.alpha[h] / 255.0f;
    const float off = fmaf(128.0f, s, a.beta[h]);
    const int row_l = int(blockIdx.y) * kBmTile + (wave >> 1) * 32 + (lane >> 5) * 4;
    const int64_t cb0 = (int64_t(b) + a.batch0) * a.c_batch;
    if (c_ok) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int rr = row_l + (v >> 2) * 8 + (v & 3);
            if (rr < a.R) Store<T>::store1(a.c, cb0 + int64_t(rr) * a.Cn + c, a.scale * fmaf(s, acc[v], off * acc1[v]));
        }
    }
}

template <bool P_CODED> static void launch_bmm_f32(BmmArgs a, int64_t batches, mesa_dtype dt, hipStream_t s)
{
    a.tiles_r = int(ceil_div(a.R, kBmTile));
    a.tiles_c = int(ceil_div(a.Cn, kBmTile));
    for (int64_t b0 = 0; b0 < batches; b0 += 65535) {
        a.batch0 = b0;
        a.head0 = int(b0 % a.heads);
        const int64_t nb = batches - b0 < 65535 ? batches - b0 : 65535;
#define MESA_LAUNCH_PLAIN(T) \
    hipLaunchKernelGGL((k_bmm_q_f32<P_CODED, T>), dim3(unsigned(a.tiles_c), unsigned(a.tiles_r), unsigned(nb)), dim3(kThreads), 0, s, a)
        MESA_FOR_DTYPE(dt, MESA_LAUNCH_PLAIN);
#undef MESA_LAUNCH_PLAIN
    }
}

// ---- the two products whose contraction index is the unit-stride index of BOTH operands' rows --------
// They need no transposition and (almost) no LDS: an MFMA operand fragment -- lane l: line l%32, the eight
// contraction slots 8*(l/32) ..+7 of a 16-slot step -- is one vector load straight from global memory.

// dA[i,j] = sum_d dO[i,d] * V_hat[j,d].  A workgroup takes 32 rows i of one head; its waves share out the
// blocks of 32 columns j.  Both operands' blocks are contiguous in memory (32 rows of dO, 32 rows of V
// codes): they come in as consecutive aligned 16-byte vectors -- a lane per row would cost the memory
// pipeline one access per lane -- and pass through LDS (dO once per workgroup, the codes privately per
// wave) into the fragments.  The MFMA runs with the operands exchanged (codes as the M side, dO as the N
// side), so that a lane ends up with ONE row i = l%32 and runs of four consecutive columns: the beta term's
// row sum of dO is then a per-lane scalar, and the tile goes to LDS with 8-byte writes.  The 32 x N output
// block is one contiguous piece of memory whose start is only element-aligned (N is odd for ViT): LDS holds
// it at the same offset from a 16-byte boundary, and it leaves as aligned 16-byte vectors; the few elements
// before the first and after the last whole vector are written one by one (the neighbouring blocks own the
// rest of those vectors).  Dh == 16 * KS, KS even.
// LDS: [output block, 64 N + 32 bytes | staged dO, 32 rows]  (the same space, one after the other in time),
// then 32 code rows per wave at `codes_at`.
// SOLO (short rows, N <= 64): a wave takes an item (head, block of 32 rows) all by itself, with its own
// piece of LDS and no barrier, so that no wave of the workgroup idles for want of column blocks.
template <int KS> struct DaCfg {
    static constexpr int Dh = 16 * KS;
    static constexpr int kRowO = 2 * Dh + 16;   // bytes per staged dO row (padded against bank conflicts)
    static constexpr int kRowV = Dh + 16;       // bytes per staged code row
    static constexpr int kVecO = Dh / 8;        // 16-byte vectors per dO row
    static constexpr int kVecV = Dh / 16;       // and per code row
    static constexpr int kCodeVecs = 32 * kVecV / 64;   // vectors per lane for a block of 32 code rows
    static constexpr int kWaves = kThreads / 64;
    // offset of the staged codes: behind the output block / the staged dO rows, whichever is longer
    static size_t codes_at(int64_t N)
    {
        const size_t out = size_t(N) * 64 + 32, stage = size_t(32) * kRowO;
        return ((out > stage ? out : stage) + 15) & ~size_t(15);
    }
    static size_t wave_bytes(int64_t N) { return codes_at(N) + size_t(32) * kRowV; }           // SOLO: per wave
    static size_t lds_bytes(int64_t N, bool solo) { return solo ? kWaves * wave_bytes(N) : codes_at(N) + size_t(kWaves) * 32 * kRowV; }
};

template <int KS, bool SOLO, typename ET>
__global__ __launch_bounds__(kThreads, KS <= 4 ? 7 : 4) void k_attn_da(const _Float16 *__restrict__ dO,
                                                                      const int8_t *__restrict__ vq, _Float16 *__restrict__ dA,
                                                                      int N, int heads, const float *__restrict__ alpha_v,
                                                                      const float *__restrict__ beta_v, int64_t batch0, int codes_at,
                                                                      unsigned items)
{
    typedef DaCfg<KS> C;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_all[];
    constexpr int Dh = C::Dh;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int fl = lane & 31, fk = (lane >> 5) * 8;
    const int nblocks = (N + 31) >> 5;
    // the threads that share an item, this thread's rank among them, and the column blocks this wave takes
    constexpr int kTeam = SOLO ? 64 : kThreads;
    const int t = SOLO ? lane : int(threadIdx.x);
    const int cb_first = SOLO ? 0 : wave, cb_step = SOLO ? 1 : C::kWaves;
    int64_t bh;
    int r0;
    if (SOLO) {                                            // items (at most 2^32) count (head, row block) pairs
        const unsigned item = blockIdx.x * C::kWaves + wave;
        if (item >= items) return;                         // no barrier in this mode
        const unsigned q = item / unsigned(nblocks);
        bh = q;
        r0 = int(item - q * unsigned(nblocks)) * 32;
    } else {
        bh = batch0 + blockIdx.y;
        r0 = int(blockIdx.x) * 32;
    }
    auto team_sync = [&]() {
        if constexpr (!SOLO) __syncthreads();
    };
    unsigned char *lds_da = SOLO ? lds_all + wave * (codes_at + 32 * C::kRowV) : lds_all;
    unsigned char *lv = SOLO ? lds_da + codes_at : lds_all + codes_at + wave * (32 * C::kRowV);
    constexpr int kOVecs = (32 * C::kVecO + kTeam - 1) / kTeam;   // dO vectors per thread
    const int code_vecs = N * C::kVecV;                    // of one head
    const int rows = N - r0 < 32 ? N - r0 : 32;
    const u32x4 *vvec = reinterpret_cast<const u32x4 *>(vq + bh * N * int64_t(Dh));
    auto load_codes = [&](int c0, u32x4 (&raw)[C::kCodeVecs]) {
#pragma unroll
        for (int i = 0; i < C::kCodeVecs; ++i) {
            const int g = c0 * C::kVecV + lane + 64 * i;   // rows past the head's end repeat its last vector; never used
            raw[i] = vvec[g < code_vecs ? g : code_vecs - 1];
        }
    };
    auto store_codes = [&](const u32x4 (&raw)[C::kCodeVecs]) {
#pragma unroll
        for (int i = 0; i < C::kCodeVecs; ++i) {
            const int idx = lane + 64 * i;
            *reinterpret_cast<u32x4 *>(lv + (idx / C::kVecV) * C::kRowV + (idx % C::kVecV) * 16) = raw[i];
        }
    };
    u32x4 raw[C::kCodeVecs];
    if (cb_first < nblocks) load_codes(cb_first * 32, raw);
    {
        const int o_vecs = rows * C::kVecO;
        const u32x4 *ovec = reinterpret_cast<const u32x4 *>(dO + (bh * N + r0) * int64_t(Dh));
        u32x4 ov[kOVecs];
#pragma unroll
        for (int k = 0; k < kOVecs; ++k) {                 // rows past the last one repeat its last vector
            const int idx = t + k * kTeam;
            ov[k] = ovec[idx < o_vecs ? idx : o_vecs - 1];
        }
#pragma unroll
        for (int k = 0; k < kOVecs; ++k) {
            const int idx = t + k * kTeam;
            if (idx < 32 * C::kVecO) *reinterpret_cast<u32x4 *>(lds_da + (idx / C::kVecO) * C::kRowO + (idx % C::kVecO) * 16) = ov[k];
        }
    }
    team_sync();
    bm_v8h fo[KS];
    float rsum = 0.0f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        fo[ks] = *reinterpret_cast<const bm_v8h *>(lds_da + fl * C::kRowO + (ks * 16 + fk) * 2);
#pragma unroll
        for (int j = 0; j < 8; j += 2)
            rsum = BmNum<ET>::dot_ones(fo[ks][j], fo[ks][j + 1], rsum);
    }
    rsum += __shfl_xor(rsum, 32);                          // both halves of the row's slots
    team_sync();                                           // every wave holds its fragments: the space becomes the output block
    const int h = int(bh % heads);
    const float s = alpha_v[h] / 255.0f;
    const float add = fmaf(BmNum<ET>::kCentre, s, beta_v[h]) * rsum;

    const int64_t e0 = (bh * N + r0) * int64_t(N);         // first element of the output block
    const int mis = int(e0 & 7);                           // its offset from a 16-byte boundary, in elements
    _Float16 *lo = reinterpret_cast<_Float16 *>(lds_da);    // element (i, j) of the block at mis + i * N + j

    for (int cbk = cb_first; cbk < nblocks; cbk += cb_step) {
        const int c0 = cbk * 32;
        store_codes(raw);
        if (cbk + cb_step < nblocks) load_codes(c0 + 32 * cb_step, raw);   // the wave's next block
        bm_v8h fc[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) fc[ks] = BmNum<ET>::codes8(*reinterpret_cast<const bm_v2i *>(lv + fl * C::kRowV + ks * 16 + fk));
        bm_v16f acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) acc = BmNum<ET>::mfma(fc[ks], fo[ks], acc);
        // lane l, register v: column c0 + 8*(v/4) + 4*(l/32) + v%4, row l%32
        if (fl < rows) {
            const int at = mis + fl * N + c0 + (lane >> 5) * 4;
            if (c0 + 32 <= N) {                            // uniform: the whole column block lies inside
                // Four consecutive elements from an element-aligned position, with aligned writes only
                // (LDS stalls for dozens of cycles on a misaligned 8-byte write): the first and the last
                // element alone, the 4-byte word that holds elements 1, 2 (odd position) or 0, 1 (even),
                // and element 2 (even) or, again, 3 (odd).
                const bool odd = at & 1;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    bm_v4h o;
#pragma unroll
                    for (int k = 0; k < 4; ++k) o[k] = BmNum<ET>::round(fmaf(s, acc[4 * g + k], add));
                    _Float16 *q = lo + at + 8 * g;
                    q[0] = o[0];
                    q[3] = o[3];
                    *reinterpret_cast<bm_v2h *>(q + (odd ? 1 : 0)) = odd ? bm_v2h{o[1], o[2]} : bm_v2h{o[0], o[1]};
                    q[odd ? 3 : 2] = odd ? o[3] : o[2];
                }
            } else {
#pragma unroll
                for (int g = 0; g < 4; ++g)
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        if (c0 + (lane >> 5) * 4 + 8 * g + k < N) lo[at + 8 * g + k] = BmNum<ET>::round(fmaf(s, acc[4 * g + k], add));
            }
        }
    }
    team_sync();

    // the block leaves: elements [e0, e1) of dA; LDS element x holds global element (e0 - mis) + x
    const int total = rows * N;
    const int64_t ebase = e0 - mis;
    const int v_first = (mis + 7) >> 3, v_end = (mis + total) >> 3;   // whole vectors, in units of 8 elements from ebase
    for (int v = v_first + t; v < v_end; v += kTeam)
        *reinterpret_cast<u32x4 *>(dA + ebase + 8 * int64_t(v)) = *reinterpret_cast<const u32x4 *>(lo + 8 * v);
    if (t < 8) {                                            // before the first whole vector
        const int x = mis + t;
        if (x < 8 * v_first && x < mis + total) dA[ebase + x] = lo[x];
    } else if (t < 16) {                                    // after the last one
        const int x = 8 * v_end + (t - 8);
        if (x >= 8 * v_first && x < mis + total) dA[ebase + x] = lo[x];
    }
}

// ---- dA for long sequences (N a multiple of 8, beyond what k_attn_da's 32 x N output block can hold in LDS) ----------
// A workgroup takes 64 rows i and 256 columns j of one head: the 64 rows of dO and the 256 rows of V codes go to LDS
// once (the codes only until every wave holds its fragments), wave w multiplies the 64 rows by the code rows 64 w ..+63 (four accumulator tiles, codes on the M side as in
// k_attn_da: a lane ends up with one row i and runs of four consecutive j), and its 64 x 64 piece of the result leaves
// through a private LDS region, 32 rows at a time, as aligned 16-byte vectors: 128 contiguous bytes per row and wave,
// 512 per row and workgroup.  The column tiles of a row block are neighbours in the grid.  Dh == 16 * KS.
template <int KS> struct DcCfg {
    static constexpr int Dh = 16 * KS;
    static constexpr int kRowO = 2 * Dh + 16, kRowV = Dh + 16;     // bytes per staged row of dO, of codes
    static constexpr int kRowOut = 64 * 2 + 16;                    // bytes per staged row of a wave's result
    static constexpr int kVecO = Dh / 8, kVecV = Dh / 16;
    // the waves' result regions take the place of the codes once every wave holds its code fragments
    static constexpr int kRows = KS <= 4 ? 128 : 64;               // rows of dO per workgroup (the codes are read once for all of them)
    static constexpr int kCodesAt = kRows * kRowO, kOutAt = kCodesAt;
    static constexpr int kLds = kCodesAt + (256 * kRowV > 4 * 32 * kRowOut ? 256 * kRowV : 4 * 32 * kRowOut);
};

template <int KS, typename ET>
__global__ __launch_bounds__(kThreads, KS <= 4 ? 3 : 2) void k_attn_da_cols(const _Float16 *__restrict__ dO, const int8_t *__restrict__ vq,
                                                                            _Float16 *__restrict__ dA, int N, int heads, int tiles_j,
                                                                            int tiles_i, const float *__restrict__ alpha_v,
                                                                            const float *__restrict__ beta_v)
{
    typedef DcCfg<KS> C;
    __shared__ __attribute__((aligned(16))) unsigned char lds_dc[C::kLds];
    constexpr int Dh = C::Dh;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int fl = lane & 31, fk = (lane >> 5) * 8;
    const unsigned tj = blockIdx.x % unsigned(tiles_j), rest = blockIdx.x / unsigned(tiles_j);
    const int64_t bh = rest / unsigned(tiles_i);
    const int i0 = int(rest % unsigned(tiles_i)) * C::kRows, j0 = int(tj) * 256;
    const int rows = N - i0 < C::kRows ? N - i0 : C::kRows, cols = N - j0 < 256 ? N - j0 : 256;

    {   // staging: rows past the end repeat the last one (their results are never written)
        const u32x4 *ovec = reinterpret_cast<const u32x4 *>(dO + (bh * N + i0) * int64_t(Dh));
        const int o_vecs = rows * C::kVecO;
#pragma unroll
        for (int k = 0; k < (C::kRows * C::kVecO + kThreads - 1) / kThreads; ++k) {
            const int idx = tid + k * kThreads;
            if (idx < C::kRows * C::kVecO)
                *reinterpret_cast<u32x4 *>(lds_dc + (idx / C::kVecO) * C::kRowO + (idx % C::kVecO) * 16) = ovec[idx < o_vecs ? idx : o_vecs - 1];
        }
        const u32x4 *vvec = reinterpret_cast<const u32x4 *>(vq + (bh * N + j0) * int64_t(Dh));
        const int v_vecs = cols * C::kVecV;
#pragma unroll
        for (int k = 0; k < 256 * C::kVecV / kThreads; ++k) {
            const int idx = tid + k * kThreads;
            *reinterpret_cast<u32x4 *>(lds_dc + C::kCodesAt + (idx / C::kVecV) * C::kRowV + (idx % C::kVecV) * 16) = vvec[idx < v_vecs ? idx : v_vecs - 1];
        }
    }
    __syncthreads();
    const int h = int(bh % heads);
    const float s = alpha_v[h] / 255.0f;
    const float off = fmaf(BmNum<ET>::kCentre, s, beta_v[h]);
    unsigned char *lout = lds_dc + C::kOutAt + wave * (32 * C::kRowOut);
    auto wave_sync = [&]() {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };
    // the codes of this wave's 64 columns, as operands: lane l holds code row l%32 (+32), slots 8*(l/32) ..+7 of a step
    bm_v8h fc[2][KS];
#pragma unroll
    for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            fc[jb][ks] = BmNum<ET>::codes8(*reinterpret_cast<const bm_v2i *>(lds_dc + C::kCodesAt + (wave * 64 + jb * 32 + fl) * C::kRowV + ks * 16 + fk));
    __syncthreads();                                       // the codes' place becomes the result regions
    if (wave * 64 >= cols) return;                         // this wave's columns lie past N (no barrier follows)
#pragma unroll
    for (int rb = 0; rb < C::kRows / 32; ++rb) {
        if (rb * 32 >= rows) break;                        // uniform
        bm_v8h fo[KS];
        float rsum = 0.0f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            fo[ks] = *reinterpret_cast<const bm_v8h *>(lds_dc + (rb * 32 + fl) * C::kRowO + (ks * 16 + fk) * 2);
#pragma unroll
            for (int j = 0; j < 8; j += 2) rsum = BmNum<ET>::dot_ones(fo[ks][j], fo[ks][j + 1], rsum);
        }
        rsum += __shfl_xor(rsum, 32);                      // both halves of the row's slots
        const float add = off * rsum;
#pragma unroll
        for (int jb = 0; jb < 2; ++jb) {
            bm_v16f acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) acc = BmNum<ET>::mfma(fc[jb][ks], fo[ks], acc);
            // lane l, register v: column 32*jb + 8*(v/4) + 4*(l/32) + v%4 of the wave's 64, row l%32
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                bm_v4h o;
#pragma unroll
                for (int k = 0; k < 4; ++k) o[k] = BmNum<ET>::round(fmaf(s, acc[4 * g + k], add));
                *reinterpret_cast<bm_v4h *>(lout + fl * C::kRowOut + (jb * 32 + 8 * g + (lane >> 5) * 4) * 2) = o;
            }
        }
        wave_sync();
        // 32 rows x eight vectors of eight columns: lane l takes vector l%8 of rows l/8, l/8 + 8, ..
        const int cv = lane & 7;
        if (wave * 64 + cv * 8 < cols) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int r = (lane >> 3) + 8 * k;
                if (rb * 32 + r < rows)
                    *reinterpret_cast<u32x4 *>(dA + (bh * N + i0 + rb * 32 + r) * int64_t(N) + j0 + wave * 64 + cv * 8) =
                        *reinterpret_cast<const u32x4 *>(lout + r * C::kRowOut + cv * 16);
            }
        }
        wave_sync();                                       // the region is free for the next 32 rows
    }
}

// ---- the two products that contract over the ROW index of both operands: dK = scale * dS^T Q_hat, dV = A_hat^T dO ----
// One workgroup per head.  It walks down the rows i in chunks of 32: the chunk of the N x N operand (dS or the
// A codes) is one contiguous, merely element-aligned piece of memory that comes in as aligned 16-byte
// vectors and lies in LDS as it lies in memory; the chunk of the N x Dh operand (Q codes or dO) has aligned
// rows and goes to LDS row by row.  The next chunk's loads are in flight while a chunk is multiplied
// (two LDS buffers, one barrier per chunk).  The waves share out the blocks of 32 output rows j.  An MFMA
// fragment of the N x N operand -- lane l: column j = l%32, the eight rows 8*(l/32) ..+7 of a 16-row step --
// is gathered from LDS with eight 2-byte (1-byte) reads a row apart; the fragment of the other operand comes
// from transposing reads.  The MFMA runs with the N x Dh operand on the M side, so a lane ends up with one
// output row j and runs of four consecutive d.  Dh == 32 * DT; N <= 128 * JB (JB blocks of j per wave).
template <int DT, int JB, bool WIDE_CODED, int NW> struct TnCfg {
    static constexpr int kNt = 64 * NW;                     // threads of a workgroup (NW waves)
    // WIDE_CODED: the N x N operand is the coded one (dV: A codes, dO plain); else dK: dS plain, Q codes
    static constexpr int Dh = 32 * DT;
    static constexpr int kWideEb = WIDE_CODED ? 1 : 2;     // bytes per element of the N x N operand
    static constexpr int kRowNarrow = WIDE_CODED ? 2 * Dh + 32 : Dh + 32;   // bytes per staged row of the N x Dh operand
    static constexpr int kNarrowVecs = 32 * Dh * (WIDE_CODED ? 2 : 1) / 16;   // 16-byte vectors per chunk of it
    static constexpr int kMaxWideVecs = 4;                 // vectors of the N x N chunk per thread kept in flight
    static size_t wide_bytes(int64_t N) { return (size_t(32) * N * kWideEb + 16 + 64 + 15) & ~size_t(15); }
    static size_t narrow_bytes() { return size_t(32) * kRowNarrow; }
    static size_t lds_bytes(int64_t N) { return 2 * (wide_bytes(N) + narrow_bytes()); }
};

// waves per SIMD the register budget is set for (the accumulators are 16 * DT * JB registers)
template <int DT, int JB, int NW> constexpr int tn_waves_per_simd()
{
    return (NW < 4 ? DT <= 2 : DT * JB <= 4 && DT < 4) ? 3 : DT * JB <= 6 ? 2 : 1;
}

template <int DT, int JB, bool WIDE_CODED, int NW, typename ET>
__global__ __launch_bounds__(64 * NW, (tn_waves_per_simd<DT, JB, NW>())) void k_attn_tn(const void *__restrict__ wide_, const void *__restrict__ narrow_,
                                                         _Float16 *__restrict__ out, int N, int heads, float scale,
                                                         const float *__restrict__ alpha, const float *__restrict__ beta,
                                                         int wide_bytes, int64_t wide_elems)
{
    typedef TnCfg<DT, JB, WIDE_CODED, NW> C;
    constexpr int kNt = C::kNt;
    typedef typename BmElem<WIDE_CODED>::type WideT;        // element of the N x N operand
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_tn[];
    constexpr int Dh = C::Dh;
    constexpr int kEw = 16 / C::kWideEb;                   // elements of the N x N operand per 16-byte vector
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t bh = blockIdx.x;
    const WideT *wide = static_cast<const WideT *>(wide_);
    const unsigned char *narrow = static_cast<const unsigned char *>(narrow_) + bh * N * int64_t(Dh) * (WIDE_CODED ? 2 : 1);
    const int fl = lane & 31, half = lane >> 5;
    const int nchunks = (N + 31) >> 5;
    // LDS: [chunk of the N x N operand] x 2, then [chunk of the N x Dh operand] x 2 (offsets, so that the
    // accesses stay LDS accesses)
    auto buf_w = [&](int b) { return lds_tn + b * wide_bytes; };
    auto buf_n = [&](int b) { return lds_tn + 2 * wide_bytes + b * (32 * C::kRowNarrow); };

    // ---- staging -------------------------------------------------------------------------------------
    u32x4 wv[C::kMaxWideVecs], nv[(C::kNarrowVecs + kNt - 1) / kNt];
    int mis = 0, nvec = 0, whole = 0;                      // of the chunk held in wv
    auto chunk_geom = [&](int c, int &mis_, int &nvec_, int &whole_, int64_t &ebase_) {
        const int i0 = c * 32;
        const int rows = N - i0 < 32 ? N - i0 : 32;
        const int64_t e0 = (bh * N + i0) * int64_t(N);     // first element of the chunk
        mis_ = int(e0 & (kEw - 1));
        ebase_ = e0 - mis_;
        nvec_ = (mis_ + rows * N + kEw - 1) / kEw;
        // the last vector of the whole tensor may reach past its end: that one is read element by element
        whole_ = wide_elems - ebase_ >= int64_t(nvec_) * kEw ? nvec_ : nvec_ - 1;
    };
    auto load_chunk = [&](int c) {
        int64_t ebase;
        chunk_geom(c, mis, nvec, whole, ebase);
        const u32x4 *src = reinterpret_cast<const u32x4 *>(wide + ebase);
#pragma unroll
        for (int k = 0; k < C::kMaxWideVecs; ++k) {
            const int v = tid + k * kNt;
            if (v < whole) wv[k] = src[v];
        }
        const u32x4 *nsrc = reinterpret_cast<const u32x4 *>(narrow + int64_t(c) * 32 * Dh * (WIDE_CODED ? 2 : 1));
        const int nrows = N - c * 32 < 32 ? N - c * 32 : 32;
        const int nvecs = nrows * (C::kNarrowVecs / 32);
#pragma unroll
        for (int k = 0; k < int(sizeof(nv) / sizeof(nv[0])); ++k) {
            const int v = tid + k * kNt;
            if (v < nvecs) nv[k] = nsrc[v];
            else nv[k] = u32x4{0u, 0u, 0u, 0u};            // rows past the end: zeros (codes of 0 / plain zeros)
        }
    };
    auto store_chunk = [&](int c, int b) {
        unsigned char *lw = buf_w(b);
#pragma unroll
        for (int k = 0; k < C::kMaxWideVecs; ++k) {
            const int v = tid + k * kNt;
            if (v < whole) *reinterpret_cast<u32x4 *>(lw + v * 16) = wv[k];
        }
        if (whole < nvec && tid < kEw) {                   // the tensor's very last, partial vector
            int64_t ebase;
            int m_, n_, w_;
            chunk_geom(c, m_, n_, w_, ebase);
            const int64_t g = ebase + int64_t(whole) * kEw + tid;
            reinterpret_cast<WideT *>(lw)[whole * kEw + tid] = g < wide_elems ? wide[g] : WideT(0);
        }
        constexpr int kVecRow = C::kNarrowVecs / 32;
#pragma unroll
        for (int k = 0; k < int(sizeof(nv) / sizeof(nv[0])); ++k) {
            const int v = tid + k * kNt;
            if (v < C::kNarrowVecs) *reinterpret_cast<u32x4 *>(buf_n(b) + (v / kVecRow) * C::kRowNarrow + (v % kVecRow) * 16) = nv[k];
        }
    };

    // ---- accumulators: wave w takes the blocks j = 32 * (w + NW * jb) ----------------------------------
    bm_v16f acc[JB][DT];
    bm_v16f acc1[WIDE_CODED ? DT : 1];                     // dV: column sums of dO per d, from MFMAs against ones
    float csum[JB];                                        // dK: column sums of dS per j, per lane
#pragma unroll
    for (int jb = 0; jb < JB; ++jb) {
        csum[jb] = 0.0f;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[jb][dt][v] = 0.0f;
    }
#pragma unroll
    for (int dt = 0; dt < (WIDE_CODED ? DT : 1); ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc1[dt][v] = 0.0f;
    bm_v8h ones;
#pragma unroll
    for (int j = 0; j < 8; ++j) ones[j] = __builtin_bit_cast(_Float16, BmNum<ET>::kOne);
    const int blk = lane >> 4, sl = lane & 15;

    load_chunk(0);
    for (int c = 0; c < nchunks; ++c) {
        const int b = c & 1;
        const int mis_c = mis;
        store_chunk(c, b);
        if (c + 1 < nchunks) load_chunk(c + 1);
        __syncthreads();   // chunk c is in LDS; every wave has finished with chunk c - 1 (the other buffer)
        const int rows = N - c * 32 < 32 ? N - c * 32 : 32;
        const WideT *lw = reinterpret_cast<const WideT *>(buf_w(b));
        const unsigned char *ln = buf_n(b);
        const bool ragged = rows < 32;                     // uniform: the head's last chunk
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            if (ks * 16 >= rows) break;                    // uniform
            // fragments of the N x Dh operand: lane: d = 32*dt + l%32, rows 16*ks + 8*(l/32) ..+7
            bm_v8h fn[DT];
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                if (WIDE_CODED) {
                    const unsigned char *p = ln + (ks * 16 + (blk >> 1) * 8 + (sl >> 2)) * C::kRowNarrow + (dt * 32 + (blk & 1) * 16 + (sl & 3) * 4) * 2;
                    const bm_v4h lo = __builtin_bit_cast(bm_v4h, __builtin_amdgcn_ds_read_tr16_b64_v4i16(BM_LDS3(bm_v4s, p)));
                    const bm_v4h hi = __builtin_bit_cast(bm_v4h, __builtin_amdgcn_ds_read_tr16_b64_v4i16(BM_LDS3(bm_v4s, p + 4 * C::kRowNarrow)));
                    fn[dt] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    acc1[dt] = BmNum<ET>::mfma(fn[dt], ones, acc1[dt]);
                } else {
                    const unsigned char *p = ln + (ks * 16 + (blk >> 1) * 8 + (sl >> 1)) * C::kRowNarrow + dt * 32 + (blk & 1) * 16 + (sl & 1) * 8;
                    fn[dt] = BmNum<ET>::codes8(__builtin_amdgcn_ds_read_tr8_b64_v2i32(BM_LDS3(bm_v2i, p)));
                }
            }
#pragma unroll
            for (int jb = 0; jb < JB; ++jb) {
                const int j0 = (wave + NW * jb) * 32;
                if (j0 >= N) break;                        // uniform per wave
                const int j = j0 + fl < N ? j0 + fl : N - 1;   // columns past the end repeat the last one; never written
                const int at = mis_c + (ks * 16 + half * 8) * N + j;
                bm_v8h fw;
                if (WIDE_CODED) {
                    // rows past the end meet zeros of the other operand: any code will do there
                    bm_v4u u;
#pragma unroll
                    for (int k = 0; k < 4; ++k)            // two codes per register: bits 0-7 and 16-23
                        u[k] = unsigned(reinterpret_cast<const unsigned char *>(lw)[at + (2 * k) * N]) |
                               (unsigned(reinterpret_cast<const unsigned char *>(lw)[at + (2 * k + 1) * N]) << 16);
                    fw = BmNum<ET>::gathered(u);           // stored bytes -> operand values
                } else {
#pragma unroll
                    for (int k = 0; k < 8; ++k) fw[k] = reinterpret_cast<const _Float16 *>(lw)[at + k * N];
                    if (ragged) {                          // rows past the end: zeros (LDS holds stale data there)
                        bm_v4u w4 = __builtin_bit_cast(bm_v4u, fw);
                        const int r = ks * 16 + half * 8;
#pragma unroll
                        for (int k = 0; k < 4; ++k) w4[k] &= (r + 2 * k < rows ? 0xffffu : 0u) | (r + 2 * k + 1 < rows ? 0xffff0000u : 0u);
                        fw = __builtin_bit_cast(bm_v8h, w4);
                    }
#pragma unroll
                    for (int k = 0; k < 8; k += 2)
                        csum[jb] = BmNum<ET>::dot_ones(fw[k], fw[k + 1], csum[jb]);
                }
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) acc[jb][dt] = BmNum<ET>::mfma(fn[dt], fw, acc[jb][dt]);
            }
        }
    }

    // ---- epilogue: lane l, register v of a tile: d = 32*dt + 8*(v/4) + 4*(l/32) + v%4, row j = j0 + l%32 ----
    const int h = int(bh % heads);
    const float s = alpha[h] / 255.0f;
    const float off = fmaf(BmNum<ET>::kCentre, s, beta[h]);
#pragma unroll
    for (int jb = 0; jb < JB; ++jb) {
        const int j = (wave + NW * jb) * 32 + fl;
        if (j >= N) continue;
        float cs = 0.0f;
        if (!WIDE_CODED) cs = off * (csum[jb] + __shfl_xor(csum[jb], 32));
        _Float16 *po = out + (bh * N + j) * int64_t(Dh) + half * 4;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                bm_v4h o;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const float add = WIDE_CODED ? off * acc1[dt][4 * g + k] : cs;
                    o[k] = BmNum<ET>::round(scale * fmaf(s, acc[jb][dt][4 * g + k], add));
                }
                *reinterpret_cast<bm_v4h *>(po + dt * 32 + g * 8) = o;
            }
    }
}

// ---- the same two products for long sequences (N a multiple of 16, beyond what one workgroup per head can hold) -----
// A workgroup takes 256 columns j of one head and walks down ALL rows i in chunks of 32: per chunk 32 row segments of
// 256 elements of the N x N operand (512 contiguous bytes of dS, 256 of the A codes: aligned 16-byte vectors, rows a
// multiple of 16 elements apart) and the chunk's 32 rows of the N x Dh operand.  Both lie in LDS row by row, with a
// pitch that keeps the transposing reads of sixteen lanes on different banks; every MFMA operand is one or two
// transposing reads (lane: column j or d, eight consecutive rows i).  The next chunk's vectors wait in registers
// while a chunk is multiplied (two LDS buffers, one barrier per chunk).  Wave w takes columns 64 w ..+63 of the tile.
// The workgroups of a head's column tiles are neighbours in the grid: they read adjacent segments of the same rows at
// about the same time and share the N x Dh chunks in the L2.  The N x N operand is read exactly once.
// As in k_attn_tn the N x Dh operand sits on the M side: a lane ends up with one output row j and runs of four d.
template <int DT, bool WIDE_CODED> struct TcCfg {
    static constexpr int Dh = 32 * DT;
    static constexpr int kJW = 256;                        // columns of the N x N operand per workgroup
    static constexpr int kNt = kJW;                        // threads: a wave per 64 columns (two blocks of 32)
    static constexpr int kJB = 2;
    static constexpr int kCR = 16;                         // rows per chunk (N is a multiple of 16: no ragged chunk)
    static constexpr int kAhead = WIDE_CODED ? 2 : 1;      // chunks in registers ahead of the one in LDS: the codes' chunks are
                                                           // half the bytes, and it is bytes in flight that hide the latency
    static constexpr int kWideEb = WIDE_CODED ? 1 : 2;
    static constexpr int kPitchW = kJW * kWideEb + (WIDE_CODED ? 16 : 32);   // bytes per staged row segment
    static constexpr int kVecRowW = kJW * kWideEb / 16;    // 16-byte vectors per row segment
    static constexpr int kWideVecs = kCR * kVecRowW / kNt;   // per thread and chunk: 4 (binary16) or 2 (codes)
    static constexpr int kRowN = WIDE_CODED ? 2 * Dh + 32 : Dh + 32;   // bytes per staged row of the N x Dh operand
    static constexpr int kVecRowN = Dh * (WIDE_CODED ? 2 : 1) / 16;
    static constexpr int kNarrowVecs = (kCR * kVecRowN + kNt - 1) / kNt;
    static constexpr int kStage = kCR * kPitchW + kCR * kRowN;
    static constexpr int kLds = 2 * kStage;
};

template <int DT, bool WIDE_CODED, typename ET>
__global__ __launch_bounds__((TcCfg<DT, WIDE_CODED>::kNt), DT == 4 ? 1 : 2) void k_attn_tn_cols(const void *__restrict__ wide_, const void *__restrict__ narrow_,
                                                              _Float16 *__restrict__ out, int N, int heads, int tiles_j, float scale,
                                                              const float *__restrict__ alpha, const float *__restrict__ beta)
{
    typedef TcCfg<DT, WIDE_CODED> C;
    __shared__ __attribute__((aligned(16))) unsigned char lds_tc[C::kLds];
    constexpr int Dh = C::Dh;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t bh = blockIdx.x / unsigned(tiles_j);
    const int j0 = int(blockIdx.x % unsigned(tiles_j)) * C::kJW;
    const unsigned char *wide = static_cast<const unsigned char *>(wide_) + (bh * N * int64_t(N) + j0) * C::kWideEb;
    const unsigned char *narrow = static_cast<const unsigned char *>(narrow_) + bh * N * int64_t(Dh) * (WIDE_CODED ? 2 : 1);
    const int fl = lane & 31, half = lane >> 5, blk = lane >> 4, sl = lane & 15;
    const int nchunks = N / C::kCR;
    const int cols = N - j0 < C::kJW ? N - j0 : C::kJW;    // columns of this tile that exist (a multiple of 16)

    // ---- staging: a thread's vectors sit at the same place of every chunk ---------------------------------------------
    u32x4 wv[C::kAhead][C::kWideVecs], nv[C::kAhead][C::kNarrowVecs];
    int w_src[C::kWideVecs], w_dst[C::kWideVecs];          // byte offsets from the chunk's first row: in memory (-1: past N), in LDS
#pragma unroll
    for (int k = 0; k < C::kWideVecs; ++k) {
        const int v = tid + k * C::kNt, r = v / C::kVecRowW, cv = v % C::kVecRowW;
        w_src[k] = cv * 16 < cols * C::kWideEb ? r * N * C::kWideEb + cv * 16 : -1;
        w_dst[k] = r * C::kPitchW + cv * 16;
    }
    auto load_chunk = [&](int c, auto set_) {
        constexpr int S = decltype(set_)::value;
        constexpr int rows = C::kCR;
        const unsigned char *src = wide + int64_t(c) * C::kCR * N * C::kWideEb;
#pragma unroll
        for (int k = 0; k < C::kWideVecs; ++k) {
            const int r = (tid + k * C::kNt) / C::kVecRowW;
            wv[S][k] = u32x4{0u, 0u, 0u, 0u};              // columns past N, rows past the end: zeros
            if (w_src[k] >= 0 && r < rows) wv[S][k] = *reinterpret_cast<const u32x4 *>(src + w_src[k]);
        }
        const u32x4 *nsrc = reinterpret_cast<const u32x4 *>(narrow + int64_t(c) * C::kCR * Dh * (WIDE_CODED ? 2 : 1));
#pragma unroll
        for (int k = 0; k < C::kNarrowVecs; ++k) {
            const int v = tid + k * C::kNt;
            nv[S][k] = v < rows * C::kVecRowN ? nsrc[v] : u32x4{0u, 0u, 0u, 0u};
        }
    };
    auto store_chunk = [&](int b, auto set_) {
        constexpr int S = decltype(set_)::value;
        unsigned char *lw = lds_tc + b * C::kStage, *ln = lw + C::kCR * C::kPitchW;
#pragma unroll
        for (int k = 0; k < C::kWideVecs; ++k) *reinterpret_cast<u32x4 *>(lw + w_dst[k]) = wv[S][k];
#pragma unroll
        for (int k = 0; k < C::kNarrowVecs; ++k) {
            const int v = tid + k * C::kNt;
            if (v < C::kCR * C::kVecRowN) *reinterpret_cast<u32x4 *>(ln + (v / C::kVecRowN) * C::kRowN + (v % C::kVecRowN) * 16) = nv[S][k];
        }
    };

    bm_v16f acc[C::kJB][DT];
    float dsum[DT];                                        // dV: column sums of dO for d = 32 dt + l%32 over this lane's rows
    float csum[C::kJB];                                    // dK: column sums of dS per j, per lane
#pragma unroll
    for (int jb = 0; jb < C::kJB; ++jb) {
        csum[jb] = 0.0f;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[jb][dt][v] = 0.0f;
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) dsum[dt] = 0.0f;
    // transposing reads: lane gets column (first column) + l%32 and the rows (first row) + 8*(l/32) ..+7
    const int wide_at = WIDE_CODED ? ((blk >> 1) * 8 + (sl >> 1)) * C::kPitchW + wave * 64 + (blk & 1) * 16 + (sl & 1) * 8
                                   : ((blk >> 1) * 8 + (sl >> 2)) * C::kPitchW + (wave * 64 + (blk & 1) * 16 + (sl & 3) * 4) * 2;
    const int narrow_at = WIDE_CODED ? ((blk >> 1) * 8 + (sl >> 2)) * C::kRowN + ((blk & 1) * 16 + (sl & 3) * 4) * 2
                                     : ((blk >> 1) * 8 + (sl >> 1)) * C::kRowN + (blk & 1) * 16 + (sl & 1) * 8;
    const bool wave_live = wave * 64 < cols;               // uniform per wave

    // chunk c waits in register set c % kAhead; it goes to LDS buffer c % 2 when chunk c - 1 is being multiplied
    auto chunk_step = [&](int c, auto set_) {
        const int b = c & 1;
        store_chunk(b, set_);
        if (c + C::kAhead < nchunks) load_chunk(c + C::kAhead, set_);
        __syncthreads();   // chunk c is in LDS; every wave has finished with chunk c - 1 (the other buffer)
        const unsigned char *lw = lds_tc + b * C::kStage, *ln = lw + C::kCR * C::kPitchW;
        if (!wave_live) return;                          // its columns lie past N (the barrier above is still met)
#pragma unroll
        for (int ks = 0; ks < C::kCR / 16; ++ks) {
            bm_v8h fn[DT];
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                if (WIDE_CODED) {
                    const unsigned char *p = ln + narrow_at + ks * 16 * C::kRowN + dt * 64;
                    const bm_v4h lo = __builtin_bit_cast(bm_v4h, __builtin_amdgcn_ds_read_tr16_b64_v4i16(BM_LDS3(bm_v4s, p)));
                    const bm_v4h hi = __builtin_bit_cast(bm_v4h, __builtin_amdgcn_ds_read_tr16_b64_v4i16(BM_LDS3(bm_v4s, p + 4 * C::kRowN)));
                    fn[dt] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                    for (int q = 0; q < 8; q += 2) dsum[dt] = BmNum<ET>::dot_ones(fn[dt][q], fn[dt][q + 1], dsum[dt]);
                } else {
                    fn[dt] = BmNum<ET>::codes8(__builtin_amdgcn_ds_read_tr8_b64_v2i32(BM_LDS3(bm_v2i, ln + narrow_at + ks * 16 * C::kRowN + dt * 32)));
                }
            }
#pragma unroll
            for (int jb = 0; jb < C::kJB; ++jb) {
                if (wave * 64 + jb * 32 >= cols) break;       // uniform per wave: blocks past N
                bm_v8h fw;
                if (WIDE_CODED) {
                    fw = BmNum<ET>::codes8(__builtin_amdgcn_ds_read_tr8_b64_v2i32(BM_LDS3(bm_v2i, lw + wide_at + ks * 16 * C::kPitchW + jb * 32)));
                } else {
                    const unsigned char *p = lw + wide_at + ks * 16 * C::kPitchW + jb * 64;
                    const bm_v4h lo = __builtin_bit_cast(bm_v4h, __builtin_amdgcn_ds_read_tr16_b64_v4i16(BM_LDS3(bm_v4s, p)));
                    const bm_v4h hi = __builtin_bit_cast(bm_v4h, __builtin_amdgcn_ds_read_tr16_b64_v4i16(BM_LDS3(bm_v4s, p + 4 * C::kPitchW)));
                    fw = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                    for (int k = 0; k < 8; k += 2) csum[jb] = BmNum<ET>::dot_ones(fw[k], fw[k + 1], csum[jb]);
                }
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) acc[jb][dt] = BmNum<ET>::mfma(fn[dt], fw, acc[jb][dt]);
            }
        }
    };
    load_chunk(0, std::integral_constant<int, 0>());
    if (C::kAhead == 2 && nchunks > 1) load_chunk(1, std::integral_constant<int, C::kAhead - 1>());
    for (int c = 0; c < nchunks; c += C::kAhead) {
        chunk_step(c, std::integral_constant<int, 0>());
        if (C::kAhead == 2 && c + 1 < nchunks) chunk_step(c + 1, std::integral_constant<int, C::kAhead - 1>());
    }

    // ---- epilogue: lane l, register v of a tile: d = 32*dt + 8*(v/4) + 4*(l/32) + v%4, row j = (tile's first) + l%32 ----
    const int h = int(bh % heads);
    const float s = alpha[h] / 255.0f;
    const float off = fmaf(BmNum<ET>::kCentre, s, beta[h]);
    float *dsums = reinterpret_cast<float *>(lds_tc);      // dV: the sums of dO per d, for every lane to pick its four
    if (WIDE_CODED) {
        __syncthreads();                                   // every wave is done with the chunks
        if (wave == 0) {                                   // (a live wave: column 0 of the tile always exists)
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                const float t = dsum[dt] + __shfl_xor(dsum[dt], 32);   // both halves of the rows
                if (half == 0) dsums[dt * 32 + fl] = t;
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int jb = 0; jb < C::kJB; ++jb) {
        const int j = j0 + wave * 64 + jb * 32 + fl;
        float cs = 0.0f;
        if (!WIDE_CODED) cs = off * (csum[jb] + __shfl_xor(csum[jb], 32));
        if (j >= N) continue;
        _Float16 *po = out + (bh * N + j) * int64_t(Dh) + half * 4;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                bm_v4h o;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const float add = WIDE_CODED ? off * dsums[dt * 32 + g * 8 + half * 4 + k] : cs;
                    o[k] = BmNum<ET>::round(scale * fmaf(s, acc[jb][dt][4 * g + k], add));
                }
                *reinterpret_cast<bm_v4h *>(po + dt * 32 + g * 8) = o;
            }
    }
}

// ---- dQ = scale * dS K_hat for long rows: one workgroup per head -------------------------------------------
// The head's K codes go to LDS once (rows j, zeros beyond N; fragments by transposing reads).  dS comes in
// chunks of 64 rows -- contiguous, merely element-aligned pieces that lie in LDS as they lie in memory -- the
// next chunk's vectors waiting in registers while a chunk is multiplied.  Wave w takes rows 32*(w&1) ..+31 of
// the chunk and the d tiles of half w>>1.  A lane's dS fragment (eight consecutive j of its row) starts at an
// arbitrary element of LDS: five aligned 4-byte reads, shifted into place (a misaligned 16-byte LDS read
// stalls the LDS for dozens of cycles).  The MFMA runs with the codes on the M side, so a lane ends up with one
// row i and runs of four consecutive d, and the beta term's row sum is a per-lane scalar.
// Dh == 32 * DT, DT even or 1 (each half takes DT/2 tiles; DT == 1: only the waves of half 0 multiply).
template <int DT> struct NnCfg {
    static constexpr int Dh = 32 * DT;
    static constexpr int kRowK = Dh + 32;                  // bytes per staged code row
    static constexpr int kTiles = DT >= 2 ? DT / 2 : 1;    // d tiles of 32 per wave
    static constexpr int kNt = DT >= 2 ? 256 : 128;        // threads: four waves, or two when there is one d tile
    static constexpr int kMaxVecs = 1792 / kNt;            // dS vectors per thread and chunk
    static size_t ds_bytes(int64_t N) { return (size_t(64) * N * 2 + 16 + 64 + 15) & ~size_t(15); }
    static size_t lds_bytes(int64_t N) { return ds_bytes(N) + size_t(ceil_div(N, 16)) * 16 * kRowK; }
};

template <int DT, typename ET>
__global__ __launch_bounds__(NnCfg<DT>::kNt, 3) void k_attn_nn(const _Float16 *__restrict__ dS, const int8_t *__restrict__ kq,
                                                         _Float16 *__restrict__ dQ, int N, int heads, float scale,
                                                         const float *__restrict__ alpha_k, const float *__restrict__ beta_k,
                                                         int ds_bytes, int64_t ds_elems)
{
    typedef NnCfg<DT> C;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_nn[];
    constexpr int Dh = C::Dh;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t bh = blockIdx.x;
    unsigned char *lk = lds_nn + ds_bytes;
    const int fl = lane & 31, half = lane >> 5;
    const int nchunks = (N + 63) >> 6;

    u32x4 wv[C::kMaxVecs];
    int mis = 0, nvec = 0, whole = 0;
    int64_t ebase = 0;
    auto load_chunk = [&](int c) {
        const int i0 = c * 64;
        const int rows = N - i0 < 64 ? N - i0 : 64;
        const int64_t e0 = (bh * N + i0) * int64_t(N);
        mis = int(e0 & 7);
        ebase = e0 - mis;
        nvec = (mis + rows * N + 7) >> 3;
        whole = ds_elems - ebase >= int64_t(nvec) * 8 ? nvec : nvec - 1;   // the tensor's last vector may reach past its end
        const u32x4 *src = reinterpret_cast<const u32x4 *>(dS + ebase);
#pragma unroll
        for (int k = 0; k < C::kMaxVecs; ++k) {
            const int v = tid + k * C::kNt;
            if (v < whole) wv[k] = src[v];
        }
    };
    auto store_chunk = [&]() {
#pragma unroll
        for (int k = 0; k < C::kMaxVecs; ++k) {
            const int v = tid + k * C::kNt;
            if (v < whole) *reinterpret_cast<u32x4 *>(lds_nn + v * 16) = wv[k];
        }
        if (whole < nvec && tid < 8) {
            const int64_t g = ebase + int64_t(whole) * 8 + tid;
            reinterpret_cast<_Float16 *>(lds_nn)[whole * 8 + tid] = g < ds_elems ? dS[g] : (_Float16)0.0f;
        }
    };

    load_chunk(0);
    {   // the head's K codes: rows j of Dh bytes, rows N .. (a multiple of 16) zero
        const u32x4 *kvec = reinterpret_cast<const u32x4 *>(kq + bh * N * int64_t(Dh));
        constexpr int kVecRow = Dh / 16;
        const int kvecs = N * kVecRow, all = ((N + 15) & ~15) * kVecRow;
        for (int v = tid; v < all; v += C::kNt) {
            u32x4 w = {0u, 0u, 0u, 0u};
            if (v < kvecs) w = kvec[v];
            *reinterpret_cast<u32x4 *>(lk + (v / kVecRow) * C::kRowK + (v % kVecRow) * 16) = w;
        }
    }

    const int blk = lane >> 4, sl = lane & 15;
    const int i_loc = (wave & 1) * 32 + fl;                // row of the chunk
    const int d0 = (wave >> 1) * (DT >= 2 ? Dh / 2 : 0);
    const unsigned char *pk = lk + ((blk >> 1) * 8 + (sl >> 1)) * C::kRowK + d0 + (blk & 1) * 16 + (sl & 1) * 8;
    const unsigned *lds32 = reinterpret_cast<const unsigned *>(lds_nn);
    const int h = int(bh % heads);
    const float s = alpha_k[h] / 255.0f;
    const float off = fmaf(BmNum<ET>::kCentre, s, beta_k[h]);

    for (int c = 0; c < nchunks; ++c) {
        __syncthreads();                                   // the previous chunk has been multiplied
        const int mis_c = mis;
        store_chunk();
        if (c + 1 < nchunks) load_chunk(c + 1);
        __syncthreads();
        const int rows = N - c * 64 < 64 ? N - c * 64 : 64;
        if ((wave & 1) * 32 >= rows) continue;             // uniform per wave; the barriers are at the loop's top
        const int e_row = mis_c + (i_loc < rows ? i_loc : rows - 1) * N + half * 8;   // rows past the end repeat the last one
        const int shift = (e_row & 1) * 16;
        bm_v16f acc[C::kTiles];
#pragma unroll
        for (int t = 0; t < C::kTiles; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;
        float rsum = 0.0f;
        for (int j0 = 0; j0 < N; j0 += 16) {
            const int w0 = (e_row + j0) >> 1;
            unsigned w[5];
#pragma unroll
            for (int q = 0; q < 5; ++q) w[q] = lds32[w0 + q];
            bm_v4u f;
#pragma unroll
            for (int q = 0; q < 4; ++q) f[q] = __builtin_amdgcn_alignbit(w[q + 1], w[q], shift);
            if (j0 + 16 > N) {                             // uniform: the row's ragged end, zeros beyond it
                const int j = j0 + half * 8;
#pragma unroll
                for (int q = 0; q < 4; ++q) f[q] &= (j + 2 * q < N ? 0xffffu : 0u) | (j + 2 * q + 1 < N ? 0xffff0000u : 0u);
            }
            const bm_v8h fs = __builtin_bit_cast(bm_v8h, f);
#pragma unroll
            for (int q = 0; q < 8; q += 2)
                rsum = BmNum<ET>::dot_ones(fs[q], fs[q + 1], rsum);
#pragma unroll
            for (int t = 0; t < C::kTiles; ++t) {
                const bm_v8h fc = BmNum<ET>::codes8(__builtin_amdgcn_ds_read_tr8_b64_v2i32(BM_LDS3(bm_v2i, pk + j0 * C::kRowK + t * 32)));
                acc[t] = BmNum<ET>::mfma(fc, fs, acc[t]);
            }
        }
        rsum += __shfl_xor(rsum, 32);                      // both halves of the row's slots
        if (i_loc < rows) {
            // lane l, register v of a tile: d = 32*t + 8*(v/4) + 4*(l/32) + v%4, row i = l%32
            const float add = off * rsum;
            _Float16 *po = dQ + (bh * N + c * 64 + i_loc) * int64_t(Dh) + d0 + half * 4;
#pragma unroll
            for (int t = 0; t < C::kTiles; ++t)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    bm_v4h o;
#pragma unroll
                    for (int k = 0; k < 4; ++k) o[k] = BmNum<ET>::round(scale * fmaf(s, acc[t][4 * g + k], add));
                    *reinterpret_cast<bm_v4h *>(po + t * 32 + g * 8) = o;
                }
        }
    }
}

// ---- dQ for long sequences (N a multiple of 8): a workgroup takes 64 rows i of one head and walks along the columns ----
// j in chunks of 64 (larger chunks cost workgroups per CU, which cost more than the shorter row segments): per chunk 64
// row segments of dS (aligned 16-byte vectors) and the chunk's rows of K codes, both in LDS row by row, the next two
// chunks' vectors waiting in registers (two LDS buffers, one barrier per chunk).  Wave w takes rows 32 (w & 1) ..+31 and the d tiles of parity w >> 1.  A lane's dS fragment (its row, eight
// consecutive j) is one aligned 16-byte LDS read; the codes come through the byte-transposing read.  Codes on the M
// side as in k_attn_nn: a lane ends up with one row i and runs of four consecutive d.  dS is read exactly once.
template <int DT> struct NrCfg {
    static constexpr int Dh = 32 * DT;
    static constexpr int kJC = 64;                         // columns per chunk
    static constexpr int kPitchS = kJC * 2 + 16;           // bytes per staged row segment of dS: 16 (mod 128), eight rows' reads on different banks
    static constexpr int kRowK = Dh + 32;                  // bytes per staged code row
    static constexpr int kTiles = DT >= 2 ? DT / 2 : 1;
    static constexpr int kVecRowS = kJC / 8, kVecRowK = Dh / 16;
    static constexpr int kSVecs = 64 * kVecRowS / kThreads, kKVecs = (kJC * kVecRowK + kThreads - 1) / kThreads;
    static constexpr int kStage = 64 * kPitchS + kJC * kRowK;
    static constexpr int kLds = 2 * kStage;
    static constexpr int kAhead = 2;                       // chunks in registers ahead of the one in LDS
};

template <int DT, typename ET>
__global__ __launch_bounds__(kThreads, 2) void k_attn_nn_rows(const _Float16 *__restrict__ dS, const int8_t *__restrict__ kq,
                                                              _Float16 *__restrict__ dQ, int N, int heads, int tiles_i, float scale,
                                                              const float *__restrict__ alpha_k, const float *__restrict__ beta_k)
{
    typedef NrCfg<DT> C;
    __shared__ __attribute__((aligned(16))) unsigned char lds_nr[C::kLds];
    constexpr int Dh = C::Dh;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t bh = blockIdx.x / unsigned(tiles_i);
    const int i0 = int(blockIdx.x % unsigned(tiles_i)) * 64;
    const int rows = N - i0 < 64 ? N - i0 : 64;
    const int fl = lane & 31, half = lane >> 5, blk = lane >> 4, sl = lane & 15;
    const int nchunks = (N + C::kJC - 1) / C::kJC;
    const unsigned char *srow = reinterpret_cast<const unsigned char *>(dS + (bh * N + i0) * int64_t(N));
    const unsigned char *krow = reinterpret_cast<const unsigned char *>(kq + bh * N * int64_t(Dh));

    u32x4 sv[C::kAhead][C::kSVecs], kv[C::kAhead][C::kKVecs];
    auto load_chunk = [&](int c, auto set_) {
        constexpr int S = decltype(set_)::value;
        const int j0 = c * C::kJC;
        const int cols = N - j0 < C::kJC ? N - j0 : C::kJC;   // a multiple of 8
#pragma unroll
        for (int k = 0; k < C::kSVecs; ++k) {
            const int v = tid + k * kThreads, r = v / C::kVecRowS, cv = v % C::kVecRowS;
            sv[S][k] = u32x4{0u, 0u, 0u, 0u};           // columns past N meet codes of zero weight: zeros; rows past the end are never written
            if (r < rows && cv * 8 < cols) sv[S][k] = *reinterpret_cast<const u32x4 *>(srow + (int64_t(r) * N + j0 + cv * 8) * 2);
        }
        const u32x4 *ksrc = reinterpret_cast<const u32x4 *>(krow + int64_t(j0) * Dh);
#pragma unroll
        for (int k = 0; k < C::kKVecs; ++k) {
            const int v = tid + k * kThreads;
            kv[S][k] = v < cols * C::kVecRowK ? ksrc[v] : u32x4{0u, 0u, 0u, 0u};
        }
    };
    auto store_chunk = [&](int b, auto set_) {
        constexpr int S = decltype(set_)::value;
        unsigned char *ls = lds_nr + b * C::kStage, *lk = ls + 64 * C::kPitchS;
#pragma unroll
        for (int k = 0; k < C::kSVecs; ++k) {
            const int v = tid + k * kThreads;
            *reinterpret_cast<u32x4 *>(ls + (v / C::kVecRowS) * C::kPitchS + (v % C::kVecRowS) * 16) = sv[S][k];
        }
#pragma unroll
        for (int k = 0; k < C::kKVecs; ++k) {
            const int v = tid + k * kThreads;
            if (v < C::kJC * C::kVecRowK) *reinterpret_cast<u32x4 *>(lk + (v / C::kVecRowK) * C::kRowK + (v % C::kVecRowK) * 16) = kv[S][k];
        }
    };

    const int i_loc = (wave & 1) * 32 + fl;
    const int tpar = wave >> 1;                            // this wave's d tiles: tpar, tpar + 2, ..  (DT == 1: only parity 0 multiplies)
    const bool wave_live = (wave & 1) * 32 < rows && (DT >= 2 || tpar == 0);
    const int s_at = i_loc * C::kPitchS + half * 16;
    const int k_at = ((blk >> 1) * 8 + (sl >> 1)) * C::kRowK + (blk & 1) * 16 + (sl & 1) * 8 + tpar * 32;
    bm_v16f acc[C::kTiles];
#pragma unroll
    for (int t = 0; t < C::kTiles; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;
    float rsum = 0.0f;

    // chunk c waits in register set c % 2; it goes to LDS buffer c % 2 when chunk c - 1 is being multiplied
    auto chunk_step = [&](int c, auto set_) {
        const int b = c & 1;
        store_chunk(b, set_);
        if (c + C::kAhead < nchunks) load_chunk(c + C::kAhead, set_);
        __syncthreads();   // chunk c is in LDS; every wave has finished with chunk c - 1 (the other buffer)
        if (!wave_live) return;
        const unsigned char *ls = lds_nr + b * C::kStage, *lk = ls + 64 * C::kPitchS;
        const int cols = N - c * C::kJC < C::kJC ? N - c * C::kJC : C::kJC;
#pragma unroll
        for (int ks = 0; ks < C::kJC / 16; ++ks) {
            if (ks * 16 >= cols) break;                    // uniform; a last step of eight columns multiplies zeros in its second half
            const bm_v8h fs = *reinterpret_cast<const bm_v8h *>(ls + s_at + ks * 32);
#pragma unroll
            for (int q = 0; q < 8; q += 2) rsum = BmNum<ET>::dot_ones(fs[q], fs[q + 1], rsum);
#pragma unroll
            for (int t = 0; t < C::kTiles; ++t) {
                const bm_v8h fc = BmNum<ET>::codes8(__builtin_amdgcn_ds_read_tr8_b64_v2i32(BM_LDS3(bm_v2i, lk + k_at + ks * 16 * C::kRowK + t * 64)));
                acc[t] = BmNum<ET>::mfma(fc, fs, acc[t]);
            }
        }
    };
    load_chunk(0, std::integral_constant<int, 0>());
    if (nchunks > 1) load_chunk(1, std::integral_constant<int, 1>());
    for (int c = 0; c < nchunks; c += 2) {
        chunk_step(c, std::integral_constant<int, 0>());
        if (c + 1 < nchunks) chunk_step(c + 1, std::integral_constant<int, 1>());
    }
    if (!wave_live) return;
    rsum += __shfl_xor(rsum, 32);                          // both halves of the row's slots
    if (i_loc < rows) {
        // lane l, register v of a tile: d = 32*(tile) + 8*(v/4) + 4*(l/32) + v%4, row i = l%32
        const int h = int(bh % heads);
        const float s = alpha_k[h] / 255.0f;
        const float add = fmaf(BmNum<ET>::kCentre, s, beta_k[h]) * rsum;
        _Float16 *po = dQ + (bh * N + i0 + i_loc) * int64_t(Dh) + tpar * 32 + half * 4;
#pragma unroll
        for (int t = 0; t < C::kTiles; ++t)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                bm_v4h o;
#pragma unroll
                for (int k = 0; k < 4; ++k) o[k] = BmNum<ET>::round(scale * fmaf(s, acc[t][4 * g + k], add));
                *reinterpret_cast<bm_v4h *>(po + t * 64 + g * 8) = o;
            }
    }
}

static bool nn_rows_fits(int64_t batches, int64_t N, int64_t Dh)
{
    if (Dh != 32 && Dh != 64 && Dh != 128) return false;
    return N % 8 == 0 && N >= 64 && batches * ceil_div(N, 64) < (int64_t(1) << 31);
}

template <typename ET>
static void launch_nn_rows(const _Float16 *dS, const int8_t *kq, _Float16 *dQ, int64_t batches, int N, int Dh, int heads, float scale,
                           const float *alpha_k, const float *beta_k, hipStream_t s)
{
    const int tiles_i = int(ceil_div(N, 64));
    const dim3 grid(unsigned(batches * tiles_i));
    if (Dh == 32) hipLaunchKernelGGL((k_attn_nn_rows<1, ET>), grid, dim3(kThreads), 0, s, dS, kq, dQ, N, heads, tiles_i, scale, alpha_k, beta_k);
    else if (Dh == 64) hipLaunchKernelGGL((k_attn_nn_rows<2, ET>), grid, dim3(kThreads), 0, s, dS, kq, dQ, N, heads, tiles_i, scale, alpha_k, beta_k);
    else hipLaunchKernelGGL((k_attn_nn_rows<4, ET>), grid, dim3(kThreads), 0, s, dS, kq, dQ, N, heads, tiles_i, scale, alpha_k, beta_k);
}

// whether k_attn_da can take the shape, and in which mode
static bool da_solo(int64_t batches, int64_t N) { return N <= 64 && batches * ceil_div(N, 32) < (int64_t(1) << 32); }
template <int KS> static bool da_fits(int64_t batches, int64_t N) { return DaCfg<KS>::lds_bytes(N, da_solo(batches, N)) <= 65536; }

template <int KS, typename ET> static void launch_da(const _Float16 *dO, const int8_t *vq, _Float16 *dA, int64_t batches, int N, int heads,
                                        const float *alpha_v, const float *beta_v, hipStream_t s)
{
    typedef DaCfg<KS> C;
    const int codes_at = int(C::codes_at(N));
    if (da_solo(batches, N)) {
        const int64_t items = batches * ceil_div(N, 32);
        hipLaunchKernelGGL((k_attn_da<KS, true, ET>), dim3(unsigned(ceil_div(items, C::kWaves))), dim3(kThreads), C::lds_bytes(N, true), s, dO,
                           vq, dA, N, heads, alpha_v, beta_v, int64_t(0), codes_at, unsigned(items));
        return;
    }
    const unsigned gx = unsigned(ceil_div(N, 32));
    for (int64_t b0 = 0; b0 < batches; b0 += 65535) {   // the y extent of a grid is limited to 65535
        const int64_t nb = batches - b0 < 65535 ? batches - b0 : 65535;
        hipLaunchKernelGGL((k_attn_da<KS, false, ET>), dim3(gx, unsigned(nb)), dim3(kThreads), C::lds_bytes(N, false), s, dO, vq, dA, N,
                           heads, alpha_v, beta_v, b0, codes_at, 0u);
    }
}

// whether k_attn_tn can take the shape: the chunk of 32 rows of the N x N operand within kMaxWideVecs vectors per
// thread, at most 2 blocks of j per wave, LDS within the 64 KiB a kernel gets by default
template <bool WIDE_CODED> static bool tn_fits(int64_t N, int64_t Dh)
{
    if (Dh != 32 && Dh != 64 && Dh != 96 && Dh != 128) return false;
    const int64_t eb = WIDE_CODED ? 1 : 2, per_vec = 16 / eb;
    if ((32 * N + 2 * (per_vec - 1)) / per_vec + 1 > int64_t(4) * kThreads) return false;
    if (N > 256) return false;
    const int64_t wide = (32 * N * eb + 16 + 64 + 15) / 16 * 16, narrow = 32 * (WIDE_CODED ? 2 * Dh + 32 : Dh + 32);
    return 2 * (wide + narrow) <= 65536;
}

template <int DT, int JB, bool WIDE_CODED, int NW, typename ET>
static void launch_tn_one(const void *wide, const void *narrow, _Float16 *out, int64_t batches, int N, int heads, float scale,
                          const float *alpha, const float *beta, hipStream_t s)
{
    typedef TnCfg<DT, JB, WIDE_CODED, NW> C;
    hipLaunchKernelGGL((k_attn_tn<DT, JB, WIDE_CODED, NW, ET>), dim3(unsigned(batches)), dim3(C::kNt), C::lds_bytes(N), s, wide, narrow,
                       out, N, heads, scale, alpha, beta, int(C::wide_bytes(N)), batches * N * int64_t(N));
}

template <bool WIDE_CODED, typename ET>
static void launch_tn(const void *wide, const void *narrow, _Float16 *out, int64_t batches, int N, int Dh, int heads, float scale,
                      const float *alpha, const float *beta, hipStream_t s)
{
    // waves per workgroup and blocks of j per wave, so that no wave is left without a block
#define MESA_TN(DT_) \
    do { \
        if (N <= 32) launch_tn_one<DT_, 1, WIDE_CODED, 1, ET>(wide, narrow, out, batches, N, heads, scale, alpha, beta, s); \
        else if (N <= 64) launch_tn_one<DT_, 1, WIDE_CODED, 2, ET>(wide, narrow, out, batches, N, heads, scale, alpha, beta, s); \
        else if (N <= 128) launch_tn_one<DT_, 1, WIDE_CODED, 4, ET>(wide, narrow, out, batches, N, heads, scale, alpha, beta, s); \
        else launch_tn_one<DT_, 2, WIDE_CODED, 4, ET>(wide, narrow, out, batches, N, heads, scale, alpha, beta, s); \
    } while (0)
    if (Dh == 32) MESA_TN(1);
    else if (Dh == 64) MESA_TN(2);
    else if (Dh == 96) MESA_TN(3);
    else MESA_TN(4);
#undef MESA_TN
}

// whether k_attn_nn can take the shape: a 64-row chunk of dS within kMaxVecs vectors per thread, LDS within 64 KiB
// long sequences: k_attn_da_cols
static bool da_cols_fits(int64_t batches, int64_t N, int64_t Dh)
{
    if (Dh != 32 && Dh != 64 && Dh != 128) return false;
    // from 64 on: below, at most one of a workgroup's four waves has columns (N = 48: 0.28 against 0.24 ms for N = 49 through k_attn_da)
    return N % 8 == 0 && N >= 64 && batches * ceil_div(N, 256) * ceil_div(N, 64) < (int64_t(1) << 31);   // 64: the fewest rows a workgroup takes
}

template <typename ET>
static void launch_da_cols(const _Float16 *dO, const int8_t *vq, _Float16 *dA, int64_t batches, int N, int Dh, int heads,
                           const float *alpha_v, const float *beta_v, hipStream_t s)
{
#define MESA_LAUNCH_DC(KS_) \
    do { \
        const int tiles_j = int(ceil_div(N, 256)), tiles_i = int(ceil_div(N, DcCfg<KS_>::kRows)); \
        hipLaunchKernelGGL((k_attn_da_cols<KS_, ET>), dim3(unsigned(batches * tiles_j * tiles_i)), dim3(kThreads), 0, s, dO, vq, dA, N, heads, \
                           tiles_j, tiles_i, alpha_v, beta_v); \
    } while (0)
    if (Dh == 32) MESA_LAUNCH_DC(2);
    else if (Dh == 64) MESA_LAUNCH_DC(4);
    else MESA_LAUNCH_DC(8);
#undef MESA_LAUNCH_DC
}

// long sequences: k_attn_tn_cols
static bool tn_cols_fits(int64_t batches, int64_t N, int64_t Dh)
{
    if (Dh != 32 && Dh != 64 && Dh != 128) return false;
    return N % 16 == 0 && N >= 64 && batches * ceil_div(N, 256) < (int64_t(1) << 31);
}

template <bool WIDE_CODED, typename ET>
static void launch_tn_cols(const void *wide, const void *narrow, _Float16 *out, int64_t batches, int N, int Dh, int heads, float scale,
                           const float *alpha, const float *beta, hipStream_t s)
{
#define MESA_LAUNCH_TC(DT_) \
    do { \
        typedef TcCfg<DT_, WIDE_CODED> C; \
        const int tiles_j = int(ceil_div(N, C::kJW)); \
        hipLaunchKernelGGL((k_attn_tn_cols<DT_, WIDE_CODED, ET>), dim3(unsigned(batches * tiles_j)), dim3(C::kNt), 0, s, wide, narrow, out, N, \
                           heads, tiles_j, scale, alpha, beta); \
    } while (0)
    if (Dh == 32) MESA_LAUNCH_TC(1);
    else if (Dh == 64) MESA_LAUNCH_TC(2);
    else MESA_LAUNCH_TC(4);
#undef MESA_LAUNCH_TC
}

static bool nn_fits(int64_t N, int64_t Dh)
{
    if (Dh != 32 && Dh != 64 && Dh != 128) return false;
    if ((64 * N + 14) / 8 + 1 > 1792) return false;
    const int64_t ds = (64 * N * 2 + 16 + 64 + 15) / 16 * 16;
    return ds + ceil_div(N, 16) * 16 * (Dh + 32) <= 65536;
}

template <int DT, typename ET> static void launch_nn(const _Float16 *dS, const int8_t *kq, _Float16 *dQ, int64_t batches, int N, int heads,
                                        float scale, const float *alpha_k, const float *beta_k, hipStream_t s)
{
    typedef NnCfg<DT> C;
    hipLaunchKernelGGL((k_attn_nn<DT, ET>), dim3(unsigned(batches)), dim3(C::kNt), C::lds_bytes(N), s, dS, kq, dQ, N, heads, scale,
                       alpha_k, beta_k, int(C::ds_bytes(N)), batches * N * int64_t(N));
}

static mesa_status check_attn(int64_t B, int64_t H, int64_t N, int64_t Dh, mesa_dtype dt)
{
    if (!valid_dtype(dt) || B < 0 || H < 0 || N < 0 || Dh < 0) return MESA_ERR_INVALID_ARG;
    if (N >= (int64_t(1) << 20) || Dh >= (int64_t(1) << 20)) return MESA_ERR_UNSUPPORTED;
    // 32-bit element offsets inside one (sample, head); the row / column tile counts fit a grid dimension
    if ((long double)N * (long double)N >= 2147483648.0L || (long double)N * (long double)Dh >= 2147483648.0L)
        return MESA_ERR_UNSUPPORTED;
    if ((long double)B * (long double)H >= 9.0e15L) return MESA_ERR_UNSUPPORTED;
    return MESA_OK;
}

}  // namespace mesa

using namespace mesa;

extern "C" MESA_EXPORT mesa_status mesa_attn_av_bwd_q(const int8_t *aq, const int8_t *vq, int64_t B, int64_t H, int64_t N,
                                                      int64_t Dh, const float *alpha_a, const float *beta_a,
                                                      const float *alpha_v, const float *beta_v, const void *dO, void *dA,
                                                      void *dV, mesa_dtype dt, void *stream)
{
    mesa_status st = check_attn(B, H, N, Dh, dt);
    if (st != MESA_OK) return st;
    if (B == 0 || H == 0 || N == 0 || Dh == 0) return MESA_OK;
    if (!aq || !vq || !dO || !dA || !dV || !alpha_a || !beta_a || !alpha_v || !beta_v) return MESA_ERR_INVALID_ARG;
    if (!aligned16(aq) || !aligned16(vq) || !aligned16(dO) || !aligned16(dA) || !aligned16(dV) || !aligned4(alpha_a) ||
        !aligned4(beta_a) || !aligned4(alpha_v) || !aligned4(beta_v))
        return MESA_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t batches = B * H;
    BmmArgs a{};
    a.heads = int(H);
    a.scale = 1.0f;
    // dA[i,j] = sum_d dO[i,d] * V_hat[j,d]:  P = dO (r = i, t = d),  Q = V (t = d, c = j)
    a.x = static_cast<const _Float16 *>(dO); a.y = vq; a.c = static_cast<_Float16 *>(dA);
    a.x_batch = N * Dh; a.y_batch = N * Dh; a.c_batch = N * N;
    a.R = int(N); a.Cn = int(N); a.Tn = int(Dh);
    a.p_rs = Dh; a.p_ts = 1; a.q_ts = 1; a.q_cs = Dh;
    a.alpha = alpha_v; a.beta = beta_v;
    if (dt == MESA_F32 || N < 8 || Dh < 8) {   // binary32, or an extent shorter than one load vector: the plain kernel
        launch_bmm_f32<false>(a, batches, dt, s);
        a.y = aq; a.c = static_cast<_Float16 *>(dV);
        a.y_batch = N * N; a.c_batch = N * Dh;
        a.R = int(N); a.Cn = int(Dh); a.Tn = int(N);
        a.p_rs = 1; a.p_ts = N; a.q_ts = Dh; a.q_cs = 1;
        a.alpha = alpha_a; a.beta = beta_a;
        launch_bmm_f32<true>(a, batches, dt, s);
        return launch_status();
    }
    // aligned rows (N a multiple of 8): the column-tile kernel, at every length -- k_attn_da keeps its 32 x N block at a
    // pitch of N elements, and for N a multiple of 32 its lanes' rows fall on the same LDS banks (N = 256: 0.73 against
    // 0.48 ms for the four products).  Else k_attn_da if its block fits the 64 KiB of LDS a kernel gets by default.
#define MESA_AV_DA(ET) \
    do { \
        if (da_cols_fits(batches, N, Dh)) launch_da_cols<ET>(a.x, vq, a.c, batches, int(N), int(Dh), int(H), alpha_v, beta_v, s); \
        else if (Dh == 32 && da_fits<2>(batches, N)) launch_da<2, ET>(a.x, vq, a.c, batches, int(N), int(H), alpha_v, beta_v, s); \
        else if (Dh == 64 && da_fits<4>(batches, N)) launch_da<4, ET>(a.x, vq, a.c, batches, int(N), int(H), alpha_v, beta_v, s); \
        else if (Dh == 96 && da_fits<6>(batches, N)) launch_da<6, ET>(a.x, vq, a.c, batches, int(N), int(H), alpha_v, beta_v, s); \
        else if (Dh == 128 && da_fits<8>(batches, N)) launch_da<8, ET>(a.x, vq, a.c, batches, int(N), int(H), alpha_v, beta_v, s); \
        else launch_bmm<false, true, true, ET>(a, batches, s); \
    } while (0)
    if (dt == MESA_BF16) MESA_AV_DA(__bf16); else MESA_AV_DA(_Float16);
#undef MESA_AV_DA
    // dV[j,d] = sum_i A_hat[i,j] * dO[i,d]:  P = A (r = j, t = i),  Q = dO (t = i, c = d)
    a.y = aq; a.c = static_cast<_Float16 *>(dV);
    a.y_batch = N * N; a.c_batch = N * Dh;
    a.R = int(N); a.Cn = int(Dh); a.Tn = int(N);
    a.p_rs = 1; a.p_ts = N; a.q_ts = Dh; a.q_cs = 1;
    a.alpha = alpha_a; a.beta = beta_a;
    // aligned rows (N a multiple of 16): the column-tile kernel at every length (k_attn_tn's gathers, a row apart at a
    // pitch of N elements, meet on the same banks when N is a multiple of 32)
#define MESA_AV_DV(ET) \
    do { \
        if (tn_cols_fits(batches, N, Dh)) \
            launch_tn_cols<true, ET>(aq, dO, a.c, batches, int(N), int(Dh), int(H), 1.0f, alpha_a, beta_a, s); \
        else if (tn_fits<true>(N, Dh) && batches < (int64_t(1) << 31)) \
            launch_tn<true, ET>(aq, dO, a.c, batches, int(N), int(Dh), int(H), 1.0f, alpha_a, beta_a, s); \
        else \
            launch_bmm<true, false, false, ET>(a, batches, s); \
    } while (0)
    if (dt == MESA_BF16) MESA_AV_DV(__bf16); else MESA_AV_DV(_Float16);
#undef MESA_AV_DV
    return launch_status();
}

extern "C" MESA_EXPORT mesa_status mesa_attn_qk_bwd_q(const int8_t *qq, const int8_t *kq, int64_t B, int64_t H, int64_t N,
                                                      int64_t Dh, const float *alpha_q, const float *beta_q,
                                                      const float *alpha_k, const float *beta_k, const void *dS, float scale,
                                                      void *dQ, void *dK, mesa_dtype dt, void *stream)
{
    mesa_status st = check_attn(B, H, N, Dh, dt);
    if (st != MESA_OK) return st;
    if (!(scale == scale)) return MESA_ERR_INVALID_ARG;
    if (B == 0 || H == 0 || N == 0 || Dh == 0) return MESA_OK;
    if (!qq || !kq || !dS || !dQ || !dK || !alpha_q || !beta_q || !alpha_k || !beta_k) return MESA_ERR_INVALID_ARG;
    if (!aligned16(qq) || !aligned16(kq) || !aligned16(dS) || !aligned16(dQ) || !aligned16(dK) || !aligned4(alpha_q) ||
        !aligned4(beta_q) || !aligned4(alpha_k) || !aligned4(beta_k))
        return MESA_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t batches = B * H;
    BmmArgs a{};
    a.heads = int(H);
    a.scale = scale;
    a.x = static_cast<const _Float16 *>(dS);
    a.x_batch = N * N; a.y_batch = N * Dh; a.c_batch = N * Dh;
    a.R = int(N); a.Cn = int(Dh); a.Tn = int(N);
    // dQ[i,d] = scale * sum_j dS[i,j] * K_hat[j,d]:  P = dS (r = i, t = j),  Q = K (t = j, c = d)
    a.y = kq; a.c = static_cast<_Float16 *>(dQ);
    a.p_rs = N; a.p_ts = 1; a.q_ts = Dh; a.q_cs = 1;
    a.alpha = alpha_k; a.beta = beta_k;
    if (dt == MESA_F32 || N < 8 || Dh < 8) {
        launch_bmm_f32<false>(a, batches, dt, s);
        a.y = qq; a.c = static_cast<_Float16 *>(dK);
        a.p_rs = 1; a.p_ts = N; a.q_ts = Dh; a.q_cs = 1;
        a.alpha = alpha_q; a.beta = beta_q;
        launch_bmm_f32<false>(a, batches, dt, s);
        return launch_status();
    }
    // k_attn_nn (K codes resident) where it fits, except for N a multiple of 32 (its rows' reads meet on the same banks)
#define MESA_QK_DQ(ET) \
    do { \
        if (nn_rows_fits(batches, N, Dh) && (N % 32 == 0 || !nn_fits(N, Dh))) \
            launch_nn_rows<ET>(a.x, kq, a.c, batches, int(N), int(Dh), int(H), scale, alpha_k, beta_k, s); \
        else if (nn_fits(N, Dh) && batches < (int64_t(1) << 31)) { \
            if (Dh == 32) launch_nn<1, ET>(a.x, kq, a.c, batches, int(N), int(H), scale, alpha_k, beta_k, s); \
            else if (Dh == 64) launch_nn<2, ET>(a.x, kq, a.c, batches, int(N), int(H), scale, alpha_k, beta_k, s); \
            else launch_nn<4, ET>(a.x, kq, a.c, batches, int(N), int(H), scale, alpha_k, beta_k, s); \
        } else if (nn_rows_fits(batches, N, Dh)) \
            launch_nn_rows<ET>(a.x, kq, a.c, batches, int(N), int(Dh), int(H), scale, alpha_k, beta_k, s); \
        else \
            launch_bmm<false, true, false, ET>(a, batches, s); \
    } while (0)
    if (dt == MESA_BF16) MESA_QK_DQ(__bf16); else MESA_QK_DQ(_Float16);
#undef MESA_QK_DQ
    // dK[j,d] = scale * sum_i dS[i,j] * Q_hat[i,d]:  P = dS (r = j, t = i),  Q = Q codes (t = i, c = d)
    a.y = qq; a.c = static_cast<_Float16 *>(dK);
    a.p_rs = 1; a.p_ts = N; a.q_ts = Dh; a.q_cs = 1;
    a.alpha = alpha_q; a.beta = beta_q;
#define MESA_QK_DK(ET) \
    do { \
        if (tn_cols_fits(batches, N, Dh)) \
            launch_tn_cols<false, ET>(dS, qq, a.c, batches, int(N), int(Dh), int(H), scale, alpha_q, beta_q, s); \
        else if (tn_fits<false>(N, Dh) && batches < (int64_t(1) << 31)) \
            launch_tn<false, ET>(dS, qq, a.c, batches, int(N), int(Dh), int(H), scale, alpha_q, beta_q, s); \
        else \
            launch_bmm<false, false, false, ET>(a, batches, s); \
    } while (0)
    if (dt == MESA_BF16) MESA_QK_DK(__bf16); else MESA_QK_DK(_Float16);
#undef MESA_QK_DK
    return launch_status();
}
