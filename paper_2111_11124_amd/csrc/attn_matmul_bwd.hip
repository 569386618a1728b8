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
// is multiplied.  binary16 tensors only.
#include <hip/hip_runtime.h>

#include "api_util.hpp"
#include "common.hpp"

namespace mesa {

typedef _Float16 bm_v8h __attribute__((ext_vector_type(8)));
typedef _Float16 bm_v4h __attribute__((ext_vector_type(4)));
typedef short bm_v4s __attribute__((ext_vector_type(4)));
typedef int bm_v2i __attribute__((ext_vector_type(2)));
typedef float bm_v16f __attribute__((ext_vector_type(16)));

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

struct BmmArgs {
    const _Float16 *x;          // the plain operand
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
    __device__ static __forceinline__ bm_v8h frag(const unsigned char *lds, int l0, int ks, int lane)
    {
        if (TFAST) {
            const unsigned char *p = lds + (l0 + (lane & 31)) * kPitch + (ks * 16 + (lane >> 5) * 8) * kEb;
            if (CODED) return bm_codes_to_half8(*reinterpret_cast<const bm_v2i *>(p));
            return *reinterpret_cast<const bm_v8h *>(p);
        }
        const int blk = lane >> 4, sl = lane & 15;
        if (CODED) {
            const unsigned char *p = lds + (ks * 16 + (blk >> 1) * 8 + (sl >> 1)) * kPitch + l0 + (blk & 1) * 16 + (sl & 1) * 8;
            return bm_codes_to_half8(__builtin_amdgcn_ds_read_tr8_b64_v2i32(BM_LDS3(bm_v2i, p)));
        }
        const unsigned char *p = lds + (ks * 16 + (blk >> 1) * 8 + (sl >> 2)) * kPitch + (l0 + (blk & 1) * 16 + (sl & 3) * 4) * 2;
        const bm_v4h lo = __builtin_bit_cast(bm_v4h, __builtin_amdgcn_ds_read_tr16_b64_v4i16(BM_LDS3(bm_v4s, p)));
        const bm_v4h hi = __builtin_bit_cast(bm_v4h, __builtin_amdgcn_ds_read_tr16_b64_v4i16(BM_LDS3(bm_v4s, p + 4 * kPitch)));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
};

// P_CODED: P is the coded operand (else Q).  P_TFAST / Q_TFAST: the contraction index is the unit-stride
// index of that operand in memory.
template <bool P_CODED, bool P_TFAST, bool Q_TFAST>
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
    for (int j = 0; j < 8; ++j) ones[j] = (_Float16)1.0f;

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
            const bm_v8h fa = OP::frag(LP, wr * 32, ks, lane);
            const bm_v8h fb = OQ::frag(LQ, wc * 32, ks, lane);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa, fb, acc, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(P_CODED ? ones : fa, P_CODED ? fb : ones, acc1, 0, 0, 0);
        }
    }

    // lane l, register v of a 32 x 32 tile: row 8*(v/4) + 4*(l/32) + v%4, column l%32
    const float s = a.alpha[h] / 255.0f;
    const float off = fmaf(128.0f, s, a.beta[h]);
    const int col = c0 + wc * 32 + (lane & 31);
    const int row_l = r0 + wr * 32 + (lane >> 5) * 4;
    // R * Cn < 2^31 (checked by the entry points): 32-bit offsets from the batch's base
    _Float16 *cb = a.c + (int64_t(b) + a.batch0) * a.c_batch;
    const uint32_t o0 = uint32_t(row_l) * uint32_t(a.Cn) + uint32_t(col);
    if (col < a.Cn) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int dr = (v >> 2) * 8 + (v & 3);
            if (row_l + dr < a.R) cb[o0 + uint32_t(dr) * uint32_t(a.Cn)] = (_Float16)(a.scale * fmaf(s, acc[v], off * acc1[v]));
        }
    }
}

template <bool P_CODED, bool P_TFAST, bool Q_TFAST> static void launch_bmm(BmmArgs a, int64_t batches, hipStream_t s)
{
    a.tiles_r = int(ceil_div(a.R, kBmTile));
    a.tiles_c = int(ceil_div(a.Cn, kBmTile));
    // the z extent of a grid is limited to 65535: more (sample, head) pairs than that go in several launches
    for (int64_t b0 = 0; b0 < batches; b0 += 65535) {
        a.batch0 = b0;
        a.head0 = int(b0 % a.heads);
        const int64_t nb = batches - b0 < 65535 ? batches - b0 : 65535;
        hipLaunchKernelGGL((k_bmm_q<P_CODED, P_TFAST, Q_TFAST>), dim3(unsigned(a.tiles_c), unsigned(a.tiles_r), unsigned(nb)),
                           dim3(kThreads), 0, s, a);
    }
}

static mesa_status check_attn(int64_t B, int64_t H, int64_t N, int64_t Dh, mesa_dtype dt)
{
    if (!valid_dtype(dt) || B < 0 || H < 0 || N < 0 || Dh < 0) return MESA_ERR_INVALID_ARG;
    if (dt != MESA_F16) return MESA_ERR_UNSUPPORTED;
    if (N >= (int64_t(1) << 20) || Dh >= (int64_t(1) << 20)) return MESA_ERR_UNSUPPORTED;
    if ((N > 0 && N < 8) || (Dh > 0 && Dh < 8)) return MESA_ERR_UNSUPPORTED;   // an extent shorter than one load vector
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
    launch_bmm<false, true, true>(a, batches, s);
    // dV[j,d] = sum_i A_hat[i,j] * dO[i,d]:  P = A (r = j, t = i),  Q = dO (t = i, c = d)
    a.y = aq; a.c = static_cast<_Float16 *>(dV);
    a.y_batch = N * N; a.c_batch = N * Dh;
    a.R = int(N); a.Cn = int(Dh); a.Tn = int(N);
    a.p_rs = 1; a.p_ts = N; a.q_ts = Dh; a.q_cs = 1;
    a.alpha = alpha_a; a.beta = beta_a;
    launch_bmm<true, false, false>(a, batches, s);
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
    launch_bmm<false, true, false>(a, batches, s);
    // dK[j,d] = scale * sum_i dS[i,j] * Q_hat[i,d]:  P = dS (r = j, t = i),  Q = Q codes (t = i, c = d)
    a.y = qq; a.c = static_cast<_Float16 *>(dK);
    a.p_rs = 1; a.p_ts = N; a.q_ts = Dh; a.q_cs = 1;
    a.alpha = alpha_q; a.beta = beta_q;
    launch_bmm<false, false, false>(a, batches, s);
    return launch_status();
}
