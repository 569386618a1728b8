// conv_dw.hip -- weight gradient of a two-dimensional convolution at the de-quantized input (Sec. 3.1 Eq. 2 with
// G_l the gradient of a convolution; Sec. 3.3: convolutional layers take the group-wise scheme, the input's channels
// in G groups of C_in / G consecutive channels).  Channels-first tensors:
//   dW[co,ci,kh,kw] = sum_{b,oh,ow} dy[b,co,oh,ow] * x_hat[b,ci, oh*sh - ph + kh*dh, ow*sw - pw + kw*dw],
//   x_hat = (q + 128) * s_g(ci) + beta_g(ci) inside the image, 0 outside (the forward pads with zeros).
// With u = q + 128 + c inside the image and 0 outside,
//   dW = s_g * sum dy*u  +  (beta_g - c*s_g) * V[co,kh,kw],   V = sum of dy over the outputs whose tap lies inside,
// so the matrix cores contract dy with small exact integers and the affine map is applied once to finished sums.
//
// Unlike the Linear layer's operands, both tensors here are contiguous along the contraction (the output column
// ow, for stride_w = 1), which is what an MFMA operand wants: a lane holds eight consecutive contraction values of
// one channel.  A kernel tap (kh, kw) only shifts which input row and column meet a given output: kh picks another
// staged row, kw slides the eight-value window by one element -- taken from the same six LDS words with a byte
// alignment instruction.  One stage = one output row segment of up to 128 columns: the dy rows of the workgroup's
// output channels, and for each kh the input row of its input channels, converted once to 16-bit operands as they
// are written to LDS (pads as zeros).  Every tap of a 3x3 kernel then reuses the same dy fragment: nine MFMAs per
// fragment read.  Slices of the (b, oh, segment) range are combined in a fixed order by a second kernel.
//
// This path takes 16-bit tensors with stride_w = dil_w = 1, KH, KW <= 3, pad_w <= 8, W and OW multiples of 8;
// anything else runs the plain kernel at the end of the file.
#include <hip/hip_runtime.h>

#include "api_util.hpp"
#include "common.hpp"

namespace mesa {

typedef _Float16 cv8h __attribute__((ext_vector_type(8)));
typedef __bf16 cv8b __attribute__((ext_vector_type(8)));
typedef float cv16f __attribute__((ext_vector_type(16)));

struct ConvGeom {
    int B, Cin, H, W, Cout, KH, KW, sh, sw, ph, pw, dh, dw, OH, OW;
};

constexpr int kCvSeg = 128;            // output columns per stage
constexpr int kCvPA = kCvSeg + 8;      // LDS pitch of a dy row, elements: 68 words, so eight rows' 16-byte reads miss each other's banks
constexpr int kCvXW = kCvSeg + 16;     // staged input columns: the segment and one 8-column vector on either side
constexpr int kCvPX = kCvXW;           // 72 words
constexpr int kCvXcd = 8;
constexpr int kCvThreads = 256;

template <typename E> struct CvElem;
template <> struct CvElem<_Float16> {
    static constexpr float kCentre = -1024.0f;
    // four codes -> four binary16 values 1024 + (q + 128): 0x6400 | (byte ^ 0x80), exactly
    __device__ static __forceinline__ void convert(uint32_t raw, uint32_t out[2])
    {
        const uint32_t x = raw ^ 0x80808080u;
        out[0] = __builtin_amdgcn_perm(0x64646464u, x, 0x04010400u);
        out[1] = __builtin_amdgcn_perm(0x64646464u, x, 0x04030402u);
    }
    __device__ static __forceinline__ cv16f mfma(u32x4 a, u32x4 b, cv16f c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(cv8h, a), __builtin_bit_cast(cv8h, b), c, 0, 0, 0);
    }
};
template <> struct CvElem<__bf16> {
    static constexpr float kCentre = 0.0f;
    // four codes -> four bfloat16 values q + 128 (0..255 fit its eight significant bits)
    __device__ static __forceinline__ void convert(uint32_t raw, uint32_t out[2])
    {
        const uint32_t x = raw ^ 0x80808080u;
        const uint32_t f0 = __float_as_uint(float(x & 0xFFu)), f1 = __float_as_uint(float((x >> 8) & 0xFFu));
        const uint32_t f2 = __float_as_uint(float((x >> 16) & 0xFFu)), f3 = __float_as_uint(float(x >> 24));
        out[0] = __builtin_amdgcn_perm(f1, f0, 0x07060302u);
        out[1] = __builtin_amdgcn_perm(f3, f2, 0x07060302u);
    }
    __device__ static __forceinline__ cv16f mfma(u32x4 a, u32x4 b, cv16f c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(cv8b, a), __builtin_bit_cast(cv8b, b), c, 0, 0, 0);
    }
};

// TAPS3 = true:  kernels up to 3x3; a wave owns 32 output x 32 input channels for all taps (nine accumulator tiles),
//                the workgroup 64 x 64.
// TAPS3 = false: 1x1 kernels; a wave owns 64 x 64 channels (four tiles), the workgroup 128 x 128.
template <bool TAPS3> struct CvCfg {
    static constexpr int TM = TAPS3 ? 1 : 2, TN = TAPS3 ? 1 : 2;
    static constexpr int XR = TAPS3 ? 3 : 1, XC = TAPS3 ? 3 : 1;      // staged input rows (kh), window shifts (kw)
    static constexpr int COT = 64 * TM, CIT = 64 * TN;
    static constexpr int A_BYTES = COT * kCvPA * 2;
    static constexpr int X_BYTES = XR * CIT * kCvPX * 2;
    static constexpr int LDS = A_BYTES + X_BYTES;
    static constexpr int ND = COT * (kCvSeg / 8) / kCvThreads;        // dy vectors a thread stages
    static constexpr int NXMAX = (XR * CIT * (kCvXW / 8) + kCvThreads - 1) / kCvThreads;   // input vectors, at most
};

// part[split][tap][co][ci] = sum over the split's (b, oh, segment) stages of dy * u,  tap = kh*KW + kw
template <typename E, bool TAPS3, bool PODD>
__global__ __launch_bounds__(kCvThreads, 1) void k_conv_dw(const int8_t *__restrict__ xq, const E *__restrict__ dy, ConvGeom cg,
                                                           int tiles_co, int tiles_ci, int splits, int stages_per_split,
                                                           int nseg, float *__restrict__ part)
{
    using C = CvCfg<TAPS3>;
    extern __shared__ __attribute__((aligned(16))) unsigned char cv_lds[];
    unsigned char *const lds_a = cv_lds;
    unsigned char *const lds_x = cv_lds + C::A_BYTES;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int total = gridDim.x;
    // workgroups that share a slice of the stages run on the same XCD (same L2)
    const int logical = int(blockIdx.x % kCvXcd) * (total / kCvXcd) + int(blockIdx.x / kCvXcd);
    const int ntiles = tiles_co * tiles_ci;
    if (logical >= ntiles * splits) return;
    const int split = logical / ntiles;
    const int t = logical - split * ntiles;
    const int tco = t / tiles_ci, tci = t - tco * tiles_ci;
    const int co0 = tco * C::COT, ci0 = tci * C::CIT;
    const int wm = wave >> 1, wn = wave & 1;
    const int nstages = cg.B * cg.OH * nseg;
    const int st_begin = split * stages_per_split;
    const int st_end = min(st_begin + stages_per_split, nstages);
    const int KH = cg.KH, KW = cg.KW;

    cv16f acc[C::TM][C::TN][C::XR][C::XC];
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
#pragma unroll
        for (int j = 0; j < C::TN; ++j)
#pragma unroll
            for (int a = 0; a < C::XR; ++a)
#pragma unroll
                for (int b = 0; b < C::XC; ++b)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[i][j][a][b][v] = 0.0f;

    // staging registers: what the next stage needs, in flight while this one is multiplied
    u32x4 dreg[C::ND];
    u32x2 xreg[C::NXMAX];
    const int nxrows = KH * C::CIT;                       // staged input rows (kh-major)
    const int nxvec = nxrows * (kCvXW / 8);

    auto stage_coords = [&](int st, int &b, int &oh, int &seg) {
        seg = st % nseg;
        const int r = st / nseg;
        oh = r % cg.OH;
        b = r / cg.OH;
    };
    auto load_stage = [&](int st) {
        int b, oh, seg;
        stage_coords(st, b, oh, seg);
#pragma unroll
        for (int n = 0; n < C::ND; ++n) {
            const int idx = tid + n * kCvThreads;
            const int row = idx >> 4, v = idx & 15;       // 16 vectors of eight columns per row
            const int co = co0 + row, ow0 = seg * kCvSeg + v * 8;
            u32x4 val = {0u, 0u, 0u, 0u};
            if (co < cg.Cout && ow0 < cg.OW)
                val = *reinterpret_cast<const u32x4 *>(dy + ((int64_t(b) * cg.Cout + co) * cg.OH + oh) * cg.OW + ow0);
            dreg[n] = val;
        }
#pragma unroll
        for (int n = 0; n < C::NXMAX; ++n) {
            const int idx = tid + n * kCvThreads;
            u32x2 val = {0u, 0u};
            if (idx < nxvec) {
                const int row = idx / (kCvXW / 8), v = idx - row * (kCvXW / 8);
                const int kh = row / C::CIT, ci = ci0 + (row - kh * C::CIT);
                const int ih = oh * cg.sh - cg.ph + kh * cg.dh;
                const int iw0 = seg * kCvSeg - 8 + v * 8;
                // (whether the vector lies inside the image is decided again, from the same coordinates, when it is stored)
                if (ci < cg.Cin && ih >= 0 && ih < cg.H && iw0 >= 0 && iw0 < cg.W)
                    val = *reinterpret_cast<const u32x2 *>(xq + ((int64_t(b) * cg.Cin + ci) * cg.H + ih) * cg.W + iw0);
            }
            xreg[n] = val;
        }
    };
    auto store_stage = [&](int st) {
        int b, oh, seg;
        stage_coords(st, b, oh, seg);
#pragma unroll
        for (int n = 0; n < C::ND; ++n) {
            const int idx = tid + n * kCvThreads;
            const int row = idx >> 4, v = idx & 15;
            *reinterpret_cast<u32x4 *>(lds_a + (row * kCvPA + v * 8) * 2) = dreg[n];
        }
#pragma unroll
        for (int n = 0; n < C::NXMAX; ++n) {
            const int idx = tid + n * kCvThreads;
            if (idx < nxvec) {
                const int row = idx / (kCvXW / 8), v = idx - row * (kCvXW / 8);
                const int kh = row / C::CIT, ci = ci0 + (row - kh * C::CIT);
                const int ih = oh * cg.sh - cg.ph + kh * cg.dh;
                const int iw0 = seg * kCvSeg - 8 + v * 8;
                u32x4 o = {0u, 0u, 0u, 0u};
                if (ci < cg.Cin && ih >= 0 && ih < cg.H && iw0 >= 0 && iw0 < cg.W) {
                    uint32_t lo[2], hi[2];
                    CvElem<E>::convert(xreg[n][0], lo);
                    CvElem<E>::convert(xreg[n][1], hi);
                    o = u32x4{lo[0], lo[1], hi[0], hi[1]};
                }
                *reinterpret_cast<u32x4 *>(lds_x + (row * kCvPX + v * 8) * 2) = o;
            }
        }
    };

    const int half = lane >> 5, l32 = lane & 31;
    // LDS element i of a staged input row is input column seg*128 - 8 + i; output column k of the segment meets,
    // for tap kw, element k + kw - pw + 8.  The six-word window starts at the even element k + 8 - pw - (pw & 1).
    const int win0 = 8 - cg.pw - (PODD ? 1 : 0);
    auto compute_stage = [&](int st) {
        const int seg = st % nseg;
        const int segw = min(kCvSeg, cg.OW - seg * kCvSeg);
        const int nks = (segw + 15) >> 4;
        for (int ks = 0; ks < nks; ++ks) {
            const int k0 = ks * 16 + half * 8;
            u32x4 afr[C::TM];
#pragma unroll
            for (int i = 0; i < C::TM; ++i)
                afr[i] = *reinterpret_cast<const u32x4 *>(lds_a + ((wm * 32 * C::TM + i * 32 + l32) * kCvPA + k0) * 2);
#pragma unroll
            for (int a = 0; a < C::XR; ++a) {
                if (a < KH) {
#pragma unroll
                    for (int j = 0; j < C::TN; ++j) {
                        const int row = a * C::CIT + wn * 32 * C::TN + j * 32 + l32;
                        const uint32_t *w = reinterpret_cast<const uint32_t *>(lds_x + (row * kCvPX + k0 + win0) * 2);
                        uint32_t D[6];
                        constexpr int NW = (C::XC > 1) ? 6 : 5;
#pragma unroll
                        for (int d = 0; d < NW; ++d) D[d] = w[d];
#pragma unroll
                        for (int c = 0; c < C::XC; ++c) {
                            if (c < KW) {
                                const int r = (PODD ? 1 : 0) + c;         // the window's offset from its first element
                                const int q = r >> 1;
                                u32x4 bfr;
                                if (r & 1) {
#pragma unroll
                                    for (int k = 0; k < 4; ++k) bfr[k] = __builtin_amdgcn_alignbyte(D[q + k + 1], D[q + k], 2);
                                } else {
#pragma unroll
                                    for (int k = 0; k < 4; ++k) bfr[k] = D[q + k];
                                }
#pragma unroll
                                for (int i = 0; i < C::TM; ++i) acc[i][j][a][c] = CvElem<E>::mfma(afr[i], bfr, acc[i][j][a][c]);
                            }
                        }
                    }
                }
            }
        }
    };

    if (st_begin < st_end) {
        load_stage(st_begin);
        store_stage(st_begin);
        __syncthreads();
        for (int st = st_begin; st < st_end; ++st) {
            const bool more = st + 1 < st_end;
            if (more) load_stage(st + 1);
            compute_stage(st);
            __syncthreads();          // every wave is done reading this stage
            if (more) store_stage(st + 1);
            __syncthreads();
        }
    }

    // lane l, register v of a 32x32 tile -> row (output channel) 8*(v/4) + 4*(l/32) + v%4, column (input channel) l%32
    const int ntap = KH * KW;
#pragma unroll
    for (int a = 0; a < C::XR; ++a)
#pragma unroll
        for (int c = 0; c < C::XC; ++c) {
            if (a < KH && c < KW) {
                float *P = part + (int64_t(split) * ntap + (a * KW + c)) * cg.Cout * cg.Cin;
#pragma unroll
                for (int i = 0; i < C::TM; ++i)
#pragma unroll
                    for (int j = 0; j < C::TN; ++j) {
                        const int ci = ci0 + wn * 32 * C::TN + j * 32 + l32;
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int co = co0 + wm * 32 * C::TM + i * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
                            if (co < cg.Cout && ci < cg.Cin) P[int64_t(co) * cg.Cin + ci] = acc[i][j][a][c][v];
                        }
                    }
            }
        }
}

// V[part][co][tap] = sum of dy[b,co,oh,ow] over the part's images and the outputs whose tap (kh, kw) lies inside the
// input image; tap index KH*KW holds the plain sum (the bias gradient).  One workgroup per (output channel, part);
// stride_w = dil_w = 1 and OW % 8 == 0 as in the kernel above.  Fixed summation order.
template <typename E>
__global__ __launch_bounds__(kCvThreads) void k_conv_valid_sums(const E *__restrict__ dy, ConvGeom cg, int parts, int imgs_per_part,
                                                                float *__restrict__ V)
{
    __shared__ float red[kCvThreads / 64][10];
    const int co = blockIdx.x / parts, pt = blockIdx.x - co * parts;
    const int b0 = pt * imgs_per_part, b1 = min(b0 + imgs_per_part, cg.B);
    const int vec_per_row = cg.OW >> 3;
    const int vec_per_img = cg.OH * vec_per_row;
    float acc[3][3], tot = 0.0f;
#pragma unroll
    for (int a = 0; a < 3; ++a)
#pragma unroll
        for (int c = 0; c < 3; ++c) acc[a][c] = 0.0f;
    for (int b = b0; b < b1; ++b) {
        const E *plane = dy + (int64_t(b) * cg.Cout + co) * cg.OH * cg.OW;
        for (int idx = threadIdx.x; idx < vec_per_img; idx += kCvThreads) {
            const int oh = idx / vec_per_row, ow0 = (idx - oh * vec_per_row) * 8;
            float f[8];
            Store<E>::unpack(*reinterpret_cast<const u32x4 *>(plane + int64_t(oh) * cg.OW + ow0), f);
            float cs[3] = {0.0f, 0.0f, 0.0f}, all = 0.0f;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                all += f[j];
#pragma unroll
                for (int c = 0; c < 3; ++c) {
                    const int iw = ow0 + j - cg.pw + c;
                    cs[c] += (c < cg.KW && iw >= 0 && iw < cg.W) ? f[j] : 0.0f;
                }
            }
            tot += all;
#pragma unroll
            for (int a = 0; a < 3; ++a) {
                const int ih = oh * cg.sh - cg.ph + a * cg.dh;
                if (a < cg.KH && ih >= 0 && ih < cg.H) {
#pragma unroll
                    for (int c = 0; c < 3; ++c) acc[a][c] += cs[c];
                }
            }
        }
    }
    float vals[10];
#pragma unroll
    for (int a = 0; a < 3; ++a)
#pragma unroll
        for (int c = 0; c < 3; ++c) vals[a * 3 + c] = acc[a][c];
    vals[9] = tot;
#pragma unroll
    for (int k = 0; k < 10; ++k) {
        float v = vals[k];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6][k] = v;
    }
    __syncthreads();
    if (threadIdx.x < 10) {
        float v = red[0][threadIdx.x];
#pragma unroll
        for (int w = 1; w < kCvThreads / 64; ++w) v += red[w][threadIdx.x];
        V[(int64_t(pt) * cg.Cout + co) * 10 + threadIdx.x] = v;
    }
}

// dW[co][ci][tap] = s_g(ci) * sum_splits part + (beta_g(ci) + centre * s_g(ci)) * sum_parts V[co][tap];  db = sum_parts V[co][plain]
__global__ __launch_bounds__(kCvThreads) void k_conv_finish(const float *__restrict__ part, const float *__restrict__ V, int splits,
                                                            int parts, ConvGeom cg, int per, const float *__restrict__ alpha,
                                                            const float *__restrict__ beta, float centre, float *__restrict__ dW,
                                                            float *__restrict__ db)
{
    const int64_t idx = int64_t(blockIdx.x) * kCvThreads + threadIdx.x;
    const int64_t plane = int64_t(cg.Cout) * cg.Cin;
    if (idx >= plane) return;
    const int co = int(idx / cg.Cin), ci = int(idx - int64_t(co) * cg.Cin);
    const int ntap = cg.KH * cg.KW;
    const int g = ci / per;
    const float sg = alpha[g] / 255.0f;
    const float off = fmaf(centre, sg, beta[g]);
    for (int a = 0; a < cg.KH; ++a)
        for (int c = 0; c < cg.KW; ++c) {
            const int tap = a * cg.KW + c;
            float s1 = 0.0f, v = 0.0f;
            for (int sp = 0; sp < splits; ++sp) s1 += part[(int64_t(sp) * ntap + tap) * plane + idx];
            for (int pt = 0; pt < parts; ++pt) v += V[(int64_t(pt) * cg.Cout + co) * 10 + a * 3 + c];
            dW[idx * ntap + tap] = fmaf(sg, s1, off * v);
        }
    if (db && ci == 0) {
        float v = 0.0f;
        for (int pt = 0; pt < parts; ++pt) v += V[(int64_t(pt) * cg.Cout + co) * 10 + 9];
        db[co] = v;
    }
}

// The plain path: any stride, dilation, kernel size and storage type.  One thread per element of dW, the whole sum in
// binary64 at the binary32 x_hat; threads of a workgroup share (co, ci-range) so that dy is read once per wave.
template <typename T>
__global__ __launch_bounds__(kCvThreads) void k_conv_dw_plain(const int8_t *__restrict__ xq, const void *__restrict__ dy, ConvGeom cg,
                                                              int per, const float *__restrict__ alpha, const float *__restrict__ beta,
                                                              float *__restrict__ dW, float *__restrict__ db)
{
    const int ntap = cg.KH * cg.KW;
    const int64_t per_co = int64_t(cg.Cin) * ntap;
    const int64_t idx = int64_t(blockIdx.x) * kCvThreads + threadIdx.x;
    if (idx >= per_co * cg.Cout) return;
    const int co = int(idx / per_co);
    const int rem = int(idx - int64_t(co) * per_co);
    const int ci = rem / ntap, tap = rem - ci * ntap;
    const int kh = tap / cg.KW, kw = tap - kh * cg.KW;
    const int g = ci / per;
    const float step = alpha[g] / 255.0f, off = beta[g];
    double acc = 0.0, tot = 0.0;
    const bool want_db = db && rem == 0;
    for (int b = 0; b < cg.B; ++b) {
        const int64_t dbase = (int64_t(b) * cg.Cout + co) * cg.OH * cg.OW;
        const int64_t xbase = (int64_t(b) * cg.Cin + ci) * cg.H * cg.W;
        for (int oh = 0; oh < cg.OH; ++oh) {
            const int ih = oh * cg.sh - cg.ph + kh * cg.dh;
            const bool row_in = ih >= 0 && ih < cg.H;
            if (!row_in && !want_db) continue;
            for (int ow = 0; ow < cg.OW; ++ow) {
                const float gy = Store<T>::load1(dy, dbase + int64_t(oh) * cg.OW + ow);
                if (want_db) tot += double(gy);
                const int iw = ow * cg.sw - cg.pw + kw * cg.dw;
                if (row_in && iw >= 0 && iw < cg.W) {
                    float xh = float(int(xq[xbase + int64_t(ih) * cg.W + iw]) + 128) * step;
                    xh = xh + off;
                    acc += double(gy) * double(xh);
                }
            }
        }
    }
    dW[idx] = float(acc);
    if (want_db) db[co] = float(tot);
}

struct CvPlan {
    bool fast, taps3;
    int tiles_co, tiles_ci, splits, stages_per_split, nseg, grid, parts, imgs_per_part;
};

static CvPlan cv_plan(const ConvGeom &cg, mesa_dtype dt)
{
    CvPlan p = {};
    p.fast = dt != MESA_F32 && cg.sw == 1 && cg.dw == 1 && cg.KH <= 3 && cg.KW <= 3 && cg.pw <= 8 && cg.W % 8 == 0 && cg.OW % 8 == 0;
    if (!p.fast) return p;
    p.taps3 = cg.KH * cg.KW > 1;
    const int cot = p.taps3 ? 64 : 128, cit = p.taps3 ? 64 : 128;
    p.tiles_co = int(ceil_div(cg.Cout, cot));
    p.tiles_ci = int(ceil_div(cg.Cin, cit));
    p.nseg = int(ceil_div(cg.OW, kCvSeg));
    const int64_t nstages = int64_t(cg.B) * cg.OH * p.nseg;
    const int64_t tiles = int64_t(p.tiles_co) * p.tiles_ci;
    // about two workgroups per CU over the launch, slices of at least eight stages, at most 64 slices
    int64_t splits = ceil_div(512, tiles);
    if (splits > 64) splits = 64;
    if (splits > ceil_div(nstages, 8)) splits = ceil_div(nstages, 8);
    if (splits < 1) splits = 1;
    p.stages_per_split = int(ceil_div(nstages, splits));
    p.splits = int(ceil_div(nstages, p.stages_per_split));
    p.grid = int(ceil_div(tiles * p.splits, kCvXcd) * kCvXcd);
    // the sums of dy: enough workgroups to cover the chip when there are few output channels
    int64_t parts = ceil_div(1024, cg.Cout);
    if (parts > cg.B) parts = cg.B;
    if (parts < 1) parts = 1;
    p.imgs_per_part = int(ceil_div(cg.B, parts));
    p.parts = int(ceil_div(cg.B, p.imgs_per_part));
    return p;
}

static bool cv_geom(const mesa_conv2d &cv, ConvGeom &cg)
{
    const int64_t lim = int64_t(1) << 30;
    const int64_t f[13] = {cv.B, cv.C_in, cv.H, cv.W, cv.C_out, cv.KH, cv.KW, cv.stride_h, cv.stride_w, cv.pad_h, cv.pad_w,
                           cv.dil_h, cv.dil_w};
    for (int i = 0; i < 13; ++i)
        if (f[i] < 0 || f[i] >= lim) return false;
    if (cv.C_in < 1 || cv.H < 1 || cv.W < 1 || cv.C_out < 1 || cv.KH < 1 || cv.KW < 1 || cv.stride_h < 1 || cv.stride_w < 1 ||
        cv.dil_h < 1 || cv.dil_w < 1)
        return false;
    const int64_t span_h = cv.H + 2 * cv.pad_h - cv.dil_h * (cv.KH - 1) - 1;
    const int64_t span_w = cv.W + 2 * cv.pad_w - cv.dil_w * (cv.KW - 1) - 1;
    if (span_h < 0 || span_w < 0) return false;
    cg = ConvGeom{int(cv.B), int(cv.C_in), int(cv.H), int(cv.W), int(cv.C_out), int(cv.KH), int(cv.KW), int(cv.stride_h),
                  int(cv.stride_w), int(cv.pad_h), int(cv.pad_w), int(cv.dil_h), int(cv.dil_w), int(span_h / cv.stride_h + 1),
                  int(span_w / cv.stride_w + 1)};
    return true;
}

// the sizes whose products index 32-bit quantities in the kernels
static bool cv_supported(const ConvGeom &cg)
{
    const int64_t lim = int64_t(1) << 31;
    if (int64_t(cg.Cout) * cg.Cin * cg.KH * cg.KW >= lim) return false;
    if (int64_t(cg.OH) * cg.OW >= lim || int64_t(cg.H) * cg.W >= lim) return false;
    if (int64_t(cg.B) * cg.OH * ceil_div(cg.OW, kCvSeg) >= lim) return false;
    if (int64_t(cg.sh) * cg.OH + int64_t(cg.dh) * cg.KH + cg.ph >= lim) return false;
    if (int64_t(cg.sw) * cg.OW + int64_t(cg.dw) * cg.KW + cg.pw >= lim) return false;
    return true;
}

static size_t cv_ws_bytes(const ConvGeom &cg, const CvPlan &p)
{
    if (!p.fast) return 0;
    const size_t part = size_t(p.splits) * cg.KH * cg.KW * cg.Cout * cg.Cin * sizeof(float);
    const size_t v = size_t(p.parts) * cg.Cout * 10 * sizeof(float);
    return part + ((v + 255) & ~size_t(255));
}

}  // namespace mesa

using namespace mesa;

extern "C" MESA_EXPORT size_t mesa_conv2d_dw_q_workspace_bytes(mesa_conv2d cv, mesa_dtype dt)
{
    ConvGeom cg;
    if (!valid_dtype(dt) || !cv_geom(cv, cg) || !cv_supported(cg) || cv.B == 0) return 0;
    return cv_ws_bytes(cg, cv_plan(cg, dt));
}

extern "C" MESA_EXPORT mesa_status mesa_conv2d_dw_q(const int8_t *xq, mesa_conv2d cv, int64_t G, const float *alpha, const float *beta,
                                                    const void *dy, mesa_dtype dt, float *dW, float *db, void *ws, size_t ws_bytes,
                                                    void *stream)
{
    ConvGeom cg;
    if (!valid_dtype(dt) || !cv_geom(cv, cg) || G < 1 || cv.C_in % G != 0) return MESA_ERR_INVALID_ARG;
    if (!cv_supported(cg)) return MESA_ERR_UNSUPPORTED;
    if (!dW || !alpha || !beta || !aligned16(dW) || !aligned4(alpha) || !aligned4(beta) || (db && !aligned4(db)))
        return MESA_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int per = int(cv.C_in / G);
    const int64_t nout = int64_t(cg.Cout) * cg.Cin * cg.KH * cg.KW;
    const int64_t plane = int64_t(cg.Cout) * cg.Cin;
    if (cg.B == 0) {   // an empty batch: the last kernel over no partial sums writes the zeros
        hipLaunchKernelGGL(k_conv_finish, dim3(unsigned(ceil_div(plane, kCvThreads))), dim3(kCvThreads), 0, s,
                           static_cast<const float *>(nullptr), static_cast<const float *>(nullptr), 0, 0, cg, per, alpha, beta, 0.0f,
                           dW, db);
        return launch_status();
    }
    if (!xq || !dy || !aligned16(xq) || !aligned16(dy)) return MESA_ERR_INVALID_ARG;
    const CvPlan p = cv_plan(cg, dt);
    if (!p.fast) {
        const unsigned grid = unsigned(ceil_div(nout, kCvThreads));
#define MESA_LAUNCH_CVP(T) \
        hipLaunchKernelGGL((k_conv_dw_plain<T>), dim3(grid), dim3(kCvThreads), 0, s, xq, dy, cg, per, alpha, beta, dW, db)
        MESA_FOR_DTYPE(dt, MESA_LAUNCH_CVP);
#undef MESA_LAUNCH_CVP
        return launch_status();
    }
    const size_t need = cv_ws_bytes(cg, p);
    if (!ws || ws_bytes < need || !aligned16(ws)) return MESA_ERR_WORKSPACE;
    float *part = static_cast<float *>(ws);
    const size_t part_bytes = size_t(p.splits) * cg.KH * cg.KW * cg.Cout * cg.Cin * sizeof(float);
    float *V = reinterpret_cast<float *>(static_cast<char *>(ws) + part_bytes);
    const bool podd = (cg.pw & 1) != 0;
#define MESA_LAUNCH_CV(E, T3, PO) \
    do { \
        auto kern = k_conv_dw<E, T3, PO>; \
        constexpr int lds = CvCfg<T3>::LDS; \
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess) \
            return MESA_ERR_LAUNCH; \
        hipLaunchKernelGGL(kern, dim3(p.grid), dim3(kCvThreads), lds, s, xq, static_cast<const E *>(dy), cg, p.tiles_co, p.tiles_ci, \
                           p.splits, p.stages_per_split, p.nseg, part); \
    } while (0)
#define MESA_PICK_CV(E) \
    do { \
        if (p.taps3) { if (podd) MESA_LAUNCH_CV(E, true, true); else MESA_LAUNCH_CV(E, true, false); } \
        else { if (podd) MESA_LAUNCH_CV(E, false, true); else MESA_LAUNCH_CV(E, false, false); } \
        hipLaunchKernelGGL((k_conv_valid_sums<E>), dim3(unsigned(cg.Cout) * p.parts), dim3(kCvThreads), 0, s, \
                           static_cast<const E *>(dy), cg, p.parts, p.imgs_per_part, V); \
    } while (0)
    float centre;
    if (dt == MESA_F16) { MESA_PICK_CV(_Float16); centre = CvElem<_Float16>::kCentre; }
    else { MESA_PICK_CV(__bf16); centre = CvElem<__bf16>::kCentre; }
#undef MESA_PICK_CV
#undef MESA_LAUNCH_CV
    if (launch_status() != MESA_OK) return MESA_ERR_LAUNCH;   // the last kernel must not read sums nobody wrote
    hipLaunchKernelGGL(k_conv_finish, dim3(unsigned(ceil_div(plane, kCvThreads))), dim3(kCvThreads), 0, s, part, V, p.splits, p.parts,
                       cg, per, alpha, beta, centre, dW, db);
    return launch_status();
}
