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
// input row, kw slides the eight-value window by one element.  One stage = one output row segment of up to 128
// columns: the dy rows of the workgroup's 128 output channels and ONE input row (the workgroup's kh) of its 64 input
// channels, converted once to 16-bit operands as they are written to LDS (pads as zeros).  A lane reads one aligned
// eight-element chunk per contraction step -- the middle tap's fragment as it lies; the outer taps need the last
// element of the chunk before and the first of the chunk after, which the other half of the wave holds one step
// earlier or later (ds_bpermute), then a byte alignment instruction per word.  Each of the three fragments feeds
// two MFMAs (the wave's two blocks of 32 output channels).  Slices of the (image, row, segment) range and the three
// kernel rows go to separate workgroups; the slices are combined in a fixed order by a second kernel.
//
// This path takes 16-bit tensors, 3x3 kernels with pad_w = 1 and 1x1 kernels with pad_w = 0, stride_w = dil_w = 1 (any
// row stride, dilation and padding) and widths of at least 8; anything else runs the plain kernel at the end of the file.
// Widths that are no multiples of 8 (RAG = 1): rows start at any element, so the eight-element vectors are loaded from
// unaligned addresses, and a row's last, partial vector is loaded from eight elements before the row's end instead (inside
// the row, hence inside the tensor) and written to LDS element by element where it belongs, zeros behind it.
// Widths below 8 (RAG = 2): a small kernel first copies both tensors to rows of eight elements; their one vector per row
// is loaded as it lies and the elements beyond the row's width are cleared on the way to LDS.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "api_util.hpp"
#include "common.hpp"

namespace mesa {

typedef _Float16 cv8h __attribute__((ext_vector_type(8)));
typedef __bf16 cv8b __attribute__((ext_vector_type(8)));
typedef float cv16f __attribute__((ext_vector_type(16)));

// W, OW: the row pitches of the tensors the kernels read, in elements; Wv, OWv: the columns of a row that exist (the same,
// except for maps narrower than eight columns, which the matrix-core path reads from copies with rows of eight)
struct ConvGeom {
    int B, Cin, H, W, Cout, KH, KW, sh, sw, ph, pw, dh, dw, OH, OW, Wv, OWv;
};

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

// T3 = true:  3x3 kernels with pad_w = 1; a workgroup owns 128 output x 64 input channels and ONE kernel row kh (the three
//              rows go to three workgroups: a third of the accumulators each, so that several workgroups share a CU and
//              one's staging and window shifts run while another's MFMAs do); a wave 64 x 32 channels for that row's
//              three taps (six accumulator tiles; every shifted fragment feeds two MFMAs).
// T3 = false: 1x1 kernels with pad_w = 0; a wave owns 64 x 64 channels (four tiles), the workgroup 128 x 128.
// NKS: contraction steps of 16 output columns per stage (a stage is a row segment of 16*NKS columns).
template <bool T3, int NKS> struct CvCfg {
    static constexpr int TM = 2, TN = T3 ? 1 : 2;
    static constexpr int XR = 1;                          // staged input rows: the one that the workgroup's kh meets
    static constexpr int COT = 64 * TM, CIT = 64 * TN;
    static constexpr int SEG = 16 * NKS;                  // output columns per stage
    static constexpr int NVA = 2 * NKS;                   // dy vectors (eight columns) per row
    static constexpr int NVX = T3 ? 2 * NKS + 2 : 2 * NKS;   // input vectors per row: T3 adds one vector of halo on either side
    // LDS pitches in elements: multiples of eight (16-byte rows), and such that eight rows' 16-byte reads start in
    // eight different groups of four banks
    static constexpr int PA = SEG + 8;
    static constexpr int PX = T3 ? SEG + 16 + (NKS == 1 ? 8 : 0) : SEG + 8;   // (a pitch of 32 elements would put every other row on the same banks)
    static constexpr int A_BYTES = COT * PA * 2;
    static constexpr int X_BYTES = XR * CIT * PX * 2;
    static constexpr int BUF = A_BYTES + X_BYTES;         // the stage buffer
    static constexpr int LDS = BUF;
    static constexpr int ND = COT * NVA / kCvThreads;     // dy vectors a thread stages
    static constexpr int NX = (XR * CIT * NVX + kCvThreads - 1) / kCvThreads;   // input vectors per thread
    static_assert(XR * CIT * NVX >= kCvThreads, "the ragged round wraps around once");
    static_assert(COT * NVA % kCvThreads == 0, "every thread stages the same number of dy vectors");
    static_assert(2 * LDS <= 160 * 1024, "two workgroups must fit the LDS of a CU");
};

// part[split][tap][co][ci] = sum over the split's (b, oh, segment) stages of dy * u,  tap = kh*KW + kw.
// One LDS stage buffer per workgroup and two or three workgroups per CU: the next stage's vectors are requested before a
// stage is multiplied, and converted and written to LDS after it (a barrier on either side) -- while one workgroup does
// that, the others' MFMAs keep the matrix cores busy.  (With one wave per SIMD the vector instructions of a stage and its
// MFMAs took turns instead of overlapping: 31 % matrix-core time.)
template <typename V> __device__ __forceinline__ V cv_load_unaligned(const char *p)
{
    V v;
    __builtin_memcpy(&v, p, sizeof(V));
    return v;
}

template <typename E, bool T3, int NKS, int RAG>
__global__ __launch_bounds__(kCvThreads, 2) void k_conv_dw(const int8_t *__restrict__ xq, const E *__restrict__ dy, ConvGeom cg,
                                                           int tiles_co, int tiles_ci, int splits, int stages_per_split,
                                                           int nseg, float *__restrict__ part)
{
    using C = CvCfg<T3, NKS>;
    extern __shared__ __attribute__((aligned(16))) unsigned char cv_lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int total = gridDim.x;
    // workgroups that share a slice of the stages run on the same XCD (same L2)
    const int logical = int(blockIdx.x % kCvXcd) * (total / kCvXcd) + int(blockIdx.x / kCvXcd);
    constexpr int NKH = T3 ? 3 : 1;                       // kernel rows, one workgroup each (neighbours: they share dy in L2)
    const int ntiles = tiles_co * tiles_ci;
    if (logical >= ntiles * splits * NKH) return;
    const int kh_w = logical % NKH;
    const int lt = logical / NKH;
    const int split = lt / ntiles;
    const int t = lt - split * ntiles;
    const int tco = t / tiles_ci, tci = t - tco * tiles_ci;
    const int co0 = tco * C::COT, ci0 = tci * C::CIT;
    const int wm = wave >> 1, wn = wave & 1;
    const int nstages = cg.B * cg.OH * nseg;
    const int st_begin = split * stages_per_split;
    const int st_end = min(st_begin + stages_per_split, nstages);
    constexpr int KH = 1, KW = T3 ? 3 : 1;               // taps of this workgroup: one kernel row

    cv16f acc[C::TM][C::TN][KH][KW];
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
#pragma unroll
        for (int j = 0; j < C::TN; ++j)
#pragma unroll
            for (int a = 0; a < KH; ++a)
#pragma unroll
                for (int b = 0; b < KW; ++b)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[i][j][a][b][v] = 0.0f;

    // What a thread stages, fixed for the whole kernel.  Input vector n of the thread: row (kh, channel) and vector v
    // of that row -> its place in LDS, its offset in the tensor relative to the stage's origin, and kh, v for the
    // in-image tests.  LDS element i of a staged input row is input column seg0 - 8 + i (T3) resp. seg0 + i.
    // xlds: its place in a stage buffer; xoff: its byte offset from the first byte of (image b, channel ci0); xbits: bit v
    // and bit 24 + kh, to be tested against the stage's valid vectors and rows (bit 31, never valid, marks a vector that
    // does not exist or a channel beyond C_in).
    int xlds[C::NX], xoff[C::NX];
    uint32_t xbits[C::NX];
#pragma unroll
    for (int n = 0; n < C::NX; ++n) {
        // the threads that the last, ragged round of vectors leaves without one stage one of the first vectors a second
        // time (same bytes to the same place), so that no load or store of the stage loop is conditional
        constexpr int kXVecs = C::XR * C::CIT * C::NVX;
        const int idx = tid + n * kCvThreads < kXVecs ? tid + n * kCvThreads : tid + n * kCvThreads - kXVecs;
        const int row = idx / C::NVX, v = idx - row * C::NVX;
        const int kh = row / C::CIT, cl = row - kh * C::CIT;
        const bool ok = ci0 + cl < cg.Cin;
        xlds[n] = C::A_BYTES + (row * C::PX + v * 8) * 2;
        xoff[n] = cl * cg.H * cg.W + v * 8;
        xbits[n] = ok ? (1u << v) | (1u << (24 + kh)) : 0x80000000u;
    }
    int dlds[C::ND], doff[C::ND];
    uint32_t dbits[C::ND];
#pragma unroll
    for (int n = 0; n < C::ND; ++n) {
        const int idx = tid + n * kCvThreads;
        const int row = idx / C::NVA, v = idx - row * C::NVA;
        dlds[n] = (row * C::PA + v * 8) * 2;
        doff[n] = (row * cg.OH * cg.OW + v * 8) * 2;
        dbits[n] = co0 + row < cg.Cout ? 1u << v : 0x80000000u;
    }

    u32x4 dreg[1][C::ND];
    u32x2 xreg[1][C::NX];
    uint32_t xkeep[1] = {0u};       // bit n: input vector n lies inside the image (elsewhere the forward saw padding: zeros)
    uint32_t dkeep[1] = {0u};
    // RAG: bit n: vector n is its row's partial last vector, loaded `shift` elements early (shift = 8 - its valid elements,
    // the same for every row of a stage)
    uint32_t xtail[1] = {0u}, dtail[1] = {0u};
    int xshift[1] = {0}, dshift[1] = {0};

    // the coordinates of the stage being loaded, advanced one stage at a time
    int seg = st_begin % nseg;
    int oh = (st_begin / nseg) % cg.OH;
    int b = (st_begin / nseg) / cg.OH;
    auto advance = [&]() {
        if (++seg == nseg) {
            seg = 0;
            if (++oh == cg.OH) { oh = 0; ++b; }
        }
    };
    // Loads are unconditional and their addresses a uniform base plus a 32-bit offset per lane: a vector outside its
    // tensor is fetched from offset zero instead and masked to zero when it is written to LDS (bit n of dkeep / xkeep),
    // so the stage loop has no divergent branches.
    auto load_stage = [&](auto set_tag) {   // the stage at (b, oh, seg) into register set S
        constexpr int S = decltype(set_tag)::value;
        const int seg0 = seg * C::SEG;
        const char *dbase = reinterpret_cast<const char *>(dy + (int64_t(b) * cg.Cout + co0) * cg.OH * cg.OW);
        const int ddelta = (oh * cg.OW + seg0) * 2;
        const int dfull = (cg.OWv - seg0) >> 3, dr = RAG ? (cg.OWv - seg0) & 7 : 0;
        const int dv_end = dfull + (dr ? 1 : 0);                      // vectors of this row that lie inside it, or partly so
        const uint32_t dtail_bit = (dr && dfull < C::NVA) ? 1u << dfull : 0u;
        dshift[S] = 8 - dr;
        dtail[S] = 0u;
        // (never bit 31: it marks the rows beyond C_out, which must fail the test below whatever the row's length)
        const uint32_t dmask = dv_end >= 31 ? 0x7FFFFFFFu : (1u << dv_end) - 1u;
        dkeep[S] = 0u;
#pragma unroll
        for (int n = 0; n < C::ND; ++n) {
            const bool in = (dbits[n] & dmask) == dbits[n];
            if (RAG == 1) {
                const bool tail = in && dbits[n] == dtail_bit;
                dreg[S][n] = cv_load_unaligned<u32x4>(dbase + uint32_t(in ? doff[n] + ddelta - (tail ? (8 - dr) * 2 : 0) : 0));
                dtail[S] |= tail ? 1u << n : 0u;
            } else {
                dreg[S][n] = *reinterpret_cast<const u32x4 *>(dbase + uint32_t(in ? doff[n] + ddelta : 0));
                if (RAG == 2) dtail[S] |= (in && dbits[n] == dtail_bit) ? 1u << n : 0u;
            }
            dkeep[S] |= in ? 1u << n : 0u;
        }
        const int ih0 = oh * cg.sh - cg.ph + kh_w * cg.dh;
        const char *xbase = reinterpret_cast<const char *>(xq + (int64_t(b) * cg.Cin + ci0) * cg.H * cg.W);
        const int xdelta = ih0 * cg.W + seg0 - (T3 ? 8 : 0);
        uint32_t smask = 0u;                                          // rows, then vectors, of this stage that lie in the image
#pragma unroll
        for (int a = 0; a < C::XR; ++a) {
            const int ih = ih0 + a * cg.dh;
            smask |= (ih >= 0 && ih < cg.H) ? 1u << (24 + a) : 0u;
        }
        const int v_lo = (T3 && seg0 == 0) ? 1 : 0;                   // the left halo of the first segment is padding
        const int xcols = cg.Wv - seg0 + (T3 ? 8 : 0);                // from LDS element 0 of the row to the image's last column
        const int xfull = xcols >> 3, xr = RAG ? xcols & 7 : 0;
        const int v_end = min(xfull + (xr ? 1 : 0), 24);
        const uint32_t xtail_bit = (xr && xfull < C::NVX) ? 1u << xfull : 0u;
        xshift[S] = 8 - xr;
        xtail[S] = 0u;
        smask |= ((1u << v_end) - 1u) & ~((1u << v_lo) - 1u);
        xkeep[S] = 0u;
#pragma unroll
        for (int n = 0; n < C::NX; ++n) {
            const bool in = (xbits[n] & smask) == xbits[n];
            if (RAG == 1) {
                const bool tail = in && (xbits[n] & 0x00FFFFFFu) == xtail_bit;
                xreg[S][n] = cv_load_unaligned<u32x2>(xbase + uint32_t(in ? xoff[n] + xdelta - (tail ? 8 - xr : 0) : 0));
                xtail[S] |= tail ? 1u << n : 0u;
            } else {
                xreg[S][n] = *reinterpret_cast<const u32x2 *>(xbase + uint32_t(in ? xoff[n] + xdelta : 0));
                if (RAG == 2) xtail[S] |= (in && (xbits[n] & 0x00FFFFFFu) == xtail_bit) ? 1u << n : 0u;
            }
            xkeep[S] |= in ? 1u << n : 0u;
        }
    };
    // a vector that was loaded `shift` elements early: its last 8 - shift elements to the first slots, zeros behind them
    // (the same thread's writes to LDS take effect in program order)
    auto store_tail = [&](unsigned char *at, u32x4 w, int shift) __attribute__((always_inline)) {
        *reinterpret_cast<u32x4 *>(at) = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 1; i < 8; ++i)
            if (i >= shift) *reinterpret_cast<uint16_t *>(at + (i - shift) * 2) = uint16_t(w[i >> 1] >> ((i & 1) * 16));
    };
    // a partial vector that lies where it belongs (rows of eight): its first 8 - shift elements, zeros behind them
    auto store_head = [&](unsigned char *at, u32x4 w, int shift) __attribute__((always_inline)) {
        const int r = 8 - shift;
#pragma unroll
        for (int k = 0; k < 4; ++k) w[k] &= (2 * k < r ? 0x0000FFFFu : 0u) | (2 * k + 1 < r ? 0xFFFF0000u : 0u);
        *reinterpret_cast<u32x4 *>(at) = w;
    };
    auto store_d = [&](int S, int n, unsigned char *buf) __attribute__((always_inline)) {
        const uint32_t k = 0u - ((dkeep[S] >> n) & 1u);
        const u32x4 w = u32x4{dreg[S][n][0] & k, dreg[S][n][1] & k, dreg[S][n][2] & k, dreg[S][n][3] & k};
        if (RAG == 1 && ((dtail[S] >> n) & 1u)) store_tail(buf + dlds[n], w, dshift[S]);
        else if (RAG == 2 && ((dtail[S] >> n) & 1u)) store_head(buf + dlds[n], w, dshift[S]);
        else *reinterpret_cast<u32x4 *>(buf + dlds[n]) = w;
    };
    auto store_x = [&](int S, int n, unsigned char *buf) __attribute__((always_inline)) {
        uint32_t lo[2], hi[2];
        CvElem<E>::convert(xreg[S][n][0], lo);
        CvElem<E>::convert(xreg[S][n][1], hi);
        const uint32_t k = 0u - ((xkeep[S] >> n) & 1u);
        const u32x4 w = u32x4{lo[0] & k, lo[1] & k, hi[0] & k, hi[1] & k};
        if (RAG == 1 && ((xtail[S] >> n) & 1u)) store_tail(buf + xlds[n], w, xshift[S]);
        else if (RAG == 2 && ((xtail[S] >> n) & 1u)) store_head(buf + xlds[n], w, xshift[S]);
        else *reinterpret_cast<u32x4 *>(buf + xlds[n]) = w;
    };

    const int half = lane >> 5, l32 = lane & 31;
    auto compute_stage = [&](const unsigned char *cur) {
        const unsigned char *xa = cur + C::A_BYTES;
        // T3: chunk c of a row holds input columns seg0 - 8 + 8c ..; output columns k..k+7 (k = 16ks + 8*half) meet, for
        // the taps kw = 0, 1, 2, the elements k+7.., k+8.., k+9..: the middle tap is chunk 2ks + half + 1 as it lies,
        // the outer two also need the last element of the chunk before and the first of the chunk after -- which the
        // other half of the wave holds (one step earlier or later), so each lane reads one chunk per row and step
        // and the halves exchange two words.
        // Every LDS value is requested at least one whole step before it is used: chunk j is read in step j - 3, its two
        // outer words are exchanged in step j - 2 (indices below are j + 1, j = -1 .. NKS).
        u32x4 Cc[KH][NKS + 2];
        uint32_t X0[KH][NKS + 2], X3[KH][NKS + 2];
        // chunk c of (kh row a, channel tile j) for this lane: a per-lane row address plus a constant
        const unsigned char *xrow[KH][C::TN];
#pragma unroll
        for (int a = 0; a < KH; ++a)
#pragma unroll
            for (int j = 0; j < C::TN; ++j) xrow[a][j] = xa + ((a * C::CIT + wn * 32 * C::TN + j * 32 + l32) * C::PX + half * 8) * 2;
        // T3: the step's chunk is 2ks + half + 1.  The reads before the first step and after the last one matter for
        // one half of the wave only; the other half reads the same chunk (inside the row) and its value is never used.
        auto chunk_addr = [&](int a, int j, int ks) {
            if (!T3) return xrow[a][j] + ks * 32;
            if (ks < 0) return xrow[a][j] - half * 16 + 0;                    // chunk 0 for both halves
            if (ks >= NKS) return xrow[a][j] - half * 16 + (2 * NKS + 1) * 16;   // the last chunk for both halves
            return xrow[a][j] + (2 * ks + 1) * 16;
        };
        static_assert(!T3 || C::TN == 1, "the exchange below is written for one input-channel tile per wave");
        auto rd = [&](int a, int jj) { Cc[a][jj + 1] = *reinterpret_cast<const u32x4 *>(chunk_addr(a, 0, jj)); };
        auto ex = [&](int a, int jj) {
            X0[a][jj + 1] = __shfl_xor(Cc[a][jj + 1][0], 32, 64);
            X3[a][jj + 1] = __shfl_xor(Cc[a][jj + 1][3], 32, 64);
        };
        u32x4 anext[C::TM], bnext[C::TN];
#pragma unroll
        for (int i = 0; i < C::TM; ++i)
            anext[i] = *reinterpret_cast<const u32x4 *>(cur + ((wm * 32 * C::TM + i * 32 + l32) * C::PA + half * 8) * 2);
        if (T3) {
#pragma unroll
            for (int a = 0; a < KH; ++a) { rd(a, -1); rd(a, 0); rd(a, 1); }
#pragma unroll
            for (int a = 0; a < KH; ++a) { ex(a, -1); ex(a, 0); ex(a, 1); }
#pragma unroll
            for (int a = 0; a < KH; ++a)
                if (2 <= NKS) rd(a, 2);
        } else {
#pragma unroll
            for (int j = 0; j < C::TN; ++j) bnext[j] = *reinterpret_cast<const u32x4 *>(chunk_addr(0, j, 0));
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            u32x4 afr[C::TM];
#pragma unroll
            for (int i = 0; i < C::TM; ++i) {
                afr[i] = anext[i];
                if (ks + 1 < NKS)
                    anext[i] = *reinterpret_cast<const u32x4 *>(cur + ((wm * 32 * C::TM + i * 32 + l32) * C::PA + (ks + 1) * 16 + half * 8) * 2);
            }
            if (T3) {
#pragma unroll
                for (int a = 0; a < KH; ++a)
                    if (ks + 3 <= NKS) rd(a, ks + 3);
#pragma unroll
                for (int a = 0; a < KH; ++a)
                    if (ks + 2 <= NKS) ex(a, ks + 2);
#pragma unroll
                for (int a = 0; a < KH; ++a) {
                    const u32x4 c1 = Cc[a][ks + 1];
                    // lower half: before = the other half's chunk of the previous step, after = its chunk of this step;
                    // upper half: before = the other half's chunk of this step, after = its chunk of the next step
                    const uint32_t before = half ? X3[a][ks + 1] : X3[a][ks];
                    const uint32_t after = half ? X0[a][ks + 2] : X0[a][ks + 1];
                    u32x4 f0, f2;
                    f0[0] = __builtin_amdgcn_alignbyte(c1[0], before, 2);
                    f0[1] = __builtin_amdgcn_alignbyte(c1[1], c1[0], 2);
                    f0[2] = __builtin_amdgcn_alignbyte(c1[2], c1[1], 2);
                    f0[3] = __builtin_amdgcn_alignbyte(c1[3], c1[2], 2);
                    f2[0] = __builtin_amdgcn_alignbyte(c1[1], c1[0], 2);
                    f2[1] = __builtin_amdgcn_alignbyte(c1[2], c1[1], 2);
                    f2[2] = __builtin_amdgcn_alignbyte(c1[3], c1[2], 2);
                    f2[3] = __builtin_amdgcn_alignbyte(after, c1[3], 2);
#pragma unroll
                    for (int i = 0; i < C::TM; ++i) {
                        acc[i][0][a][0] = CvElem<E>::mfma(afr[i], f0, acc[i][0][a][0]);
                        acc[i][0][a][KW > 1 ? 1 : 0] = CvElem<E>::mfma(afr[i], c1, acc[i][0][a][KW > 1 ? 1 : 0]);
                        acc[i][0][a][KW > 2 ? 2 : 0] = CvElem<E>::mfma(afr[i], f2, acc[i][0][a][KW > 2 ? 2 : 0]);
                    }
                }
            } else {
                u32x4 bfr[C::TN];
#pragma unroll
                for (int j = 0; j < C::TN; ++j) {
                    bfr[j] = bnext[j];
                    if (ks + 1 < NKS) bnext[j] = *reinterpret_cast<const u32x4 *>(chunk_addr(0, j, ks + 1));
                }
#pragma unroll
                for (int j = 0; j < C::TN; ++j)
#pragma unroll
                    for (int i = 0; i < C::TM; ++i) acc[i][j][0][0] = CvElem<E>::mfma(afr[i], bfr[j], acc[i][j][0][0]);
            }
            __builtin_amdgcn_sched_barrier(0);     // keep each step's reads and window shifts with its MFMAs
        }
    };

    if (st_begin < st_end) {
        auto store_all = [&]() __attribute__((always_inline)) {
#pragma unroll
            for (int n = 0; n < C::ND; ++n) store_d(0, n, cv_lds);
#pragma unroll
            for (int n = 0; n < C::NX; ++n) store_x(0, n, cv_lds);
        };
        load_stage(std::integral_constant<int, 0>());
        store_all();
        __syncthreads();
        // the last stage is peeled off so that the loop has a single path
        for (int st = st_begin; st + 1 < st_end; ++st) {
            advance();
            load_stage(std::integral_constant<int, 0>());   // in flight while this stage is multiplied
            compute_stage(cv_lds);
            __syncthreads();                                  // every wave is done reading this stage
            store_all();
            __syncthreads();
        }
        compute_stage(cv_lds);
    }

    // lane l, register v of a 32x32 tile -> row (output channel) 8*(v/4) + 4*(l/32) + v%4, column (input channel) l%32
    constexpr int ntap = NKH * KW;
#pragma unroll
    for (int a = 0; a < KH; ++a)
#pragma unroll
        for (int c = 0; c < KW; ++c) {
            float *P = part + (int64_t(split) * ntap + (kh_w * KW + c)) * cg.Cout * cg.Cin;
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

// V[part][co][tap] = sum of dy[b,co,oh,ow] over the part's images and the outputs whose tap (kh, kw) lies inside the
// input image; tap index KH*KW holds the plain sum (the bias gradient).  One workgroup per (output channel, part);
// stride_w = dil_w = 1 and OW % 8 == 0 as in the kernel above.  Fixed summation order.
template <typename E>
__global__ __launch_bounds__(kCvThreads) void k_conv_valid_sums(const E *__restrict__ dy, ConvGeom cg, int parts, int imgs_per_part,
                                                                int row_blocks, int rows_per_block, float *__restrict__ V)
{
    __shared__ float red[kCvThreads / 64][10];
    const int co = blockIdx.x / parts, pt = blockIdx.x - co * parts;
    const int ip = pt / row_blocks, rk = pt - ip * row_blocks;        // a part: some images, one block of their rows
    const int b0 = ip * imgs_per_part, b1 = min(b0 + imgs_per_part, cg.B);
    const int vec_per_row = cg.OW >> 3;
    const int v_begin = rk * rows_per_block * vec_per_row;
    const int v_end = min((rk + 1) * rows_per_block, cg.OH) * vec_per_row;
    float acc[3][3], tot = 0.0f;
#pragma unroll
    for (int a = 0; a < 3; ++a)
#pragma unroll
        for (int c = 0; c < 3; ++c) acc[a][c] = 0.0f;
    // the part's vectors, image after image, shared out among the threads (small maps: a part is several images of a few
    // vectors each); four vectors per thread and round, requested together
    const int vpi = v_end - v_begin;                          // vectors per image
    const int nv = (b1 - b0) * vpi;
    {
        for (int base = 0; base < nv; base += 4 * kCvThreads) {
            u32x4 raw[4];
            int at[4];                                        // the vector's index in its plane, -1: none
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int v = base + u * kCvThreads + int(threadIdx.x);
                raw[u] = u32x4{0u, 0u, 0u, 0u};
                at[u] = -1;
                if (v < nv) {
                    const int bi = v / vpi;
                    at[u] = v_begin + (v - bi * vpi);
                    const E *plane = dy + (int64_t(b0 + bi) * cg.Cout + co) * cg.OH * cg.OW;
                    raw[u] = *reinterpret_cast<const u32x4 *>(plane + int64_t(at[u]) * 8);
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int idx = at[u];
                if (idx < 0) continue;
                const int oh = idx / vec_per_row, ow0 = (idx - oh * vec_per_row) * 8;
                float f[8];
                Store<E>::unpack(raw[u], f);
                float cs[3] = {0.0f, 0.0f, 0.0f}, all = 0.0f;
#pragma unroll
                for (int j = 0; j < 8; ++j) all += f[j];
                if (ow0 - cg.pw >= 0 && ow0 + 7 - cg.pw + 2 < cg.Wv) {   // every tap of every element lies inside: all but a row's ends
#pragma unroll
                    for (int c = 0; c < 3; ++c) cs[c] = c < cg.KW ? all : 0.0f;
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j)
#pragma unroll
                        for (int c = 0; c < 3; ++c) {
                            const int iw = ow0 + j - cg.pw + c;
                            cs[c] += (c < cg.KW && iw >= 0 && iw < cg.Wv) ? f[j] : 0.0f;
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

// The same sums for widths that are no multiples of 8 (at least 8): a thread takes eight consecutive elements of the
// (image, channel) plane with one unaligned vector load -- they lie in one row, or in two with the row's end between them --,
// four such vectors requested together; the last, partial vector of a part element by element.
template <typename E>
__global__ __launch_bounds__(kCvThreads) void k_conv_valid_sums_any(const E *__restrict__ dy, ConvGeom cg, int parts, int imgs_per_part,
                                                                    int row_blocks, int rows_per_block, FastDiv div_ow,
                                                                    float *__restrict__ V)
{
    __shared__ float red[kCvThreads / 64][10];
    const int co = blockIdx.x / parts, pt = blockIdx.x - co * parts;
    const int ip = pt / row_blocks, rk = pt - ip * row_blocks;
    const int b0 = ip * imgs_per_part, b1 = min(b0 + imgs_per_part, cg.B);
    const int per_img = cg.OH * cg.OW;
    const int e_begin = rk * rows_per_block * cg.OW;
    const int e_end = min((rk + 1) * rows_per_block, cg.OH) * cg.OW;
    float acc[3][3], tot = 0.0f;
#pragma unroll
    for (int a = 0; a < 3; ++a)
#pragma unroll
        for (int c = 0; c < 3; ++c) acc[a][c] = 0.0f;
    // the part's vectors, image after image, shared out among the threads (small maps: a part is several images of a few
    // vectors each)
    const int vpi = (e_end - e_begin + 7) >> 3;               // vectors per image
    const int nv = (b1 - b0) * vpi;
    for (int base = 0; base < nv; base += 4 * kCvThreads) {
        u32x4 raw[4];
        int at[4];                                            // the vector's first element in its plane, -1: none
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int v = base + u * kCvThreads + int(threadIdx.x);
            raw[u] = u32x4{0u, 0u, 0u, 0u};
            at[u] = -1;
            if (v < nv) {
                const int bi = v / vpi, idx = e_begin + (v - bi * vpi) * 8;
                const E *plane = dy + (int64_t(b0 + bi) * cg.Cout + co) * per_img;
                at[u] = idx;
                if (idx + 8 <= e_end) {
                    raw[u] = cv_load_unaligned<u32x4>(reinterpret_cast<const char *>(plane + idx));
                } else {                                      // beyond the part there may be the end of the tensor
                    uint16_t h[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) h[j] = idx + j < e_end ? reinterpret_cast<const uint16_t *>(plane)[idx + j] : uint16_t(0);
#pragma unroll
                    for (int k = 0; k < 4; ++k) raw[u][k] = uint32_t(h[2 * k]) | (uint32_t(h[2 * k + 1]) << 16);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = at[u];
            if (idx < 0) continue;
            float f[8];
            Store<E>::unpack(raw[u], f);
            const int oh = int(fastdiv(uint32_t(idx), div_ow)), ow0 = idx - oh * cg.OW;
            // elements j < n0 lie in row oh, the others in row oh + 1 (OW >= 8: at most one row end inside a vector)
            const int n0 = cg.OW - ow0;
            float cs[2][3] = {{0.0f, 0.0f, 0.0f}, {0.0f, 0.0f, 0.0f}}, all[2] = {0.0f, 0.0f};
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const bool second = j >= n0;
                const int ow = second ? j - n0 : ow0 + j;
                all[0] += second ? 0.0f : f[j];
                all[1] += second ? f[j] : 0.0f;
#pragma unroll
                for (int c = 0; c < 3; ++c) {
                    const int iw = ow - cg.pw + c;
                    const float v = (c < cg.KW && iw >= 0 && iw < cg.Wv) ? f[j] : 0.0f;
                    cs[0][c] += second ? 0.0f : v;
                    cs[1][c] += second ? v : 0.0f;
                }
            }
            tot += all[0] + all[1];      // (zeros beyond the part's end)
#pragma unroll
            for (int r = 0; r < 2; ++r)
#pragma unroll
                for (int a = 0; a < 3; ++a) {
                    const int ih = (oh + r) * cg.sh - cg.ph + a * cg.dh;
                    if (a < cg.KH && ih >= 0 && ih < cg.H) {
#pragma unroll
                        for (int c = 0; c < 3; ++c) acc[a][c] += cs[r][c];
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
    // A thread owns one (co, ci) pair: its reads of a tap's plane are coalesced; its ntap results are consecutive in dW, so
    // the workgroup's 256 * ntap results go through LDS and leave as one contiguous run (up to nine taps; more only
    // occur with an empty batch, where plain strided stores of zeros will do).
    __shared__ float tile[kCvThreads * 9];
    const int64_t idx = int64_t(blockIdx.x) * kCvThreads + threadIdx.x;
    const int64_t plane = int64_t(cg.Cout) * cg.Cin;
    const int ntap = cg.KH * cg.KW;
    const bool staged = ntap <= 9;
    const bool live = idx < plane;
    if (live) {
        const int co = int(idx / cg.Cin), ci = int(idx - int64_t(co) * cg.Cin);
        const int g = ci / per;
        const float sg = alpha[g] / 255.0f;
        const float off = fmaf(centre, sg, beta[g]);
        if (staged) {       // the taps' sums side by side: nine loads in flight per slice instead of one
            float s1[9];
#pragma unroll
            for (int t = 0; t < 9; ++t) s1[t] = 0.0f;
            // the loads of several slices are requested together (the sums are still added slice by slice, in order): four
            // slices of nine taps (23 -> 17.5 us at 512 x 512 channels and five slices), eight slices of one tap; the two tap
            // counts of the matrix-core path as compile-time constants
            auto add_slices = [&](auto taps, auto batch) {
                constexpr int NT = decltype(taps)::value, NB = decltype(batch)::value;
                int sp = 0;
                for (; sp + NB <= splits; sp += NB) {
                    float v[NB][NT];
#pragma unroll
                    for (int k = 0; k < NB; ++k)
#pragma unroll
                        for (int t = 0; t < NT; ++t) v[k][t] = part[(int64_t(sp + k) * NT + t) * plane + idx];
#pragma unroll
                    for (int k = 0; k < NB; ++k)
#pragma unroll
                        for (int t = 0; t < NT; ++t) s1[t] += v[k][t];
                }
                for (; sp < splits; ++sp)
#pragma unroll
                    for (int t = 0; t < NT; ++t) s1[t] += part[(int64_t(sp) * NT + t) * plane + idx];
            };
            if (ntap == 9) add_slices(std::integral_constant<int, 9>(), std::integral_constant<int, 4>());
            else if (ntap == 1) add_slices(std::integral_constant<int, 1>(), std::integral_constant<int, 8>());
            else
                for (int sp = 0; sp < splits; ++sp)
#pragma unroll
                    for (int t = 0; t < 9; ++t)
                        if (t < ntap) s1[t] += part[(int64_t(sp) * ntap + t) * plane + idx];
#pragma unroll
            for (int t = 0; t < 9; ++t)
                if (t < ntap) {
                    const int a = t / cg.KW, c = t - a * cg.KW;
                    float v = 0.0f;
                    for (int pt = 0; pt < parts; ++pt) v += V[(int64_t(pt) * cg.Cout + co) * 10 + a * 3 + c];
                    tile[threadIdx.x * ntap + t] = splits == 0 ? 0.0f : fmaf(sg, s1[t], off * v);   // no slices: an empty batch
                }
        } else {
            for (int tap = 0; tap < ntap; ++tap) dW[idx * ntap + tap] = 0.0f;   // only reached with an empty batch
        }
        if (db && ci == 0) {
            float v = 0.0f;
            for (int pt = 0; pt < parts; ++pt) v += V[(int64_t(pt) * cg.Cout + co) * 10 + 9];
            db[co] = v;
        }
    }
    if (staged) {
        __syncthreads();
        const int64_t first = int64_t(blockIdx.x) * kCvThreads;
        const int64_t count = (plane - first < kCvThreads ? plane - first : kCvThreads) * ntap;
        for (int k = threadIdx.x; k < count; k += kCvThreads) dW[first * ntap + k] = tile[k];
    }
}

// The same for few channel pairs and many slices (narrow layers: 64 x 64 channels leave k_conv_finish 16 workgroups
// whose threads walk 64 slices of nine dependent loads each -- 150 us, six times the matrix-core kernel): a workgroup takes
// PW = 32 pairs (consecutive: a wave's loads of a slice are 128 contiguous bytes), SL threads share a pair's slices (every
// SL-th each, in order) and their sums are added in a fixed order; the sums of V for the workgroup's output channels are
// taken once, by its first threads.  SL * 32 threads.  ntap <= 9.
template <int SL>
__global__ __launch_bounds__(SL * 32) void k_conv_finish_few(const float *__restrict__ part, const float *__restrict__ V, int splits,
                                                                int parts, ConvGeom cg, int per, const float *__restrict__ alpha,
                                                                const float *__restrict__ beta, float centre, float *__restrict__ dW,
                                                                float *__restrict__ db)
{
    constexpr int PW = 32, NT = SL * PW;                   // pairs per workgroup, threads
    __shared__ float sums[SL][PW][9];
    __shared__ float vsum[PW][10];
    __shared__ float tile[PW * 9];
    const int pl = threadIdx.x % PW, sl = threadIdx.x / PW;
    const int64_t plane = int64_t(cg.Cout) * cg.Cin;
    const int64_t first = int64_t(blockIdx.x) * PW, idx = first + pl;
    const int ntap = cg.KH * cg.KW;
    const bool live = idx < plane;
    const int co_first = int(first / cg.Cin);              // the workgroup's pairs lie in the output channels from this one on
    const int64_t last = first + PW - 1 < plane ? first + PW - 1 : plane - 1;
    const int nco = int(last / cg.Cin) - co_first + 1;     // at most PW
    for (int k = threadIdx.x; k < nco * 10; k += NT) {
        const int c = k / 10, e = k - c * 10;
        float v = 0.0f;
        for (int pt = 0; pt < parts; ++pt) v += V[(int64_t(pt) * cg.Cout + co_first + c) * 10 + e];
        vsum[c][e] = v;
    }
    float s1[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) s1[t] = 0.0f;
    if (live)
        for (int sp = sl; sp < splits; sp += SL)
#pragma unroll
            for (int t = 0; t < 9; ++t)
                if (t < ntap) s1[t] += part[(int64_t(sp) * ntap + t) * plane + idx];
#pragma unroll
    for (int t = 0; t < 9; ++t) sums[sl][pl][t] = s1[t];
    __syncthreads();
    if (sl == 0 && live) {
        const int co = int(idx / cg.Cin), ci = int(idx - int64_t(co) * cg.Cin);
        const int g = ci / per;
        const float sg = alpha[g] / 255.0f;
        const float off = fmaf(centre, sg, beta[g]);
        const float *vs = vsum[co - co_first];
#pragma unroll
        for (int t = 0; t < 9; ++t)
            if (t < ntap) {
                float q[SL / 4];                           // groups of four in order, then the groups in order
#pragma unroll
                for (int k = 0; k < SL / 4; ++k)
                    q[k] = (sums[4 * k][pl][t] + sums[4 * k + 1][pl][t]) + (sums[4 * k + 2][pl][t] + sums[4 * k + 3][pl][t]);
                float tot = q[0];
#pragma unroll
                for (int k = 1; k < SL / 4; ++k) tot += q[k];
                const int a = t / cg.KW, c = t - a * cg.KW;
                tile[pl * ntap + t] = fmaf(sg, tot, off * vs[a * 3 + c]);
            }
        if (db && ci == 0) db[co] = vs[9];
    }
    __syncthreads();
    const int64_t count = (plane - first < PW ? plane - first : PW) * ntap;
    for (int k = threadIdx.x; k < count; k += NT) dW[first * ntap + k] = tile[k];
}

// Rows of w < 8 elements copied to rows of eight (zeros behind them): one thread per row.  V: a vector of eight elements.
template <typename Elem, typename V>
__global__ __launch_bounds__(kCvThreads) void k_conv_pad_rows(const Elem *__restrict__ in, Elem *__restrict__ out, int64_t rows, int w)
{
    const int64_t row = int64_t(blockIdx.x) * kCvThreads + threadIdx.x;
    if (row >= rows) return;
    union { Elem e[8]; V v; } u;
#pragma unroll
    for (int j = 0; j < 8; ++j) u.e[j] = j < w ? in[row * w + j] : Elem(0);
    *reinterpret_cast<V *>(out + row * 8) = u.v;
}

// The plain path: any stride, dilation, kernel size and storage type.  One workgroup per (output channel, input channel):
// its threads share out the output positions (consecutive threads, consecutive columns of dy), every thread keeps the
// kernel taps' sums -- nine taps at a time -- in binary64 at the binary32 x_hat, and the threads' sums are added in a
// fixed order (lanes, then waves).  Workgroups of input channel 0 also sum dy for the bias gradient.
constexpr int kCvPlainTaps = 9;
template <typename T>
__global__ __launch_bounds__(kCvThreads) void k_conv_dw_plain(const int8_t *__restrict__ xq, const void *__restrict__ dy, ConvGeom cg,
                                                              int per, const float *__restrict__ alpha, const float *__restrict__ beta,
                                                              float *__restrict__ dW, float *__restrict__ db)
{
    __shared__ double red[kCvThreads / 64][kCvPlainTaps + 1];
    const int ntap = cg.KH * cg.KW;
    const int co = int(blockIdx.x / unsigned(cg.Cin)), ci = int(blockIdx.x % unsigned(cg.Cin));
    const int g = ci / per;
    const float step = alpha[g] / 255.0f, off = beta[g];
    const int plane = cg.OH * cg.OW;                       // < 2^31 (checked by the entry point)
    const bool want_db = db && ci == 0;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int tap0 = 0; tap0 < ntap; tap0 += kCvPlainTaps) {
        int dih[kCvPlainTaps], diw[kCvPlainTaps];          // a tap's offset from (oh * sh, ow * sw)
#pragma unroll
        for (int t = 0; t < kCvPlainTaps; ++t) {
            const int tap = tap0 + t < ntap ? tap0 + t : tap0;
            const int kh = tap / cg.KW, kw = tap - kh * cg.KW;
            dih[t] = kh * cg.dh - cg.ph;
            diw[t] = kw * cg.dw - cg.pw;
        }
        double acc[kCvPlainTaps], tot = 0.0;
#pragma unroll
        for (int t = 0; t < kCvPlainTaps; ++t) acc[t] = 0.0;
        for (int b = 0; b < cg.B; ++b) {
            const int64_t dbase = (int64_t(b) * cg.Cout + co) * plane;
            const int8_t *xb = xq + (int64_t(b) * cg.Cin + ci) * cg.H * cg.W;
            for (int r = threadIdx.x; r < plane; r += kCvThreads) {
                const int oh = r / cg.OW, ow = r - oh * cg.OW;
                const float gy = Store<T>::load1(dy, dbase + r);
                tot += double(gy);
#pragma unroll
                for (int t = 0; t < kCvPlainTaps; ++t) {
                    const int ih = oh * cg.sh + dih[t], iw = ow * cg.sw + diw[t];
                    if (tap0 + t < ntap && ih >= 0 && ih < cg.H && iw >= 0 && iw < cg.W) {
                        float xh = float(int(xb[ih * cg.W + iw]) + 128) * step;     // H * W < 2^31 (checked by the entry point)
                        xh = xh + off;
                        acc[t] += double(gy) * double(xh);
                    }
                }
            }
        }
        // lanes, then waves, in a fixed order
#pragma unroll
        for (int t = 0; t <= kCvPlainTaps; ++t) {
            double v = t < kCvPlainTaps ? acc[t] : tot;
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m);
            if (lane == 0) red[wave][t] = v;
        }
        __syncthreads();
        if (threadIdx.x <= kCvPlainTaps) {
            const int t = threadIdx.x;
            const double v = (red[0][t] + red[1][t]) + (red[2][t] + red[3][t]);
            if (t < kCvPlainTaps) {
                if (tap0 + t < ntap) dW[(int64_t(co) * cg.Cin + ci) * ntap + tap0 + t] = float(v);
            } else if (want_db && tap0 == 0) {
                db[co] = float(v);
            }
        }
        __syncthreads();                                   // the next nine taps reuse `red`
    }
}

struct CvPlan {
    bool fast, taps3, rag, pad;     // rag: widths that are no multiples of 8; pad: below 8, read from copies with rows of eight
    int nks, tiles_co, tiles_ci, splits, stages_per_split, nseg, grid, parts, imgs_per_part, row_blocks, rows_per_block;
};

static CvPlan cv_plan(const ConvGeom &cg, mesa_dtype dt)
{
    CvPlan p = {};
    const bool k3 = cg.KH == 3 && cg.KW == 3 && cg.pw == 1, k1 = cg.KH == 1 && cg.KW == 1 && cg.pw == 0;
    // per-lane byte offsets inside a tile of 128 channels, plus the stage's own offset, stay below 2^31
    const int64_t lim = int64_t(1) << 22;
    p.pad = cg.W < 8 || cg.OW < 8;
    const int W = p.pad ? 8 : cg.W, OW = p.pad ? 8 : cg.OW;     // the row pitches the kernels see
    p.fast = dt != MESA_F32 && cg.sw == 1 && cg.dw == 1 && (k3 || k1) &&
             (int64_t(cg.H) + 2 * cg.ph + 3 * int64_t(cg.dh)) * W <= lim && int64_t(cg.OH) * OW <= lim;
    // (the copies' rows are shared out one per thread of a 32-bit grid)
    if (p.pad && (int64_t(cg.B) * cg.Cin * cg.H >= (int64_t(1) << 31) || int64_t(cg.B) * cg.Cout * cg.OH >= (int64_t(1) << 31))) p.fast = false;
    if (!p.fast) return p;
    p.taps3 = k3;
    p.rag = !p.pad && (cg.W % 8 != 0 || cg.OW % 8 != 0);
    p.nks = OW <= 16 ? 1 : OW <= 32 ? 2 : OW <= 64 ? 4 : 8;
    const int cot = 128, cit = p.taps3 ? 64 : 128;
    p.tiles_co = int(ceil_div(cg.Cout, cot));
    p.tiles_ci = int(ceil_div(cg.Cin, cit));
    p.nseg = int(ceil_div(OW, 16 * p.nks));
    const int64_t nstages = int64_t(cg.B) * cg.OH * p.nseg;
    const int64_t tiles = int64_t(p.tiles_co) * p.tiles_ci * (p.taps3 ? 3 : 1);
    // two workgroups per CU: as many slices as fill one such round of the chip without starting a second (a round and
    // an eighth costs two rounds); slices of at least eight stages, at most 64 slices
    int64_t splits = 512 / tiles;
    if (splits > 64) splits = 64;
    if (splits > ceil_div(nstages, 8)) splits = ceil_div(nstages, 8);
    if (splits < 1) splits = 1;
    p.stages_per_split = int(ceil_div(nstages, splits));
    p.splits = int(ceil_div(nstages, p.stages_per_split));
    p.grid = int(ceil_div(tiles * p.splits, kCvXcd) * kCvXcd);
    // the sums of dy: enough workgroups to cover the chip when there are few output channels
    // (a part is a run of images, or -- with fewer images than parts wanted -- a block of rows of one image, 8192 elements or more;
    // at most 32 parts: the last kernel adds them up per output channel)
    int64_t want = ceil_div(2048, cg.Cout);
    if (want > 32) want = 32;
    int64_t img_parts = want < cg.B ? want : cg.B;
    if (img_parts < 1) img_parts = 1;
    p.imgs_per_part = int(ceil_div(cg.B, img_parts));
    img_parts = ceil_div(cg.B, p.imgs_per_part);
    int64_t rb = 1;
    if (img_parts < want) {
        rb = ceil_div(want, img_parts);
        if (rb > ceil_div(cg.OH, 8)) rb = ceil_div(cg.OH, 8);
        const int64_t by_size = int64_t(cg.OH) * OW / 8192;       // a block keeps every thread at least four vectors
        if (rb > by_size) rb = by_size < 1 ? 1 : by_size;
    }
    p.rows_per_block = int(ceil_div(cg.OH, rb));
    p.row_blocks = int(ceil_div(cg.OH, p.rows_per_block));
    p.parts = int(img_parts) * p.row_blocks;
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
                  int(span_w / cv.stride_w + 1), int(cv.W), int(span_w / cv.stride_w + 1)};
    return true;
}

// the sizes whose products index 32-bit quantities in the kernels
static bool cv_supported(const ConvGeom &cg)
{
    const int64_t lim = int64_t(1) << 31;
    if (int64_t(cg.Cout) * cg.Cin * cg.KH * cg.KW >= lim) return false;
    if (int64_t(cg.OH) * cg.OW >= lim || int64_t(cg.H) * cg.W >= lim) return false;
    if (int64_t(cg.B) * cg.OH * ceil_div(cg.OW, 32) >= lim) return false;
    if (int64_t(cg.sh) * cg.OH + int64_t(cg.dh) * cg.KH + cg.ph >= lim) return false;
    if (int64_t(cg.sw) * cg.OW + int64_t(cg.dw) * cg.KW + cg.pw >= lim) return false;
    return true;
}

static size_t cv_pad_x_bytes(const ConvGeom &cg) { return (size_t(cg.B) * cg.Cin * cg.H * 8 + 255) & ~size_t(255); }
static size_t cv_pad_d_bytes(const ConvGeom &cg) { return (size_t(cg.B) * cg.Cout * cg.OH * 8 * 2 + 255) & ~size_t(255); }

static size_t cv_ws_bytes(const ConvGeom &cg, const CvPlan &p)
{
    if (!p.fast) return 0;
    const size_t part = size_t(p.splits) * cg.KH * cg.KW * cg.Cout * cg.Cin * sizeof(float);
    const size_t v = size_t(p.parts) * cg.Cout * 10 * sizeof(float);
    size_t n = part + ((v + 255) & ~size_t(255));
    if (p.pad) n = ((n + 255) & ~size_t(255)) + cv_pad_x_bytes(cg) + cv_pad_d_bytes(cg);   // the copies with rows of eight: codes, then dy
    return n;
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
        const unsigned grid = unsigned(plane);             // one workgroup per (co, ci): C_out * C_in < 2^31
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
    // what the kernels read: the caller's tensors, or -- maps narrower than eight columns -- copies with rows of eight
    const int8_t *kx = xq;
    const void *kd = dy;
    ConvGeom ck = cg;
    if (p.pad) {
        const size_t vbytes = (size_t(p.parts) * cg.Cout * 10 * sizeof(float) + 255) & ~size_t(255);
        char *copies = static_cast<char *>(ws) + ((part_bytes + vbytes + 255) & ~size_t(255));
        int8_t *xp = reinterpret_cast<int8_t *>(copies);
        uint16_t *dp = reinterpret_cast<uint16_t *>(copies + cv_pad_x_bytes(cg));
        const int64_t xrows = int64_t(cg.B) * cg.Cin * cg.H, drows = int64_t(cg.B) * cg.Cout * cg.OH;
        hipLaunchKernelGGL((k_conv_pad_rows<int8_t, u32x2>), dim3(unsigned(ceil_div(xrows, kCvThreads))), dim3(kCvThreads), 0, s, xq, xp,
                           xrows, cg.W);
        hipLaunchKernelGGL((k_conv_pad_rows<uint16_t, u32x4>), dim3(unsigned(ceil_div(drows, kCvThreads))), dim3(kCvThreads), 0, s,
                           static_cast<const uint16_t *>(dy), dp, drows, cg.OW);
        if (launch_status() != MESA_OK) return MESA_ERR_LAUNCH;
        kx = xp;
        kd = dp;
        ck.W = 8;
        ck.OW = 8;
    }
#define MESA_LAUNCH_CV(E, T3, NKS, RAG) \
    do { \
        auto kern = k_conv_dw<E, T3, NKS, RAG>; \
        constexpr int lds = CvCfg<T3, NKS>::LDS; \
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess) \
            return MESA_ERR_LAUNCH; \
        hipLaunchKernelGGL(kern, dim3(p.grid), dim3(kCvThreads), lds, s, kx, static_cast<const E *>(kd), ck, p.tiles_co, p.tiles_ci, \
                           p.splits, p.stages_per_split, p.nseg, part); \
    } while (0)
#define MESA_PICK_NKS(E, T3, RAG) \
    do { \
        if (p.nks == 8) MESA_LAUNCH_CV(E, T3, 8, RAG); \
        else if (p.nks == 4) MESA_LAUNCH_CV(E, T3, 4, RAG); \
        else if (p.nks == 2) MESA_LAUNCH_CV(E, T3, 2, RAG); \
        else MESA_LAUNCH_CV(E, T3, 1, RAG); \
    } while (0)
#define MESA_PICK_CV(E) \
    do { \
        if (p.pad) { \
            if (p.taps3) MESA_LAUNCH_CV(E, true, 1, 2); else MESA_LAUNCH_CV(E, false, 1, 2); \
            hipLaunchKernelGGL((k_conv_valid_sums<E>), dim3(unsigned(cg.Cout) * p.parts), dim3(kCvThreads), 0, s, \
                               static_cast<const E *>(kd), ck, p.parts, p.imgs_per_part, p.row_blocks, p.rows_per_block, V); \
        } else if (p.rag) { \
            if (p.taps3) MESA_PICK_NKS(E, true, 1); else MESA_PICK_NKS(E, false, 1); \
            hipLaunchKernelGGL((k_conv_valid_sums_any<E>), dim3(unsigned(cg.Cout) * p.parts), dim3(kCvThreads), 0, s, \
                               static_cast<const E *>(dy), cg, p.parts, p.imgs_per_part, p.row_blocks, p.rows_per_block, \
                               make_fastdiv(uint32_t(cg.OW)), V); \
        } else { \
            if (p.taps3) MESA_PICK_NKS(E, true, 0); else MESA_PICK_NKS(E, false, 0); \
            hipLaunchKernelGGL((k_conv_valid_sums<E>), dim3(unsigned(cg.Cout) * p.parts), dim3(kCvThreads), 0, s, \
                               static_cast<const E *>(dy), cg, p.parts, p.imgs_per_part, p.row_blocks, p.rows_per_block, V); \
        } \
    } while (0)
    float centre;
    if (dt == MESA_F16) { MESA_PICK_CV(_Float16); centre = CvElem<_Float16>::kCentre; }
    else { MESA_PICK_CV(__bf16); centre = CvElem<__bf16>::kCentre; }
#undef MESA_PICK_CV
#undef MESA_PICK_NKS
#undef MESA_LAUNCH_CV
    if (launch_status() != MESA_OK) return MESA_ERR_LAUNCH;   // the last kernel must not read sums nobody wrote
    if (plane <= 32768 && p.splits >= 32)       // very few pairs: 32 threads per pair, so that the chip has workgroups enough
        hipLaunchKernelGGL(k_conv_finish_few<32>, dim3(unsigned(ceil_div(plane, 32))), dim3(1024), 0, s, part, V, p.splits, p.parts, cg,
                           per, alpha, beta, centre, dW, db);
    else if (plane <= 262144 && p.splits >= 8)
        hipLaunchKernelGGL(k_conv_finish_few<8>, dim3(unsigned(ceil_div(plane, 32))), dim3(kCvThreads), 0, s, part, V, p.splits, p.parts, cg,
                           per, alpha, beta, centre, dW, db);
    else
        hipLaunchKernelGGL(k_conv_finish, dim3(unsigned(ceil_div(plane, kCvThreads))), dim3(kCvThreads), 0, s, part, V, p.splits, p.parts,
                           cg, per, alpha, beta, centre, dW, db);
    return launch_status();
}
