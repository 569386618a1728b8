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

constexpr int kSmU = 4;                            // vectors per thread in a tile
constexpr int kSmTileVec = kThreads * kSmU;        // 1024 vectors = 8192 elements per tile
constexpr int kSmMaxRows = kSmTileVec;             // cols >= 8 -> at most one row per vector

template <typename T>
__global__ __launch_bounds__(kThreads) void k_softmax_bwd(const int8_t *__restrict__ yq, const void *dy, void *dx,
                                                          int64_t total_rows, uint32_t cols, uint32_t R, int64_t tiles,
                                                          FastDiv div_cols, FastDiv div_rows, FastDiv div_heads,
                                                          const float *__restrict__ alpha, const float *__restrict__ beta)
{
    __shared__ float rowS[kSmMaxRows], rowB[kSmMaxRows], rowD[kSmMaxRows];
    __shared__ float PA[kSmTileVec], PB[kSmTileVec];

    const uint32_t tid = threadIdx.x;
    for (int64_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
        const int64_t row0 = tile * R;
        const uint32_t nrows = uint32_t((total_rows - row0 < int64_t(R)) ? (total_rows - row0) : int64_t(R));
        const uint32_t nelem = nrows * cols;
        const uint32_t nvec = (nelem + kVec - 1) / kVec;
        const int64_t e0 = row0 * cols;

        // per-row scale and offset of the row's head
        for (uint32_t r = tid; r < nrows; r += kThreads) {
            uint32_t slab = fastdiv(uint32_t(row0) + r, div_rows);          // (b*H + h)
            uint32_t h = slab - fastdiv(slab, div_heads) * div_heads.d;
            rowS[r] = alpha[h] / 255.0f;
            rowB[r] = beta[h];
        }
        __syncthreads();

        u32x2 cq[kSmU];
        typename Store<T>::raw_t cd[kSmU];
        uint32_t r1[kSmU], nb[kSmU];
#pragma unroll
        for (int u = 0; u < kSmU; ++u) {
            const uint32_t v = u * kThreads + tid;
            if (v < nvec) {
                const uint32_t le = v * kVec;
                const int64_t e = e0 + le;
                float g[8], y[8];
                if (le + kVec <= nelem) {
                    cq[u] = load_codes8(yq, e);
                    cd[u] = Store<T>::load(dy, e);
                    Store<T>::unpack(cd[u], g);
                } else {  // ragged end of the whole tensor
                    int8_t cb[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        bool in = le + j < nelem;
                        cb[j] = in ? yq[e + j] : int8_t(0);
                        g[j] = in ? Store<T>::load1(dy, e + j) : 0.0f;
                    }
                    cq[u][0] = uint32_t(uint8_t(cb[0])) | (uint32_t(uint8_t(cb[1])) << 8) | (uint32_t(uint8_t(cb[2])) << 16) |
                               (uint32_t(uint8_t(cb[3])) << 24);
                    cq[u][1] = uint32_t(uint8_t(cb[4])) | (uint32_t(uint8_t(cb[5])) << 8) | (uint32_t(uint8_t(cb[6])) << 16) |
                               (uint32_t(uint8_t(cb[7])) << 24);
                    cd[u] = Store<T>::pack(g);   // exact: g came from T
                }
                r1[u] = fastdiv(le, div_cols);
                nb[u] = (r1[u] + 1) * cols - le;   // elements of this vector that lie in row r1
                const uint32_t r2 = (r1[u] + 1 < nrows) ? r1[u] + 1 : r1[u];
                const float sA = rowS[r1[u]], bA = rowB[r1[u]], sB = rowS[r2], bB = rowB[r2];
                codes_to_float(cq[u], y);
                float pA = 0.0f, pB = 0.0f;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const bool first = uint32_t(j) < nb[u];
                    const float yh = fmaf(y[j], first ? sA : sB, first ? bA : bB);
                    const float p = g[j] * yh;
                    pA += first ? p : 0.0f;
                    pB += first ? 0.0f : p;
                }
                PA[v] = pA;
                PB[v] = pB;
            }
        }
        __syncthreads();

        // 16 lanes per row: the row's own part of its first vector, then the vectors that start in it
        {
            const uint32_t lane16 = tid & 15u;
            for (uint32_t r = tid >> 4; r < nrows; r += kThreads / 16) {
                const uint32_t start = r * cols;
                const uint32_t vs = start >> 3;
                const uint32_t ve = (start + cols - 1) >> 3;
                float s = 0.0f;
                if (lane16 == 0) s = (start & 7u) ? PB[vs] : PA[vs];
                for (uint32_t v = vs + 1 + lane16; v <= ve; v += 16) s += PA[v];
                s = lanes_sum<16>(s);
                if (lane16 == 0) rowD[r] = s;
            }
        }
        __syncthreads();

#pragma unroll
        for (int u = 0; u < kSmU; ++u) {
            const uint32_t v = u * kThreads + tid;
            if (v < nvec) {
                const uint32_t le = v * kVec;
                const int64_t e = e0 + le;
                const uint32_t r2 = (r1[u] + 1 < nrows) ? r1[u] + 1 : r1[u];
                const float sA = rowS[r1[u]], bA = rowB[r1[u]], sB = rowS[r2], bB = rowB[r2];
                const float dA = rowD[r1[u]], dB = rowD[r2];
                float g[8], y[8], o[8];
                Store<T>::unpack(cd[u], g);
                codes_to_float(cq[u], y);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const bool first = uint32_t(j) < nb[u];
                    const float yh = fmaf(y[j], first ? sA : sB, first ? bA : bB);
                    o[j] = yh * (g[j] - (first ? dA : dB));
                }
                if (le + kVec <= nelem) {
                    Store<T>::store(dx, e, Store<T>::pack(o));
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (le + j < nelem) Store<T>::store1(dx, e + j, o[j]);
                }
            }
        }
        __syncthreads();  // the next tile rewrites the row tables and partial sums
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
    if (H > kMaxGroups || rows >= (int64_t(1) << 31) || cols < kVec || cols > kSmTileVec * kVec) return MESA_ERR_UNSUPPORTED;
    const long double tr = (long double)B * (long double)H * (long double)rows;
    if (tr >= 2147483648.0L) return MESA_ERR_UNSUPPORTED;
    const int64_t total_rows = B * H * rows;
    // rows per tile: a multiple of 8/gcd(cols, 8) so that every tile starts on a vector boundary
    int64_t gc = cols, b8 = 8;
    while (b8) { int64_t t = gc % b8; gc = b8; b8 = t; }
    const int64_t unit = 8 / gc;
    int64_t R = (int64_t(kSmTileVec) * kVec / cols) / unit * unit;
    if (R < unit) return MESA_ERR_UNSUPPORTED;   // unit rows of this length do not fit one tile
    if (R > total_rows) R = ceil_div(total_rows, unit) * unit;
    const int64_t tiles = ceil_div(total_rows, R);
    const int grid = int(tiles < 1024 ? tiles : 1024);
    FastDiv dc = make_fastdiv(uint32_t(cols)), dr = make_fastdiv(uint32_t(rows)), dh = make_fastdiv(uint32_t(H));
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dt == MESA_F16)
        hipLaunchKernelGGL((k_softmax_bwd<_Float16>), dim3(grid), dim3(kThreads), 0, s, yq, dy, dx, total_rows, uint32_t(cols),
                           uint32_t(R), tiles, dc, dr, dh, alpha, beta);
    else
        hipLaunchKernelGGL((k_softmax_bwd<float>), dim3(grid), dim3(kThreads), 0, s, yq, dy, dx, total_rows, uint32_t(cols),
                           uint32_t(R), tiles, dc, dr, dh, alpha, beta);
    return launch_status();
}
