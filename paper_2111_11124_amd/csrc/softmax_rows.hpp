// softmax_rows.hpp -- what the two row-per-lane-group softmax kernels (forward with quantizer, backward at
// de-quantized codes) share: the tile shape, the wave-level synchronisation, reductions inside a lane group and
// the staged element's conversions.
//
// Rows of an attention map (197, 49 elements) start at odd byte offsets.  A wave owns a tile of R consecutive rows
// with R * cols a multiple of 8, i.e. a run of whole 8-element vectors that is 16-byte aligned in the tensors and
// 8-byte aligned in the codes: memory is only touched as whole aligned vectors (flat phases), the tile lies in the
// wave's LDS region as it lies in memory, and in between a row belongs to a group of LPR lanes, lane l holding
// elements l, l + LPR, ... in EPL register slots, each a constant distance from the lane's first element.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "common.hpp"
#include "quantize.hpp"

namespace mesa {

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

constexpr int kSrTileElems = 2048;                    // elements of a wave's tile at most
constexpr int kSrFlat = kSrTileElems / kVec / 64;     // vectors per lane in the flat phases
constexpr int kSrMaxCols = 256;
constexpr int kSrSlack = 1024;                        // bytes past the last region that unused slots may read

template <int WIDTH, bool MAX> __device__ __forceinline__ float lanes_extreme_dpp(float v)
{
    static_assert(WIDTH == 8 || WIDTH == 16, "lane groups inside a DPP row");
    v = MAX ? vmax(v, dpp_move<0xB1>(v)) : vmin(v, dpp_move<0xB1>(v));      // quad_perm [1,0,3,2]
    v = MAX ? vmax(v, dpp_move<0x4E>(v)) : vmin(v, dpp_move<0x4E>(v));      // quad_perm [2,3,0,1]
    v = MAX ? vmax(v, dpp_move<0x141>(v)) : vmin(v, dpp_move<0x141>(v));    // row_half_mirror
    if (WIDTH >= 16) v = MAX ? vmax(v, dpp_move<0x140>(v)) : vmin(v, dpp_move<0x140>(v));   // row_mirror
    return v;
}

// one staged element <-> binary32; put() returns the value as stored
template <typename T> struct LdsElem;
template <> struct LdsElem<_Float16> {
    __device__ static __forceinline__ float get(const unsigned char *p) { return float(*reinterpret_cast<const _Float16 *>(p)); }
    __device__ static __forceinline__ float put(unsigned char *p, float v)
    {
        const _Float16 h = _Float16(v);
        *reinterpret_cast<_Float16 *>(p) = h;
        return float(h);
    }
};
template <> struct LdsElem<__bf16> {
    __device__ static __forceinline__ float get(const unsigned char *p)
    {
        return __uint_as_float(uint32_t(*reinterpret_cast<const uint16_t *>(p)) << 16);
    }
    __device__ static __forceinline__ float put(unsigned char *p, float v)
    {
        const __bf16 h = __bf16(v);
        const uint16_t bits = __builtin_bit_cast(uint16_t, h);
        *reinterpret_cast<uint16_t *>(p) = bits;
        return __uint_as_float(uint32_t(bits) << 16);
    }
};
template <> struct LdsElem<float> {
    __device__ static __forceinline__ float get(const unsigned char *p) { return *reinterpret_cast<const float *>(p); }
    __device__ static __forceinline__ float put(unsigned char *p, float v)
    {
        *reinterpret_cast<float *>(p) = v;
        return v;
    }
};

// lanes per row, slots per lane and rows per tile for rows of `cols` <= kSrMaxCols elements
struct SrShape {
    int lpr, epl;
    bool tight;          // cols > lpr * (epl - 1): only a lane's last slot can lie beyond the row's end
    int64_t R, tiles;
};

inline SrShape sr_shape(int64_t total_rows, int64_t cols)
{
    SrShape p{};
    if (cols <= 56) { p.lpr = 8; p.epl = 7; }
    else if (cols <= 64) { p.lpr = 8; p.epl = 8; }         // 8 x 8 windows: every slot used (8 x 13 leaves 38 % idle)
    else if (cols <= 104) { p.lpr = 8; p.epl = 13; }
    else if (cols <= 128) { p.lpr = 8; p.epl = 16; }
    else if (cols <= 200) { p.lpr = 8; p.epl = 25; }
    else { p.lpr = 16; p.epl = 16; }
    p.tight = cols > int64_t(p.lpr) * (p.epl - 1);
    int64_t gc = cols, b8 = 8;
    while (b8) { int64_t t = gc % b8; gc = b8; b8 = t; }
    const int64_t unit = 8 / gc, rpp = 64 / p.lpr;
    const int64_t step = unit > rpp ? unit : rpp;          // whole vectors per tile, whole passes
    p.R = (kSrTileElems / cols) / step * step;             // step * cols <= 8 * 256
    if (p.R > total_rows) p.R = (total_rows + step - 1) / step * step;
    p.tiles = (total_rows + p.R - 1) / p.R;
    return p;
}

}  // namespace mesa
