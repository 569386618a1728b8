// common.hpp -- device-side building blocks of the streaming kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "host_math.hpp"
#include "mesa.h"

namespace mesa {

constexpr int kThreads = 256;  // workgroup size of every streaming kernel (4 waves)
constexpr int kVec = 8;        // elements one thread handles per vector: 16 B of binary16, 8 B of codes
constexpr int kMaxGroups = 8192;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));

// ---------------------------------------------------------------------------------------------
// integer helpers
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t fastdiv(uint32_t n, const FastDiv &f)
{
    return (__umulhi(n, f.mul) + n) >> f.shift;
}

struct Cursor {
    uint32_t rem;  // position of the vector's first element inside its slab
    uint32_t g;    // group of that slab
};

// e < 2^53.  Quotient through a binary64 reciprocal, then corrected by at most one.
__device__ __forceinline__ Cursor cursor_init(int64_t e, const GroupGeom &gg)
{
    double q = floor(double(e) / double(gg.inner));
    int64_t slab = int64_t(q);
    int64_t rem = e - slab * int64_t(gg.inner);
    if (rem < 0) { rem += gg.inner; slab -= 1; }
    if (rem >= int64_t(gg.inner)) { rem -= gg.inner; slab += 1; }
    double qg = floor(double(slab) / double(gg.groups));
    int64_t g = slab - int64_t(qg) * int64_t(gg.groups);
    if (g < 0) g += gg.groups;
    if (g >= int64_t(gg.groups)) g -= gg.groups;
    Cursor c;
    c.rem = uint32_t(rem);
    c.g = uint32_t(g);
    return c;
}

__device__ __forceinline__ void cursor_advance(Cursor &c, const GroupGeom &gg)
{
    uint32_t r = c.rem + gg.step_rem;          // < 2 * inner < 2^32
    uint32_t carry = (r >= gg.inner) ? 1u : 0u;
    c.rem = r - (carry ? gg.inner : 0u);
    uint32_t g = c.g + gg.step_g + carry;      // < 2 * groups
    c.g = (g >= gg.groups) ? g - gg.groups : g;
}

// the cursor `delta` elements further on (delta < 2^16; inner < 2^30 keeps the dividend below 2^31)
__device__ __forceinline__ Cursor cursor_offset(const Cursor &c, uint32_t delta, const GroupGeom &gg)
{
    uint32_t r = c.rem + delta;
    uint32_t adv = fastdiv(r, gg.div_inner);
    Cursor o;
    o.rem = r - adv * gg.inner;
    uint32_t t = c.g + adv;
    o.g = t - fastdiv(t, gg.div_groups) * gg.groups;
    return o;
}

// group of element j (0..7) of a vector that starts at cursor c and may cross slab ends
__device__ __forceinline__ uint32_t group_of(const Cursor &c, uint32_t j, const GroupGeom &gg)
{
    uint32_t r = c.rem + j;
    uint32_t g = c.g;
    while (r >= gg.inner) {
        r -= gg.inner;
        g = (g + 1 == gg.groups) ? 0u : g + 1;
    }
    return g;
}

// ---------------------------------------------------------------------------------------------
// storage types: 8 consecutive elements <-> 8 floats
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ h2 as_h2(uint32_t w) { return __builtin_bit_cast(h2, w); }
__device__ __forceinline__ uint32_t as_u32(h2 v) { return __builtin_bit_cast(uint32_t, v); }

template <typename T> struct Store;  // T = float, _Float16 or __bf16

template <> struct Store<_Float16> {
    typedef u32x4 raw_t;  // 8 elements
    static constexpr int kBytes = 2;
    __device__ static __forceinline__ raw_t load(const void *base, int64_t e)
    {
        return *reinterpret_cast<const u32x4 *>(static_cast<const char *>(base) + e * 2);
    }
    __device__ static __forceinline__ void store(void *base, int64_t e, raw_t v)
    {
        *reinterpret_cast<u32x4 *>(static_cast<char *>(base) + e * 2) = v;
    }
    __device__ static __forceinline__ void unpack(raw_t v, float f[8])
    {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            h2 p = as_h2(v[k]);
            f[2 * k] = float(p.x);
            f[2 * k + 1] = float(p.y);
        }
    }
    __device__ static __forceinline__ raw_t pack(const float f[8])
    {
        raw_t v;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            h2 p;
            p.x = _Float16(f[2 * k]);      // round to nearest even
            p.y = _Float16(f[2 * k + 1]);
            v[k] = as_u32(p);
        }
        return v;
    }
    __device__ static __forceinline__ float load1(const void *base, int64_t e)
    {
        return float(static_cast<const _Float16 *>(base)[e]);
    }
    __device__ static __forceinline__ void store1(void *base, int64_t e, float f)
    {
        static_cast<_Float16 *>(base)[e] = _Float16(f);
    }
};

// bfloat16: the upper half of a binary32 word; widening is a shift, narrowing rounds to nearest even
template <> struct Store<__bf16> {
    typedef u32x4 raw_t;  // 8 elements
    typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
    static constexpr int kBytes = 2;
    __device__ static __forceinline__ raw_t load(const void *base, int64_t e)
    {
        return *reinterpret_cast<const u32x4 *>(static_cast<const char *>(base) + e * 2);
    }
    __device__ static __forceinline__ void store(void *base, int64_t e, raw_t v)
    {
        *reinterpret_cast<u32x4 *>(static_cast<char *>(base) + e * 2) = v;
    }
    __device__ static __forceinline__ void unpack(raw_t v, float f[8])
    {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            f[2 * k] = __uint_as_float(v[k] << 16);
            f[2 * k + 1] = __uint_as_float(v[k] & 0xFFFF0000u);
        }
    }
    __device__ static __forceinline__ raw_t pack(const float f[8])
    {
        raw_t v;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            bf2 p;
            p.x = __bf16(f[2 * k]);        // round to nearest even
            p.y = __bf16(f[2 * k + 1]);
            v[k] = __builtin_bit_cast(uint32_t, p);
        }
        return v;
    }
    __device__ static __forceinline__ float load1(const void *base, int64_t e)
    {
        return __uint_as_float(uint32_t(static_cast<const uint16_t *>(base)[e]) << 16);
    }
    __device__ static __forceinline__ void store1(void *base, int64_t e, float f)
    {
        static_cast<__bf16 *>(base)[e] = __bf16(f);
    }
};

template <> struct Store<float> {
    struct raw_t { u32x4 lo, hi; };
    static constexpr int kBytes = 4;
    __device__ static __forceinline__ raw_t load(const void *base, int64_t e)
    {
        const u32x4 *p = reinterpret_cast<const u32x4 *>(static_cast<const char *>(base) + e * 4);
        raw_t r;
        r.lo = p[0];
        r.hi = p[1];
        return r;
    }
    __device__ static __forceinline__ void store(void *base, int64_t e, raw_t v)
    {
        u32x4 *p = reinterpret_cast<u32x4 *>(static_cast<char *>(base) + e * 4);
        p[0] = v.lo;
        p[1] = v.hi;
    }
    __device__ static __forceinline__ void unpack(raw_t v, float f[8])
    {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            f[k] = __uint_as_float(v.lo[k]);
            f[4 + k] = __uint_as_float(v.hi[k]);
        }
    }
    __device__ static __forceinline__ raw_t pack(const float f[8])
    {
        raw_t v;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            v.lo[k] = __float_as_uint(f[k]);
            v.hi[k] = __float_as_uint(f[4 + k]);
        }
        return v;
    }
    __device__ static __forceinline__ float load1(const void *base, int64_t e)
    {
        return static_cast<const float *>(base)[e];
    }
    __device__ static __forceinline__ void store1(void *base, int64_t e, float f)
    {
        static_cast<float *>(base)[e] = f;
    }
};

// ---------------------------------------------------------------------------------------------
// streaming accesses: every byte is touched once, so mark them non-temporal
// ---------------------------------------------------------------------------------------------
template <typename V> __device__ __forceinline__ V nt_load(const void *p)
{
    return __builtin_nontemporal_load(static_cast<const V *>(p));
}
template <typename V> __device__ __forceinline__ void nt_store(void *p, V v)
{
    __builtin_nontemporal_store(v, static_cast<V *>(p));
}

template <typename T> struct Nt;
template <> struct Nt<_Float16> {
    __device__ static __forceinline__ u32x4 load(const void *b, int64_t e) { return nt_load<u32x4>(static_cast<const char *>(b) + e * 2); }
    __device__ static __forceinline__ void store(void *b, int64_t e, u32x4 v) { nt_store<u32x4>(static_cast<char *>(b) + e * 2, v); }
};
template <> struct Nt<__bf16> : Nt<_Float16> {};
template <> struct Nt<float> {
    __device__ static __forceinline__ Store<float>::raw_t load(const void *b, int64_t e)
    {
        Store<float>::raw_t r;
        r.lo = nt_load<u32x4>(static_cast<const char *>(b) + e * 4);
        r.hi = nt_load<u32x4>(static_cast<const char *>(b) + e * 4 + 16);
        return r;
    }
    __device__ static __forceinline__ void store(void *b, int64_t e, Store<float>::raw_t v)
    {
        nt_store<u32x4>(static_cast<char *>(b) + e * 4, v.lo);
        nt_store<u32x4>(static_cast<char *>(b) + e * 4 + 16, v.hi);
    }
};

// 8 codes (int8, q = x_bar - 128) <-> 8 floats holding x_bar in [0, 255]
__device__ __forceinline__ u32x2 load_codes8(const int8_t *q, int64_t e)
{
    return *reinterpret_cast<const u32x2 *>(q + e);
}

__device__ __forceinline__ void codes_to_float(u32x2 c, float u[8])
{
#pragma unroll
    for (int w = 0; w < 2; ++w) {
        uint32_t b = c[w] ^ 0x80808080u;  // +128 on each signed byte
        u[4 * w + 0] = float(b & 0xFFu);
        u[4 * w + 1] = float((b >> 8) & 0xFFu);
        u[4 * w + 2] = float((b >> 16) & 0xFFu);
        u[4 * w + 3] = float(b >> 24);
    }
}

__device__ __forceinline__ float code_to_float(int8_t c) { return float(int(c) + 128); }

// w[] are integers in [0, 255] held as floats
__device__ __forceinline__ u32x2 float_to_codes(const float w[8])
{
    u32x2 c;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        uint32_t b = uint32_t(w[4 * k]) | (uint32_t(w[4 * k + 1]) << 8) | (uint32_t(w[4 * k + 2]) << 16) |
                     (uint32_t(w[4 * k + 3]) << 24);
        c[k] = b ^ 0x80808080u;  // -128 on each byte
    }
    return c;
}

__device__ __forceinline__ float clamp_code(float w) { return fminf(fmaxf(w, 0.0f), 255.0f); }

// ---------------------------------------------------------------------------------------------
// wave / workgroup reductions (wave64)
// ---------------------------------------------------------------------------------------------
template <int WIDTH> __device__ __forceinline__ float lanes_sum(float v)
{
#pragma unroll
    for (int off = WIDTH / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// The same sum over aligned groups of WIDTH lanes, every lane receiving it, with the first four
// levels done by data-parallel-primitive lane swaps inside the adder instruction (pairs, quads,
// mirrored halves of 8 and of 16: after each level both partners hold the same value, so a mirror
// is as good as an exchange) and only the levels across 16-lane rows through the LDS crossbar.
template <int CTRL> __device__ __forceinline__ float dpp_move(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
template <int WIDTH> __device__ __forceinline__ float lanes_sum_dpp(float v)
{
    static_assert(WIDTH == 4 || WIDTH == 8 || WIDTH == 16 || WIDTH == 32 || WIDTH == 64, "aligned power-of-two lane groups");
    v += dpp_move<0xB1>(v);                      // quad_perm [1,0,3,2]
    v += dpp_move<0x4E>(v);                      // quad_perm [2,3,0,1]
    if (WIDTH >= 8) v += dpp_move<0x141>(v);     // row_half_mirror
    if (WIDTH >= 16) v += dpp_move<0x140>(v);    // row_mirror
    if (WIDTH >= 32) v += __shfl_xor(v, 16, 64);
    if (WIDTH >= 64) v += __shfl_xor(v, 32, 64);
    return v;
}

}  // namespace mesa
