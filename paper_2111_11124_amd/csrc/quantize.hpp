// quantize.hpp -- the pieces of the quantizer that more than one kernel file uses: the counter-based random
// bits of stochastic rounding, Eq. (3)-(4) for one element, code packing, and the order-preserving integer
// keys of the per-group extrema.  Device code; every file that includes it is compiled with floating-point
// contraction off, which Eq. (3)'s separately rounded operations rely on.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "common.hpp"

namespace mesa {

__device__ __forceinline__ int order_key(float f)  // monotone map binary32 -> int32 (an involution)
{
    int b = __float_as_int(f);
    return b >= 0 ? b : b ^ 0x7FFFFFFF;
}
__device__ __forceinline__ float order_val(int k) { return __int_as_float(k >= 0 ? k : k ^ 0x7FFFFFFF); }


// ---------------------------------------------------------------------------------------------
// Philox-4x32-10 (Salmon et al., SC'11): ten rounds of two 32x32->64 multiplies and a key bump
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t k0, uint32_t k1, uint32_t out[4])
{
    uint32_t c2 = 0u, c3 = 0u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        uint64_t p0 = uint64_t(0xD2511F53u) * uint64_t(c0);
        uint64_t p1 = uint64_t(0xCD9E8D57u) * uint64_t(c2);
        uint32_t n0 = __builtin_amdgcn_bitop3_b32(uint32_t(p1 >> 32), c1, k0, 0x96);   // a ^ b ^ c in one instruction
        uint32_t n2 = __builtin_amdgcn_bitop3_b32(uint32_t(p0 >> 32), c3, k1, 0x96);
        c1 = uint32_t(p1);
        c3 = uint32_t(p0);
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// 16 random bits (as a float in [0, 65536)) for each of the eight elements of block `counter`
__device__ __forceinline__ void sr_bits(uint64_t seed, uint64_t counter, float b[8])
{
    uint32_t w[4];
    philox4x32_10(uint32_t(counter), uint32_t(counter >> 32), uint32_t(seed), uint32_t(seed >> 32), w);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        b[2 * k] = float(w[k] & 0xFFFFu);
        b[2 * k + 1] = float(w[k] >> 16);
    }
}

// Eq. (3)-(4) for one element; returns the integer x_bar (unclipped) as a float.
// Stochastic rounding adds u = bits*2^-16: the product is exact, so the fused form rounds once,
// exactly like the separate sum v + u.
// SYM: the scale-only symmetric scheme of the ablation (Sec. 5.2) -- no offset, v = x * r with r = 127 / m, and the
// integer returned is already moved to the stored form's range: max(w, -127) + 128 in [1, 255] (the packing below
// saturates the upper end and takes the 128 off again), so that the code is clip(w, -127, 127).
template <bool SR, bool SYM = false> __device__ __forceinline__ float quantize_one(float x, float r, float b, float bits)
{
    float t = SYM ? x : x - b;
    float v = t * r;
    float w = SR ? floorf(__builtin_fmaf(bits, 1.52587890625e-05f, v)) : rintf(v);  // nearest: ties to even
    if (SYM) w = fmaxf(w, -127.0f) + 128.0f;
    return w;
}

// eight unclipped integers -> eight codes; the conversion instruction saturates to [0, 255]
__device__ __forceinline__ u32x2 pack_codes(const float w[8])
{
    u32x2 c;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        uint32_t b = 0u;
        b = __builtin_amdgcn_cvt_pk_u8_f32(w[4 * k + 0], 0, b);
        b = __builtin_amdgcn_cvt_pk_u8_f32(w[4 * k + 1], 1, b);
        b = __builtin_amdgcn_cvt_pk_u8_f32(w[4 * k + 2], 2, b);
        b = __builtin_amdgcn_cvt_pk_u8_f32(w[4 * k + 3], 3, b);
        c[k] = b ^ 0x80808080u;  // -128 on each byte
    }
    return c;
}

// plain selection instructions: the data holds no NaN by contract, so no canonicalisation is wanted
__device__ __forceinline__ float vmin(float a, float b) { float r; asm("v_min_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b)); return r; }
__device__ __forceinline__ float vmax(float a, float b) { float r; asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b)); return r; }
__device__ __forceinline__ uint32_t pkmin(uint32_t a, uint32_t b) { uint32_t r; asm("v_pk_min_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b)); return r; }
__device__ __forceinline__ uint32_t pkmax(uint32_t a, uint32_t b) { uint32_t r; asm("v_pk_max_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b)); return r; }

// Host side: combine the per-workgroup extrema part[nwg][2 * groups] (minima, then maxima) and move the running
// estimates, Eq. (6)-(7); defined with the kernel in stream_kernels.hip.  variant: 0 plain, 1 symmetric range,
// 2 fixed offset (beta_fixed).
void launch_ema_finalize(const float *part, int nwg, uint32_t groups, float *alpha, float *beta, float lambda, int first_call,
                         int variant, float beta_fixed, hipStream_t stream);

}  // namespace mesa
