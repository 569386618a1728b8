// stream_kernels.hip -- the HBM-bound element-wise half of libmesa for gfx950:
//   per-group min/max + running-estimate update   (Sec. 3.2 Eq. 6-7)
//   quantize with nearest or stochastic rounding  (Sec. 3.2 Eq. 3-4)
//   de-quantize                                    (Sec. 3.2 Eq. 5)
//   GELU backward at the de-quantized input        (Sec. 3.1 Eq. 2)
// plus a plain copy kernel and HIP-event helpers for measurement.
//
// Shape of every kernel: 256-thread workgroups, grid-stride; per iteration a thread owns U
// vectors of 8 consecutive elements (one 128-bit load of binary16, one 64-bit access of codes),
// a whole grid apart from each other so that each wave instruction touches one contiguous span.
// The group of a vector is tracked by a cursor (adds and compares only); vectors that cross a
// slab end, and the ragged tail, take a per-element path.
//
// Everything that feeds a code or a running parameter is binary32 with separately rounded
// operations: contraction into fused multiply-adds is switched off for this file, and the one
// kernel that may fuse (GELU backward) asks for it explicitly with fmaf.
#include <hip/hip_runtime.h>

#include <atomic>
#include <type_traits>

#include "api_util.hpp"
#include "common.hpp"
#include "quantize.hpp"

#pragma clang fp contract(off)

namespace mesa {

// Launch shape, found by sweeping on the MI355X: the read-modify-write streams do best with two
// vectors in flight per thread and many workgroups (more waves to hide the integer multiplies of
// the random generator); the read-only min/max scan with four vectors and fewer workgroups.
constexpr int kU = 2;                            // vectors per thread and iteration
constexpr int kGridCap = 1 << 20;                // one chunk per workgroup up to 2^32 elements: the workgroups in flight then sweep the tensor as one compact window (a grid-stride loop has them at 2^12-element pieces spread over the whole tensor, measured 15 % slower at 2^31 elements)
constexpr int kMmU = 4;                          // the same two numbers for the min/max scan
constexpr int kMmGridCap = 1024;
constexpr int kMmFew = 8;                        // groups for which a thread can hold every group's extrema
constexpr int kFuU = 2;                          // and for the single-pass quantize + min/max
constexpr int kFuGridCap = 2048;
constexpr int kLutMaxGroups = 64;                // GELU-gradient table: groups * 256 floats in LDS

// The cursors of a thread's U vectors: vector u of the chunk that starts at `base` covers
// elements base + (u*256 + tid)*8 ... + 7.
template <int U> __device__ __forceinline__ void place_cursors(Cursor c[U], const GroupGeom &gg, int64_t numel)
{
    constexpr int kChunk = kThreads * U * kVec;   // what a workgroup moves per iteration
    const int64_t e0 = int64_t(blockIdx.x) * kChunk + int64_t(threadIdx.x) * kVec;
    if (numel < (int64_t(1) << 31)) {   // uniform branch: two multiplies instead of binary64 divisions
        Cursor z;
        z.rem = 0u;
        z.g = 0u;
        c[0] = (e0 < numel) ? cursor_offset(z, uint32_t(e0), gg) : z;
    } else {
        c[0] = cursor_init(e0, gg);
    }
#pragma unroll
    for (int u = 1; u < U; ++u) c[u] = cursor_offset(c[0], uint32_t(u * kThreads * kVec), gg);
}

// ---------------------------------------------------------------------------------------------
// per-group parameter table in LDS: (scale, beta) per group
// ---------------------------------------------------------------------------------------------
// (QuantSym / DequantSym: the scale-only symmetric scheme -- alpha holds m, the running estimate of max |x|;
// 127 steps on each side of zero, no offset, beta is not read)
enum class Scale { Quant, Dequant, QuantSym, DequantSym };

template <Scale S>
__device__ __forceinline__ void fill_table(float2 *tab, const float *alpha, const float *beta, uint32_t groups)
{
    for (uint32_t g = threadIdx.x; g < groups; g += kThreads) {
        float a = alpha[g];
        float s;
        if (S == Scale::Quant) s = (a > 0.0f) ? 255.0f / a : 0.0f;  // correctly rounded division
        else if (S == Scale::QuantSym) s = (a > 0.0f) ? 127.0f / a : 0.0f;
        else if (S == Scale::DequantSym) s = a / 127.0f;
        else s = a / 255.0f;
        tab[g] = make_float2(s, (S == Scale::QuantSym || S == Scale::DequantSym) ? 0.0f : beta[g]);
    }
    __syncthreads();
}

// The same for a kernel whose workgroups take ONE chunk of `chunk` consecutive elements each (the grid covers the
// tensor): with many groups -- per-sample statistics are a layout of B * G groups -- a workgroup fills only the
// entries of the groups its chunk touches, a cyclic run of the group numbers.  Filling all 3072 entries of the layout
// (1, 3072, 38809) in every workgroup (twelve loads and divisions per thread before the first element moves) held
// quantize at 2.5 TB/s where six groups reach 3.7.
template <Scale S>
__device__ __forceinline__ void fill_table_touched(float2 *tab, const float *alpha, const float *beta, const GroupGeom &gg, int64_t numel,
                                                   int64_t chunk)
{
    const int64_t base = int64_t(blockIdx.x) * chunk;
    const int64_t row = int64_t(gg.groups) * gg.inner;
    if (gg.groups <= uint32_t(kThreads) || int64_t(gridDim.x) * chunk < numel || chunk >= row || base >= numel) {
        fill_table<S>(tab, alpha, beta, gg.groups);
        return;
    }
    const int64_t last = (base + chunk <= numel ? base + chunk : numel) - 1;
    const uint32_t g_first = cursor_init(base, gg).g, g_last = cursor_init(last, gg).g;
    const uint32_t count = (g_last >= g_first ? g_last - g_first : g_last + gg.groups - g_first) + 1;
    for (uint32_t t = threadIdx.x; t < count; t += kThreads) {
        uint32_t g = g_first + t;
        g -= g >= gg.groups ? gg.groups : 0u;
        float a = alpha[g];
        float s;
        if (S == Scale::Quant) s = (a > 0.0f) ? 255.0f / a : 0.0f;
        else if (S == Scale::QuantSym) s = (a > 0.0f) ? 127.0f / a : 0.0f;
        else if (S == Scale::DequantSym) s = a / 127.0f;
        else s = a / 255.0f;
        tab[g] = make_float2(s, (S == Scale::QuantSym || S == Scale::DequantSym) ? 0.0f : beta[g]);
    }
    __syncthreads();
}

// ---------------------------------------------------------------------------------------------
// min / max
// ---------------------------------------------------------------------------------------------
template <typename T> struct MinMax;

template <> struct MinMax<float> {
    float mn, mx;
    __device__ __forceinline__ void init() { mn = __builtin_inff(); mx = -__builtin_inff(); }
    __device__ __forceinline__ void add(const Store<float>::raw_t &v)
    {
        float f[8];
        Store<float>::unpack(v, f);
#pragma unroll
        for (int j = 0; j < 8; ++j) { mn = vmin(mn, f[j]); mx = vmax(mx, f[j]); }
    }
    __device__ __forceinline__ void add1(float f) { mn = vmin(mn, f); mx = vmax(mx, f); }
    __device__ __forceinline__ void merge(const MinMax<float> &o) { mn = vmin(mn, o.mn); mx = vmax(mx, o.mx); }
    __device__ __forceinline__ float lo() const { return mn; }
    __device__ __forceinline__ float hi() const { return mx; }
};

// bfloat16 data: widened (a shift or a mask per element) and compared as binary32
template <> struct MinMax<__bf16> {
    float mn, mx;
    __device__ __forceinline__ void init() { mn = __builtin_inff(); mx = -__builtin_inff(); }
    __device__ __forceinline__ void add(const Store<__bf16>::raw_t &v)
    {
        float f[8];
        Store<__bf16>::unpack(v, f);
#pragma unroll
        for (int j = 0; j < 8; ++j) { mn = vmin(mn, f[j]); mx = vmax(mx, f[j]); }
    }
    __device__ __forceinline__ void add1(float f) { mn = vmin(mn, f); mx = vmax(mx, f); }
    __device__ __forceinline__ void merge(const MinMax<__bf16> &o) { mn = vmin(mn, o.mn); mx = vmax(mx, o.mx); }
    __device__ __forceinline__ float lo() const { return mn; }
    __device__ __forceinline__ float hi() const { return mx; }
};

// binary16 data: selection is exact in any precision, so compare packed pairs directly
template <> struct MinMax<_Float16> {
    uint32_t mn, mx;
    __device__ __forceinline__ void init()
    {
        mn = 0x7C007C00u;  // +inf, +inf
        mx = 0xFC00FC00u;  // -inf, -inf
    }
    __device__ __forceinline__ void add(const Store<_Float16>::raw_t &v)
    {
        mn = pkmin(mn, pkmin(pkmin(v[0], v[1]), pkmin(v[2], v[3])));
        mx = pkmax(mx, pkmax(pkmax(v[0], v[1]), pkmax(v[2], v[3])));
    }
    __device__ __forceinline__ void add1(float f)
    {
        h2 p;
        p.x = _Float16(f);
        p.y = p.x;
        mn = pkmin(mn, as_u32(p));
        mx = pkmax(mx, as_u32(p));
    }
    __device__ __forceinline__ void merge(const MinMax<_Float16> &o) { mn = pkmin(mn, o.mn); mx = pkmax(mx, o.mx); }
    __device__ __forceinline__ float lo() const { h2 p = as_h2(mn); return vmin(float(p.x), float(p.y)); }
    __device__ __forceinline__ float hi() const { h2 p = as_h2(mx); return vmax(float(p.x), float(p.y)); }
};

__device__ __forceinline__ void flush_lane(int *lmn, int *lmx, uint32_t g, float lo, float hi)
{
    if (lo <= hi) {  // something was accumulated
        atomicMin(&lmn[g], order_key(lo));
        atomicMax(&lmx[g], order_key(hi));
    }
}

// All 64 lanes call this together; the lanes with `flush` set hand their extrema to LDS.  Lanes of a
// wave cover 512 consecutive elements, so they normally leave a head's slab together and for the
// same old group: then the wave combines in registers and one lane issues the two atomics
// (64 same-address LDS atomics from one instruction are serialised and cost thousands of cycles).
__device__ __forceinline__ void flush_wave(int *lmn, int *lmx, bool flush, uint32_t g, float lo, float hi)
{
    const unsigned long long mask = __ballot(flush);
    const int first = __ffsll((long long)mask) - 1;
    const uint32_t g0 = __builtin_amdgcn_readlane(g, first);
    if (__ballot(flush && g != g0) == 0ull) {
        lo = flush ? lo : __builtin_inff();
        hi = flush ? hi : -__builtin_inff();
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            lo = vmin(lo, __shfl_xor(lo, off, 64));
            hi = vmax(hi, __shfl_xor(hi, off, 64));
        }
        if (int(threadIdx.x & 63) == first) flush_lane(lmn, lmx, g0, lo, hi);
    } else if (flush) {
        flush_lane(lmn, lmx, g, lo, hi);
    }
}

// the elements of a vector taken one by one: for vectors that cross a slab end and for the ragged tail
template <typename T> struct MinMaxState {
    MinMax<T> acc;
    uint32_t cur;
};

template <typename T>
__device__ __forceinline__ void minmax_element(MinMaxState<T> &st, uint32_t g, float f, int *lmn, int *lmx)
{
    if (g != st.cur) {
        flush_lane(lmn, lmx, st.cur, st.acc.lo(), st.acc.hi());
        st.cur = g;
        st.acc.init();
    }
    st.acc.add1(f);
}

// End of a kernel that tracked extrema: what the threads still hold goes to the LDS tables, and the
// tables become this workgroup's partials.  The U accumulators that sit in the same group are folded
// first, and a wave whose lanes all sit in one group (head-wise tensors) combines in registers
// before touching LDS.
template <typename T, int U>
__device__ __forceinline__ void minmax_finish(MinMaxState<T> (&st)[U], int *lmn, int *lmx, float *__restrict__ part,
                                              const GroupGeom &gg)
{
    float lo = st[0].acc.lo(), hi = st[0].acc.hi();
#pragma unroll
    for (int u = 1; u < U; ++u) {
        if (st[u].cur == st[0].cur) {
            lo = vmin(lo, st[u].acc.lo());
            hi = vmax(hi, st[u].acc.hi());
        } else {
            flush_lane(lmn, lmx, st[u].cur, st[u].acc.lo(), st[u].acc.hi());
        }
    }
    const uint32_t g0 = __builtin_amdgcn_readfirstlane(st[0].cur);
    if (__all(st[0].cur == g0)) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            lo = vmin(lo, __shfl_xor(lo, off, 64));
            hi = vmax(hi, __shfl_xor(hi, off, 64));
        }
        if ((threadIdx.x & 63) == 0) flush_lane(lmn, lmx, g0, lo, hi);
    } else {
        flush_lane(lmn, lmx, st[0].cur, lo, hi);
    }
    __syncthreads();
    float *out = part + int64_t(blockIdx.x) * 2 * gg.groups;
    for (uint32_t g = threadIdx.x; g < gg.groups; g += kThreads) {
        out[g] = order_val(lmn[g]);
        out[gg.groups + g] = order_val(lmx[g]);
    }
}

// Partial extrema of each workgroup: part[wg][0..G) = min, part[wg][G..2G) = max.  (Letting the last
// workgroup to finish do the final step in the same launch was tried and dropped: the device-scope
// fence it needs flushes the per-XCD L2 once per workgroup, which costs far more than a second launch.)
template <typename T, int U>
__global__ __launch_bounds__(kThreads) void k_minmax_partial(const void *__restrict__ x, int64_t numel, GroupGeom gg,
                                                             float *__restrict__ part)
{
    extern __shared__ int lds_mm[];
    int *lmn = lds_mm;
    int *lmx = lds_mm + gg.groups;
    for (uint32_t g = threadIdx.x; g < gg.groups; g += kThreads) {
        lmn[g] = order_key(__builtin_inff());
        lmx[g] = order_key(-__builtin_inff());
    }
    __syncthreads();

    Cursor c[U];
    place_cursors<U>(c, gg, numel);
    MinMaxState<T> st[U];
#pragma unroll
    for (int u = 0; u < U; ++u) { st[u].cur = c[u].g; st[u].acc.init(); }

    constexpr int kChunk = kThreads * U * kVec;
    const int64_t stride = int64_t(gridDim.x) * kChunk;
    const int64_t toff = int64_t(threadIdx.x) * kVec;
    // CHECK = false: the chunk lies wholly inside the tensor, no per-vector bounds test
    auto chunk = [&](int64_t base, auto check) {
        constexpr bool CHECK = decltype(check)::value;
        typename Store<T>::raw_t v[U];
        bool full[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t e = base + u * (kThreads * kVec) + toff;
            full[u] = !CHECK || e + kVec <= numel;
            if (full[u]) v[u] = Nt<T>::load(x, e);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t e = base + u * (kThreads * kVec) + toff;
            const bool one = full[u] && c[u].rem + kVec <= gg.inner;
            const bool moved = one && c[u].g != st[u].cur;   // on to another group: hand the finished one to LDS
            if (__any(moved)) {                               // wave-uniform, rare
                flush_wave(lmn, lmx, moved, st[u].cur, st[u].acc.lo(), st[u].acc.hi());
                if (moved) {
                    st[u].cur = c[u].g;
                    st[u].acc.init();
                }
            }
            if (__builtin_expect(one, 1)) {
                st[u].acc.add(v[u]);
            } else if (full[u]) {   // crosses a slab end: element by element, from the registers
                float f[8];
                Store<T>::unpack(v[u], f);
#pragma unroll
                for (int j = 0; j < 8; ++j) minmax_element<T>(st[u], group_of(c[u], j, gg), f[j], lmn, lmx);
            } else if (e < numel) {   // the ragged end of the tensor, once per launch
                for (int j = 0; e + j < numel; ++j)
                    minmax_element<T>(st[u], group_of(c[u], j, gg), Store<T>::load1(x, e + j), lmn, lmx);
            }
            cursor_advance(c[u], gg);
        }
    };
    int64_t base = int64_t(blockIdx.x) * kChunk;
    for (; base + kChunk <= numel; base += stride) chunk(base, std::false_type());
    if (base < numel) chunk(base, std::true_type());   // the chunk that holds the end of the tensor
    minmax_finish<T, U>(st, lmn, lmx, part, gg);
}

// Few groups (at most GMAX) whose slabs are short and of awkward length -- a 49 x 49 window's attention
// map -- so that a thread meets another group at almost every step: instead of handing extrema to LDS
// whenever the group changes, every thread keeps running extrema for ALL groups (a select per group and
// vector) and nothing is flushed before the end.  Same partials as k_minmax_partial.
template <typename T, int U, int GMAX>
__global__ __launch_bounds__(kThreads) void k_minmax_partial_few(const void *__restrict__ x, int64_t numel, GroupGeom gg,
                                                                 float *__restrict__ part)
{
    extern __shared__ int lds_mm[];
    int *lmn = lds_mm;
    int *lmx = lds_mm + gg.groups;
    for (uint32_t g = threadIdx.x; g < gg.groups; g += kThreads) {
        lmn[g] = order_key(__builtin_inff());
        lmx[g] = order_key(-__builtin_inff());
    }
    __syncthreads();

    Cursor c[U];
    place_cursors<U>(c, gg, numel);
    MinMax<T> acc[GMAX];
#pragma unroll
    for (int k = 0; k < GMAX; ++k) acc[k].init();
    // a vector's (or an element's) own extrema go to the accumulator of group g, the others keep theirs
    auto merge = [&](uint32_t g, const MinMax<T> &m) {
#pragma unroll
        for (int k = 0; k < GMAX; ++k) {
            MinMax<T> t = acc[k];
            t.merge(m);
            if (g == uint32_t(k)) acc[k] = t;
        }
    };

    constexpr int kChunk = kThreads * U * kVec;
    const int64_t stride = int64_t(gridDim.x) * kChunk;
    const int64_t toff = int64_t(threadIdx.x) * kVec;
    auto chunk = [&](int64_t base, auto check) {
        constexpr bool CHECK = decltype(check)::value;
        typename Store<T>::raw_t v[U];
        bool full[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t e = base + u * (kThreads * kVec) + toff;
            full[u] = !CHECK || e + kVec <= numel;
            if (full[u]) v[u] = Nt<T>::load(x, e);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t e = base + u * (kThreads * kVec) + toff;
            if (full[u] && c[u].rem + kVec <= gg.inner) {
                MinMax<T> m;
                m.init();
                m.add(v[u]);
                merge(c[u].g, m);
            } else if (full[u]) {   // crosses a slab end: element by element, from the registers
                float f[8];
                Store<T>::unpack(v[u], f);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    MinMax<T> m;
                    m.init();
                    m.add1(f[j]);
                    merge(group_of(c[u], j, gg), m);
                }
            } else if (e < numel) {   // the ragged end of the tensor, once per launch
                for (int j = 0; e + j < numel; ++j) {
                    MinMax<T> m;
                    m.init();
                    m.add1(Store<T>::load1(x, e + j));
                    merge(group_of(c[u], j, gg), m);
                }
            }
            cursor_advance(c[u], gg);
        }
    };
    int64_t base = int64_t(blockIdx.x) * kChunk;
    for (; base + kChunk <= numel; base += stride) chunk(base, std::false_type());
    if (base < numel) chunk(base, std::true_type());

#pragma unroll
    for (int k = 0; k < GMAX; ++k) {
        if (uint32_t(k) < gg.groups) {
            float lo = acc[k].lo(), hi = acc[k].hi();
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) {
                lo = vmin(lo, __shfl_xor(lo, off, 64));
                hi = vmax(hi, __shfl_xor(hi, off, 64));
            }
            if ((threadIdx.x & 63) == 0) flush_lane(lmn, lmx, uint32_t(k), lo, hi);
        }
    }
    __syncthreads();
    float *out = part + int64_t(blockIdx.x) * 2 * gg.groups;
    for (uint32_t g = threadIdx.x; g < gg.groups; g += kThreads) {
        out[g] = order_val(lmn[g]);
        out[gg.groups + g] = order_val(lmx[g]);
    }
}

// Eq. (6)-(7) for one group from its extrema: each product, difference and sum rounded on its own.
// (alpha_old, beta_old: the running estimates as they were, read by the caller ahead of time)
__device__ __forceinline__ void ema_update(float mn, float mx, float alpha_old, float beta_old, float *alpha, float *beta,
                                           uint32_t g, float lambda, int first_call)
{
    mn = mn + 0.0f;  // -0.0 -> +0.0
    mx = mx + 0.0f;
    float range = mx - mn;
    if (first_call) {
        alpha[g] = range;
        beta[g] = mn;
    } else {
        float a = lambda * alpha_old;
        float b = 1.0f - lambda;
        float c = b * range;
        alpha[g] = a + c;
        float e = lambda * beta_old;
        float f = b * mn;
        beta[g] = e + f;
    }
}

// one workgroup per group: combine the partial extrema, then Eq. (6)-(7)
// variant kEmaSymmetric: the extrema are replaced by -m and +m, m = max |x| = max(-min, max);
// variant kEmaFixedBeta: the offset is beta_fixed, only alpha is a running estimate (of max - beta_fixed)
// variant kEmaScaleOnly: the scale-only symmetric scheme -- alpha is the running estimate of m = max |x|, beta is not touched
enum { kEmaPlain = 0, kEmaSymmetric = 1, kEmaFixedBeta = 2, kEmaScaleOnly = 3 };
__global__ __launch_bounds__(kThreads) void k_ema_finalize(const float *__restrict__ part, int nwg, uint32_t groups,
                                                           float *alpha, float *beta, float lambda, int first_call,
                                                           int variant = kEmaPlain, float beta_fixed = 0.0f)
{
    __shared__ float smn[kThreads / 64], smx[kThreads / 64];
    const uint32_t g = blockIdx.x;
    const float alpha_old = alpha[g], beta_old = variant == kEmaScaleOnly ? 0.0f : beta[g];   // in flight together with the partial extrema
    float mn = __builtin_inff(), mx = -__builtin_inff();
    for (int w = threadIdx.x; w < nwg; w += kThreads) {
        mn = vmin(mn, part[int64_t(w) * 2 * groups + g]);
        mx = vmax(mx, part[int64_t(w) * 2 * groups + groups + g]);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        mn = vmin(mn, __shfl_xor(mn, off, 64));
        mx = vmax(mx, __shfl_xor(mx, off, 64));
    }
    if ((threadIdx.x & 63) == 0) { smn[threadIdx.x >> 6] = mn; smx[threadIdx.x >> 6] = mx; }
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < kThreads / 64; ++w) { mn = vmin(mn, smn[w]); mx = vmax(mx, smx[w]); }
        if (variant == kEmaSymmetric) {
            mx = vmax(-mn, mx);
            mn = -mx;
        }
        if (variant == kEmaScaleOnly) {
            const float m = vmax(-mn, mx) + 0.0f;
            if (first_call) {
                alpha[g] = m;
            } else {
                float a = lambda * alpha_old;
                float b = 1.0f - lambda;
                float c = b * m;
                alpha[g] = a + c;
            }
        } else if (variant == kEmaFixedBeta) {
            ema_update(beta_fixed, mx, alpha_old, beta_old, alpha, beta, g, lambda, first_call);
            beta[g] = beta_fixed;
        } else {
            ema_update(mn, mx, alpha_old, beta_old, alpha, beta, g, lambda, first_call);
        }
    }
}

// per-element (scale, beta) of a vector whose elements do not all lie in one slab
__device__ __forceinline__ void params_of(const Cursor &c, const GroupGeom &gg, const float2 *tab, float2 p[8])
{
#pragma unroll
    for (int j = 0; j < 8; ++j) p[j] = tab[group_of(c, j, gg)];
}

template <typename T, int U, bool SR, bool SYM = false>
__global__ __launch_bounds__(kThreads) void k_quantize(const void *__restrict__ x, int8_t *__restrict__ q, int64_t numel,
                                                       GroupGeom gg, const float *__restrict__ alpha,
                                                       const float *__restrict__ beta, uint64_t seed, uint64_t offset)
{
    extern __shared__ float2 lds_tab[];
    constexpr int kChunk = kThreads * U * kVec;
    fill_table_touched<SYM ? Scale::QuantSym : Scale::Quant>(lds_tab, alpha, beta, gg, numel, kChunk);

    Cursor c[U];
    place_cursors<U>(c, gg, numel);
    const int64_t stride = int64_t(gridDim.x) * kChunk;
    const int64_t toff = int64_t(threadIdx.x) * kVec;
    // CHECK = false: the chunk lies wholly inside the tensor, no per-vector bounds test
    auto chunk = [&](int64_t base, auto check) {
        constexpr bool CHECK = decltype(check)::value;
        typename Store<T>::raw_t v[U];
        bool full[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t e = base + u * (kThreads * kVec) + toff;
            full[u] = !CHECK || e + kVec <= numel;
            if (full[u]) v[u] = Nt<T>::load(x, e);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t e = base + u * (kThreads * kVec) + toff;
            if (full[u]) {
                float f[8], w[8], bits[8];
                if (SR) sr_bits(seed, offset + uint64_t(e >> 3), bits);
                Store<T>::unpack(v[u], f);
                if (__builtin_expect(c[u].rem + kVec <= gg.inner, 1)) {
                    const float2 p = lds_tab[c[u].g];
#pragma unroll
                    for (int j = 0; j < 8; ++j) w[j] = quantize_one<SR, SYM>(f[j], p.x, p.y, SR ? bits[j] : 0.0f);
                } else {   // the vector crosses a slab end: parameters per element
                    float2 p[8];
                    params_of(c[u], gg, lds_tab, p);
#pragma unroll
                    for (int j = 0; j < 8; ++j) w[j] = quantize_one<SR, SYM>(f[j], p[j].x, p[j].y, SR ? bits[j] : 0.0f);
                }
                nt_store<u32x2>(q + e, pack_codes(w));
            } else if (e < numel) {   // the ragged end of the tensor, once per launch
                float bits[8];
                if (SR) sr_bits(seed, offset + uint64_t(e >> 3), bits);
                for (int j = 0; e + j < numel; ++j) {
                    const float2 p = lds_tab[group_of(c[u], j, gg)];
                    const float w = clamp_code(quantize_one<SR, SYM>(Store<T>::load1(x, e + j), p.x, p.y, SR ? bits[j] : 0.0f));
                    q[e + j] = int8_t(int(w) - 128);
                }
            }
            cursor_advance(c[u], gg);
        }
    };
    int64_t base = int64_t(blockIdx.x) * kChunk;
    for (; base + kChunk <= numel; base += stride) chunk(base, std::false_type());
    if (base < numel) chunk(base, std::true_type());   // the chunk that holds the end of the tensor
}

// Quantize and take the extrema in one pass over x: the loop of k_quantize with the bookkeeping of
// k_minmax_partial on the same registers.  Dynamic LDS: the (scale, beta) table, then the two
// ordered-int extrema tables.  Partials as k_minmax_partial writes them.
// gelu(x) = x * Phi(x), Phi(-|x|) = erfc(|x|/sqrt 2)/2 by Abramowitz & Stegun 7.1.26 (|error| <= 7.5e-8 on Phi;
// the coefficients below are the published ones halved).  With h = Phi(-|x|):  x >= 0: x - |x| h,  x < 0: -|x| h,
// i.e. max(x, 0) - |x| h in both cases.
__device__ __forceinline__ float gelu_value(float x)
{
    const float ax = fabsf(x);
    const float t = __builtin_amdgcn_rcpf(fmaf(ax, 0.3275911f * 0.70710678118654752f, 1.0f));
    float poly = fmaf(t, 0.5f * 1.061405429f, 0.5f * -1.453152027f);
    poly = fmaf(poly, t, 0.5f * 1.421413741f);
    poly = fmaf(poly, t, 0.5f * -0.284496736f);
    poly = fmaf(poly, t, 0.5f * 0.254829592f);
    const float h = (poly * t) * __builtin_amdgcn_exp2f(x * x * -0.72134752044448170f);   // Phi(-|x|)
    return fmaf(-ax, h, vmax(x, 0.0f));
}

// GELU_FWD: the kernel is a GELU layer's whole forward -- y = gelu(x) leaves in the same pass that takes the codes of x
template <typename T, int U, bool SR, bool GELU_FWD = false>
__global__ __launch_bounds__(kThreads) void k_quantize_minmax(const void *__restrict__ x, int8_t *__restrict__ q, int64_t numel,
                                                              GroupGeom gg, const float *__restrict__ alpha,
                                                              const float *__restrict__ beta, uint64_t seed, uint64_t offset,
                                                              float *__restrict__ part, void *__restrict__ y = nullptr)
{
    extern __shared__ float2 lds_tab[];
    int *lmn = reinterpret_cast<int *>(lds_tab + gg.groups);
    int *lmx = lmn + gg.groups;
    for (uint32_t g = threadIdx.x; g < gg.groups; g += kThreads) {
        lmn[g] = order_key(__builtin_inff());
        lmx[g] = order_key(-__builtin_inff());
    }
    fill_table<Scale::Quant>(lds_tab, alpha, beta, gg.groups);   // ends with a barrier

    Cursor c[U];
    place_cursors<U>(c, gg, numel);
    MinMaxState<T> st[U];
#pragma unroll
    for (int u = 0; u < U; ++u) { st[u].cur = c[u].g; st[u].acc.init(); }

    constexpr int kChunk = kThreads * U * kVec;
    const int64_t stride = int64_t(gridDim.x) * kChunk;
    const int64_t toff = int64_t(threadIdx.x) * kVec;
    auto chunk = [&](int64_t base, auto check) {
        constexpr bool CHECK = decltype(check)::value;
        typename Store<T>::raw_t v[U];
        bool full[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t e = base + u * (kThreads * kVec) + toff;
            full[u] = !CHECK || e + kVec <= numel;
            if (full[u]) v[u] = Nt<T>::load(x, e);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t e = base + u * (kThreads * kVec) + toff;
            const bool one = full[u] && c[u].rem + kVec <= gg.inner;
            const bool moved = one && c[u].g != st[u].cur;
            if (__any(moved)) {
                flush_wave(lmn, lmx, moved, st[u].cur, st[u].acc.lo(), st[u].acc.hi());
                if (moved) {
                    st[u].cur = c[u].g;
                    st[u].acc.init();
                }
            }
            if (full[u]) {
                float f[8], w[8], bits[8];
                if (SR) sr_bits(seed, offset + uint64_t(e >> 3), bits);
                Store<T>::unpack(v[u], f);
                if (GELU_FWD) {
                    float yv[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) yv[j] = gelu_value(f[j]);
                    Nt<T>::store(y, e, Store<T>::pack(yv));
                }
                if (__builtin_expect(one, 1)) {
                    st[u].acc.add(v[u]);
                    const float2 p = lds_tab[c[u].g];
#pragma unroll
                    for (int j = 0; j < 8; ++j) w[j] = quantize_one<SR>(f[j], p.x, p.y, SR ? bits[j] : 0.0f);
                } else {   // the vector crosses a slab end: group and parameters per element
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const uint32_t g = group_of(c[u], j, gg);
                        minmax_element<T>(st[u], g, f[j], lmn, lmx);
                        const float2 p = lds_tab[g];
                        w[j] = quantize_one<SR>(f[j], p.x, p.y, SR ? bits[j] : 0.0f);
                    }
                }
                nt_store<u32x2>(q + e, pack_codes(w));
            } else if (e < numel) {   // the ragged end of the tensor, once per launch
                float bits[8];
                if (SR) sr_bits(seed, offset + uint64_t(e >> 3), bits);
                for (int j = 0; e + j < numel; ++j) {
                    const uint32_t g = group_of(c[u], j, gg);
                    const float xv = Store<T>::load1(x, e + j);
                    if (GELU_FWD) Store<T>::store1(y, e + j, gelu_value(xv));
                    minmax_element<T>(st[u], g, xv, lmn, lmx);
                    const float2 p = lds_tab[g];
                    const float w = clamp_code(quantize_one<SR>(xv, p.x, p.y, SR ? bits[j] : 0.0f));
                    q[e + j] = int8_t(int(w) - 128);
                }
            }
            cursor_advance(c[u], gg);
        }
    };
    int64_t base = int64_t(blockIdx.x) * kChunk;
    for (; base + kChunk <= numel; base += stride) chunk(base, std::false_type());
    if (base < numel) chunk(base, std::true_type());
    minmax_finish<T, U>(st, lmn, lmx, part, gg);
}

// ---------------------------------------------------------------------------------------------
// de-quantize
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float dequant_exact(float u, float s, float b)
{
    float xh = u * s;
    xh = xh + b;
    return xh;
}
// scale-only symmetric scheme: x_hat = q * (m / 127); u = q + 128 as the code bytes unpack
__device__ __forceinline__ float dequant_sym(float u, float s) { return (u - 128.0f) * s; }

template <typename T, int U, bool SYM = false>
__global__ __launch_bounds__(kThreads) void k_dequantize(const int8_t *__restrict__ q, void *__restrict__ xh, int64_t numel,
                                                         GroupGeom gg, const float *__restrict__ alpha,
                                                         const float *__restrict__ beta)
{
    extern __shared__ float2 lds_tab[];
    constexpr int kChunk = kThreads * U * kVec;
    fill_table_touched<SYM ? Scale::DequantSym : Scale::Dequant>(lds_tab, alpha, beta, gg, numel, kChunk);

    Cursor c[U];
    place_cursors<U>(c, gg, numel);
    const int64_t stride = int64_t(gridDim.x) * kChunk;
    const int64_t toff = int64_t(threadIdx.x) * kVec;
    // CHECK = false: the chunk lies wholly inside the tensor, no per-vector bounds test
    auto chunk = [&](int64_t base, auto check) {
        constexpr bool CHECK = decltype(check)::value;
        u32x2 v[U];
        bool full[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t e = base + u * (kThreads * kVec) + toff;
            full[u] = !CHECK || e + kVec <= numel;
            if (full[u]) v[u] = nt_load<u32x2>(q + e);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t e = base + u * (kThreads * kVec) + toff;
            if (full[u]) {
                float uu[8], f[8];
                codes_to_float(v[u], uu);
                if (__builtin_expect(c[u].rem + kVec <= gg.inner, 1)) {
                    const float2 p = lds_tab[c[u].g];
#pragma unroll
                    for (int j = 0; j < 8; ++j) f[j] = (SYM ? dequant_sym(uu[j], p.x) : dequant_exact(uu[j], p.x, p.y));
                } else {
                    float2 p[8];
                    params_of(c[u], gg, lds_tab, p);
#pragma unroll
                    for (int j = 0; j < 8; ++j) f[j] = (SYM ? dequant_sym(uu[j], p[j].x) : dequant_exact(uu[j], p[j].x, p[j].y));
                }
                Nt<T>::store(xh, e, Store<T>::pack(f));
            } else if (e < numel) {
                for (int j = 0; e + j < numel; ++j) {
                    const float2 p = lds_tab[group_of(c[u], j, gg)];
                    Store<T>::store1(xh, e + j, (SYM ? dequant_sym(code_to_float(q[e + j]), p.x) : dequant_exact(code_to_float(q[e + j]), p.x, p.y)));
                }
            }
            cursor_advance(c[u], gg);
        }
    };
    int64_t base = int64_t(blockIdx.x) * kChunk;
    for (; base + kChunk <= numel; base += stride) chunk(base, std::false_type());
    if (base < numel) chunk(base, std::true_type());   // the chunk that holds the end of the tensor
}

// ---------------------------------------------------------------------------------------------
// GELU backward at x_hat
// ---------------------------------------------------------------------------------------------
// gelu'(x) = Phi(x) + x*phi(x).  With E = exp(-x^2/2):  phi = E/sqrt(2 pi) and
// Phi(-|x|) = erfc(|x|/sqrt 2)/2 = P(t)*E/2, t = 1/(1 + p|x|/sqrt 2), P the degree-5 polynomial of
// Abramowitz & Stegun 7.1.26 (|error| <= 1.5e-7 on erf): one exponential serves both terms.
__device__ __forceinline__ float gelu_grad(float x)
{
    float ax = fabsf(x);
    float t = __builtin_amdgcn_rcpf(fmaf(ax, 0.3275911f * 0.70710678118654752f, 1.0f));
    float poly = fmaf(t, 1.061405429f, -1.453152027f);
    poly = fmaf(poly, t, 1.421413741f);
    poly = fmaf(poly, t, -0.284496736f);
    poly = fmaf(poly, t, 0.254829592f);
    poly = poly * t;
    float E = __builtin_amdgcn_exp2f(x * x * -0.72134752044448170f);  // exp(-x^2/2)
    float h = 0.5f * poly * E;
    float cdf = (x >= 0.0f) ? 1.0f - h : h;
    return fmaf(x * E, 0.39894228040143268f, cdf);
}

// The derivative of the activation at x_hat = x_bar*step + beta.  GELU: smooth, the fused form of x_hat will do
// (tolerance-checked).  ReLU: a 0/1 decision, taken on the separately rounded x_hat that mesa_dequantize returns.
enum { kActGelu = 0, kActRelu = 1 };
template <int ACT> __device__ __forceinline__ float act_grad(float x_bar, float step, float beta)
{
    if (ACT == kActRelu) return dequant_exact(x_bar, step, beta) > 0.0f ? 1.0f : 0.0f;
    return gelu_grad(fmaf(x_bar, step, beta));
}

// x_hat takes only 256 values per group, so gelu'(x_hat) is a table of groups*256 entries: each
// workgroup fills it once (indexed by the raw code byte) and the stream becomes one LDS gather and
// one multiply per element.  With more than kLutMaxGroups groups the table does not fit and the
// derivative is evaluated per element instead (LUT = false).
template <typename T, int U, bool LUT, int ACT = kActGelu>
__global__ __launch_bounds__(kThreads) void k_gelu_bwd(const int8_t *__restrict__ q, const void *dy, void *dx, int64_t numel,
                                                       GroupGeom gg, const float *__restrict__ alpha,
                                                       const float *__restrict__ beta)
{
    extern __shared__ float lds_gelu[];
    float2 *tab2 = reinterpret_cast<float2 *>(lds_gelu);   // LUT = false: (step, beta) per group
    if (LUT) {
        for (uint32_t i = threadIdx.x; i < gg.groups * 256u; i += kThreads) {
            const uint32_t g = i >> 8;
            const float u = float((i & 255u) ^ 0x80u);   // raw byte -> x_bar
            lds_gelu[i] = act_grad<ACT>(u, alpha[g] / 255.0f, beta[g]);
        }
        __syncthreads();
    } else {
        fill_table_touched<Scale::Dequant>(tab2, alpha, beta, gg, numel, int64_t(kThreads) * U * kVec);
    }

    auto grad_of = [&](uint32_t g, uint32_t raw) -> float {
        if (LUT) return lds_gelu[g * 256u + raw];
        const float2 p = tab2[g];
        return act_grad<ACT>(float(raw ^ 0x80u), p.x, p.y);
    };

    Cursor c[U];
    place_cursors<U>(c, gg, numel);
    constexpr int kChunk = kThreads * U * kVec;
    const int64_t stride = int64_t(gridDim.x) * kChunk;
    const int64_t toff = int64_t(threadIdx.x) * kVec;
    // CHECK = false: the chunk lies wholly inside the tensor, no per-vector bounds test
    auto chunk = [&](int64_t base, auto check) {
        constexpr bool CHECK = decltype(check)::value;
        u32x2 v[U];
        typename Store<T>::raw_t d[U];
        bool full[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t e = base + u * (kThreads * kVec) + toff;
            full[u] = !CHECK || e + kVec <= numel;
            if (full[u]) {
                v[u] = nt_load<u32x2>(q + e);
                d[u] = Nt<T>::load(dy, e);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t e = base + u * (kThreads * kVec) + toff;
            if (full[u]) {
                float g[8];
                Store<T>::unpack(d[u], g);
                if (__builtin_expect(c[u].rem + kVec <= gg.inner, 1)) {
                    if (LUT) {
                        const float *row = lds_gelu + c[u].g * 256u;
#pragma unroll
                        for (int j = 0; j < 8; ++j) g[j] = g[j] * row[(v[u][j >> 2] >> (8 * (j & 3))) & 0xFFu];
                    } else {
                        const float2 p = tab2[c[u].g];
                        float uu[8];
                        codes_to_float(v[u], uu);
#pragma unroll
                        for (int j = 0; j < 8; ++j) g[j] = g[j] * act_grad<ACT>(uu[j], p.x, p.y);
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        g[j] = g[j] * grad_of(group_of(c[u], j, gg), (v[u][j >> 2] >> (8 * (j & 3))) & 0xFFu);
                }
                Nt<T>::store(dx, e, Store<T>::pack(g));
            } else if (e < numel) {
                for (int j = 0; e + j < numel; ++j)
                    Store<T>::store1(dx, e + j, Store<T>::load1(dy, e + j) *
                                                    grad_of(group_of(c[u], j, gg), uint32_t(uint8_t(q[e + j]))));
            }
            cursor_advance(c[u], gg);
        }
    };
    int64_t base = int64_t(blockIdx.x) * kChunk;
    for (; base + kChunk <= numel; base += stride) chunk(base, std::false_type());
    if (base < numel) chunk(base, std::true_type());   // the chunk that holds the end of the tensor
}

// ---------------------------------------------------------------------------------------------
// plain copy (measurement)
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void k_copy(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, int64_t n16)
{
    const int64_t chunk = kThreads * 4;
    for (int64_t base = int64_t(blockIdx.x) * chunk; base < n16; base += int64_t(gridDim.x) * chunk) {
        u32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t i = base + u * kThreads + threadIdx.x;
            if (i < n16) v[u] = nt_load<u32x4>(src + i);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t i = base + u * kThreads + threadIdx.x;
            if (i < n16) nt_store<u32x4>(dst + i, v[u]);
        }
    }
}


// read-only and write-only probes: what the memory system delivers in one direction alone.  The read probe
// folds what it loads into one word per thread and stores it only if it is a value no fold of the caller's
// data produces twice in a row (the store exists so that the loads cannot be dropped; it moves 4 bytes a thread).
__global__ __launch_bounds__(kThreads) void k_read_probe(const u32x4 *__restrict__ src, int64_t n16, uint32_t *__restrict__ sink)
{
    const int64_t chunk = kThreads * 4;
    uint32_t acc = 0u;
    for (int64_t base = int64_t(blockIdx.x) * chunk; base < n16; base += int64_t(gridDim.x) * chunk) {
        u32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t i = base + u * kThreads + threadIdx.x;
            v[u] = (i < n16) ? nt_load<u32x4>(src + i) : u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) acc ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
    }
    if (acc == 0x9E3779B9u) sink[0] = acc;
}

__global__ __launch_bounds__(kThreads) void k_fill_probe(u32x4 *__restrict__ dst, int64_t n16, uint32_t word)
{
    const int64_t chunk = kThreads * 4;
    const u32x4 v = {word, word, word, word};
    for (int64_t base = int64_t(blockIdx.x) * chunk; base < n16; base += int64_t(gridDim.x) * chunk) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t i = base + u * kThreads + threadIdx.x;
            if (i < n16) nt_store<u32x4>(dst + i, v);
        }
    }
}

void launch_ema_finalize(const float *part, int nwg, uint32_t groups, float *alpha, float *beta, float lambda, int first_call,
                         int variant, float beta_fixed, hipStream_t stream)
{
    hipLaunchKernelGGL(k_ema_finalize, dim3(groups), dim3(kThreads), 0, stream, part, nwg, groups, alpha, beta, lambda, first_call,
                       variant, beta_fixed);
}

}  // namespace mesa

// =================================================================================================
// entry points
// =================================================================================================
using namespace mesa;

// min_chunks: how many chunks a workgroup should move at the very least (a kernel that builds a table per workgroup
// wants the table paid for by more than one chunk)
static int stream_grid(int64_t numel, int64_t row, int min_chunks = 1)
{
    const int64_t chunk = int64_t(kThreads) * kU * kVec;
    int64_t cap = kGridCap;
    if (min_chunks > 1) {
        const int64_t fit = numel / (chunk * min_chunks);
        if (fit < cap) cap = fit < 256 ? 256 : fit;
    }
    return plan_grid(numel, chunk, int(cap), row);
}

// grid of a kernel that tracks extrema with `unroll` vectors per thread and at most `grid_cap` workgroups
// max_wgs > 0: never more workgroups than that (a caller with a fixed amount of scratch)
static int minmax_grid(const mesa_layout &L, int unroll = kMmU, int grid_cap = kMmGridCap, int max_wgs = 0)
{
    int64_t numel = layout_numel(L);
    // many groups: every workgroup writes 2*groups partial values (8 bytes per group), so keep their number down -- to
    // what the tensor pays for: the partial values stay below an eighth of an element's byte per element.  (A fixed
    // 64 / groups of the cap left the per-sample layout (1, 3072, 38809) with 32 workgroups: 1.04 ms for 238 MB.)
    int cap = grid_cap;
    if (L.groups > 64) {
        const int64_t fixed = int64_t(grid_cap) * 64 / L.groups, paid = numel / (64 * L.groups);
        int64_t c = fixed > paid ? fixed : paid;
        if (c < 32) c = 32;
        if (c < cap) cap = int(c);
    }
    if (max_wgs > 0 && cap > max_wgs) cap = max_wgs;
    const int64_t chunk = int64_t(kThreads) * unroll * kVec;
    int n = plan_grid(numel, chunk, cap, L.groups > 1 ? L.groups * L.inner : 0);
    // Long slabs (head-wise tensors): a thread hands its extrema to LDS whenever its group changes,
    // so pick a grid whose step is a whole number of group cycles plus a small remainder -- then a
    // thread stays with one head for many iterations instead of meeting a new one every time.
    const int64_t row = L.groups * L.inner;
    if (L.groups > 1 && L.inner > chunk && ceil_div(numel, chunk) > n) {
        int best = n;
        int64_t best_rem = (int64_t(n) * chunk) % row;
        const int k_end = max_wgs > 0 && n + 256 > max_wgs + 1 ? max_wgs + 1 : n + 256;
        for (int k = n + 1; k < k_end && best_rem >= L.inner / 16; ++k) {
            const int64_t rem = (int64_t(k) * chunk) % row;
            if (rem < best_rem) { best_rem = rem; best = k; }
        }
        n = best;
    }
    return n;
}

// True when a thread of the min/max scan would meet another group at almost every step of the grid:
// few groups, and the grid's step is neither a whole number of group cycles nor close to one.
static bool minmax_few_groups(const mesa_layout &L, int grid, int unroll)
{
    if (L.groups < 2 || L.groups > kMmFew) return false;
    const int64_t row = L.groups * L.inner;
    const int64_t step = (int64_t(grid) * kThreads * unroll * kVec) % row;
    const int64_t off = step < row - step ? step : row - step;   // how far a step lands from where it started, in the cycle
    return off > L.inner / 16;
}

// max_wgs > 0: the scan runs on at most that many workgroups and the workspace need only hold their partial values
static mesa_status update_running_params(const void *x, mesa_dtype dt, mesa_layout L, float *alpha, float *beta, float lambda,
                                         int first_call, int variant, float beta_fixed, void *ws, size_t ws_bytes, void *stream,
                                         int max_wgs = 0)
{
    if (!valid_dtype(dt)) return MESA_ERR_INVALID_ARG;
    mesa_status st = check_layout(L);
    if (st != MESA_OK) return st;
    if (!(lambda >= 0.0f && lambda <= 1.0f)) return MESA_ERR_INVALID_ARG;
    const int64_t numel = layout_numel(L);
    if (numel == 0) return MESA_OK;
    if (!x || !alpha || !aligned16(x) || !aligned4(alpha)) return MESA_ERR_INVALID_ARG;
    if (variant != kEmaScaleOnly && (!beta || !aligned4(beta))) return MESA_ERR_INVALID_ARG;
    const int grid = minmax_grid(L, kMmU, kMmGridCap, max_wgs);
    const size_t need = max_wgs > 0 ? size_t(grid) * 2 * size_t(L.groups) * sizeof(float) : update_ws_bytes(L.outer, L.groups, L.inner);
    if (!ws || !aligned16(ws) || ws_bytes < need) return MESA_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    GroupGeom gg = make_geom(L.groups, L.inner, int64_t(grid) * kThreads * kMmU * kVec);
    const size_t lds = size_t(2) * gg.groups * sizeof(int);
    float *part = static_cast<float *>(ws);
    if (minmax_few_groups(L, grid, kMmU)) {
#define MESA_LAUNCH_FEW(T, GM) \
    hipLaunchKernelGGL((k_minmax_partial_few<T, kMmU, GM>), dim3(grid), dim3(kThreads), lds, s, x, numel, gg, part)
#define MESA_LAUNCH_FEW_T(T) \
    do { \
        if (L.groups <= 2) MESA_LAUNCH_FEW(T, 2); \
        else if (L.groups == 3) MESA_LAUNCH_FEW(T, 3); \
        else if (L.groups == 4) MESA_LAUNCH_FEW(T, 4); \
        else if (L.groups <= 6) MESA_LAUNCH_FEW(T, 6); \
        else MESA_LAUNCH_FEW(T, 8); \
    } while (0)
        MESA_FOR_DTYPE(dt, MESA_LAUNCH_FEW_T);
#undef MESA_LAUNCH_FEW_T
#undef MESA_LAUNCH_FEW
    } else {
#define MESA_LAUNCH_MM(T) hipLaunchKernelGGL((k_minmax_partial<T, kMmU>), dim3(grid), dim3(kThreads), lds, s, x, numel, gg, part)
        MESA_FOR_DTYPE(dt, MESA_LAUNCH_MM);
#undef MESA_LAUNCH_MM
    }
    if (launch_status() != MESA_OK) return MESA_ERR_LAUNCH;   // the consumer must not run on partials nobody wrote
    hipLaunchKernelGGL(k_ema_finalize, dim3(gg.groups), dim3(kThreads), 0, s, part, grid, gg.groups, alpha, beta, lambda,
                       first_call, variant, beta_fixed);
    return launch_status();
}

extern "C" MESA_EXPORT mesa_status mesa_update_running_params(const void *x, mesa_dtype dt, mesa_layout L, float *alpha, float *beta,
                                                  float lambda, int first_call, void *ws, size_t ws_bytes, void *stream)
{
    return update_running_params(x, dt, L, alpha, beta, lambda, first_call, kEmaPlain, 0.0f, ws, ws_bytes, stream);
}

extern "C" MESA_EXPORT mesa_status mesa_update_running_params_sym(const void *x, mesa_dtype dt, mesa_layout L, float *alpha,
                                                      float *beta, float lambda, int first_call, void *ws, size_t ws_bytes,
                                                      void *stream)
{
    return update_running_params(x, dt, L, alpha, beta, lambda, first_call, kEmaSymmetric, 0.0f, ws, ws_bytes, stream);
}

extern "C" MESA_EXPORT mesa_status mesa_update_running_params_fixed_beta(const void *x, mesa_dtype dt, mesa_layout L, float *alpha,
                                                             float *beta, float lambda, int first_call, float beta_fixed,
                                                             void *ws, size_t ws_bytes, void *stream)
{
    if (!(beta_fixed == beta_fixed) || beta_fixed - beta_fixed != 0.0f) return MESA_ERR_INVALID_ARG;   // NaN or infinite
    return update_running_params(x, dt, L, alpha, beta, lambda, first_call, kEmaFixedBeta, beta_fixed, ws, ws_bytes, stream);
}

// ---- the running-estimate update for callers that cannot allocate device memory -----------------
// The partial extrema go to a file-scope device array instead of a caller's workspace.  The array's
// name is a host-side stand-in, not a device address: host code asks the runtime for the address
// once per device (with that device current) and hands the kernels that pointer.
constexpr size_t kStaticScratchBytes = size_t(1) << 20;
constexpr int kStaticMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static std::atomic<void *> g_scratch_ptr[kStaticMaxDevices];

// device address of `scratch` on the current device; nullptr when the runtime cannot tell
static void *static_scratch_ptr()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kStaticMaxDevices) return nullptr;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p) return p;
    void *q = nullptr;
    if (hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)) != hipSuccess || !q) return nullptr;
    g_scratch_ptr[dev].store(q, std::memory_order_release);   // every thread finds the same address: a benign race
    return q;
}

extern "C" MESA_EXPORT mesa_status mesa_update_running_params_static(const void *x, mesa_dtype dt, mesa_layout L, float *alpha,
                                                                     float *beta, float lambda, int first_call, void *stream)
{
    // the argument checks come first, so that a bad call reports the same status as the workspace form
    if (!valid_dtype(dt)) return MESA_ERR_INVALID_ARG;
    mesa_status st = check_layout(L);
    if (st != MESA_OK) return st;
    if (!(lambda >= 0.0f && lambda <= 1.0f)) return MESA_ERR_INVALID_ARG;
    if (layout_numel(L) == 0) return MESA_OK;
    // as many workgroups as the array has room for (2 * groups partial values each), and no fewer than the scan's minimum of 32
    const int max_wgs = int(kStaticScratchBytes / (size_t(2) * size_t(L.groups < 1 ? 1 : L.groups) * sizeof(float)));
    if (max_wgs < 32) return MESA_ERR_UNSUPPORTED;          // groups > 4096
    void *ws = static_scratch_ptr();
    if (!ws) return MESA_ERR_LAUNCH;
    // every workgroup overwrites its whole row of partial extrema before the second kernel reads
    // them, so nothing of the previous call's contents is ever read and nothing needs clearing
    return update_running_params(x, dt, L, alpha, beta, lambda, first_call, kEmaPlain, 0.0f, ws, kStaticScratchBytes, stream, max_wgs);
}

extern "C" MESA_EXPORT size_t mesa_static_scratch_bytes(void) { return kStaticScratchBytes; }

// sym: the scale-only symmetric scheme (alpha holds m, beta is absent)
static mesa_status quantize(const void *x, mesa_dtype dt, mesa_layout L, const float *alpha, const float *beta, int8_t *q,
                            mesa_round mode, uint64_t seed, uint64_t offset, bool sym, void *stream)
{
    if (!valid_dtype(dt) || (mode != MESA_ROUND_NEAREST_EVEN && mode != MESA_ROUND_STOCHASTIC)) return MESA_ERR_INVALID_ARG;
    mesa_status st = check_layout(L);
    if (st != MESA_OK) return st;
    const int64_t numel = layout_numel(L);
    if (numel == 0) return MESA_OK;
    if (!x || !q || !alpha || !aligned16(x) || !aligned16(q) || !aligned4(alpha)) return MESA_ERR_INVALID_ARG;
    if (!sym && (!beta || !aligned4(beta))) return MESA_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int grid = stream_grid(numel, L.groups > 1 ? L.groups * L.inner : 0);
    GroupGeom gg = make_geom(L.groups, L.inner, int64_t(grid) * kThreads * kU * kVec);
    const size_t lds = size_t(gg.groups) * sizeof(float2);
    const bool sr = mode == MESA_ROUND_STOCHASTIC;
#define MESA_LAUNCH_Q(T, SRF, SYMF) \
    hipLaunchKernelGGL((k_quantize<T, kU, SRF, SYMF>), dim3(grid), dim3(kThreads), lds, s, x, q, numel, gg, alpha, beta, seed, offset)
#define MESA_LAUNCH_Q_T(T) \
    do { \
        if (sym) { if (sr) MESA_LAUNCH_Q(T, true, true); else MESA_LAUNCH_Q(T, false, true); } \
        else { if (sr) MESA_LAUNCH_Q(T, true, false); else MESA_LAUNCH_Q(T, false, false); } \
    } while (0)
    MESA_FOR_DTYPE(dt, MESA_LAUNCH_Q_T);
#undef MESA_LAUNCH_Q_T
#undef MESA_LAUNCH_Q
    return launch_status();
}

extern "C" MESA_EXPORT mesa_status mesa_quantize_headwise(const void *x, mesa_dtype dt, mesa_layout L, const float *alpha,
                                              const float *beta, int8_t *q, mesa_round mode, uint64_t seed, uint64_t offset,
                                              void *stream)
{
    return quantize(x, dt, L, alpha, beta, q, mode, seed, offset, false, stream);
}

extern "C" MESA_EXPORT mesa_status mesa_quantize_sym(const void *x, mesa_dtype dt, mesa_layout L, const float *m, int8_t *q,
                                                     mesa_round mode, uint64_t seed, uint64_t offset, void *stream)
{
    return quantize(x, dt, L, m, nullptr, q, mode, seed, offset, true, stream);
}

extern "C" MESA_EXPORT mesa_status mesa_update_running_scale_sym(const void *x, mesa_dtype dt, mesa_layout L, float *m, float lambda,
                                                                 int first_call, void *ws, size_t ws_bytes, void *stream)
{
    return update_running_params(x, dt, L, m, nullptr, lambda, first_call, kEmaScaleOnly, 0.0f, ws, ws_bytes, stream);
}

// the single-pass forward, optionally with the layer's own output: gelu_fwd: y = gelu(x) leaves in the same pass
static mesa_status quantize_update_fused(const void *x, mesa_dtype dt, mesa_layout L, float *alpha, float *beta, float lambda,
                                         bool gelu_fwd, void *y, int8_t *q, mesa_round mode, uint64_t seed, uint64_t offset,
                                         void *ws, size_t ws_bytes, void *stream)
{
    if (!valid_dtype(dt) || (mode != MESA_ROUND_NEAREST_EVEN && mode != MESA_ROUND_STOCHASTIC)) return MESA_ERR_INVALID_ARG;
    mesa_status st = check_layout(L);
    if (st != MESA_OK) return st;
    if (!(lambda >= 0.0f && lambda <= 1.0f)) return MESA_ERR_INVALID_ARG;
    const int64_t numel = layout_numel(L);
    if (numel == 0) return MESA_OK;
    if (!x || !q || !alpha || !beta || !aligned16(x) || !aligned16(q) || !aligned4(alpha) || !aligned4(beta))
        return MESA_ERR_INVALID_ARG;
    if (gelu_fwd && (!y || !aligned16(y) || y == x)) return MESA_ERR_INVALID_ARG;   // not in place: the kernel's pointers do not alias
    if (!gelu_fwd) y = nullptr;
    if (!ws || !aligned16(ws) || ws_bytes < update_ws_bytes(L.outer, L.groups, L.inner)) return MESA_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int grid = minmax_grid(L, kFuU, kFuGridCap);
    GroupGeom gg = make_geom(L.groups, L.inner, int64_t(grid) * kThreads * kFuU * kVec);
    const size_t lds = size_t(gg.groups) * (sizeof(float2) + 2 * sizeof(int));
    float *part = static_cast<float *>(ws);
    const bool sr = mode == MESA_ROUND_STOCHASTIC;
    // parameter table and extrema of every group live in LDS, 16 bytes a group: beyond the 64 KiB a launch gets by default
    // (more than 4096 groups, up to the layout's limit of 8192: 128 KiB) the kernel is given leave for more
#define MESA_LAUNCH_QM(T, SRF, GF) \
    do { \
        auto kern = k_quantize_minmax<T, kFuU, SRF, GF>; \
        if (lds > size_t(64) * 1024 && \
            hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, int(lds)) != hipSuccess) \
            return MESA_ERR_LAUNCH; \
        hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), lds, s, x, q, numel, gg, alpha, beta, seed, offset, part, y); \
    } while (0)
#define MESA_LAUNCH_QM_T(T) \
    do { \
        if (y) { if (sr) MESA_LAUNCH_QM(T, true, true); else MESA_LAUNCH_QM(T, false, true); } \
        else { if (sr) MESA_LAUNCH_QM(T, true, false); else MESA_LAUNCH_QM(T, false, false); } \
    } while (0)
    MESA_FOR_DTYPE(dt, MESA_LAUNCH_QM_T);
#undef MESA_LAUNCH_QM_T
#undef MESA_LAUNCH_QM
    if (launch_status() != MESA_OK) return MESA_ERR_LAUNCH;
    hipLaunchKernelGGL(k_ema_finalize, dim3(gg.groups), dim3(kThreads), 0, s, part, grid, gg.groups, alpha, beta, lambda, 0);
    return launch_status();
}

extern "C" MESA_EXPORT mesa_status mesa_quantize_update_fused(const void *x, mesa_dtype dt, mesa_layout L, float *alpha, float *beta,
                                                              float lambda, int8_t *q, mesa_round mode, uint64_t seed,
                                                              uint64_t offset, void *ws, size_t ws_bytes, void *stream)
{
    return quantize_update_fused(x, dt, L, alpha, beta, lambda, false, nullptr, q, mode, seed, offset, ws, ws_bytes, stream);
}

extern "C" MESA_EXPORT mesa_status mesa_gelu_fwd_q(const void *x, mesa_dtype dt, mesa_layout L, float *alpha, float *beta,
                                                   float lambda, void *y, int8_t *q, mesa_round mode, uint64_t seed,
                                                   uint64_t offset, void *ws, size_t ws_bytes, void *stream)
{
    return quantize_update_fused(x, dt, L, alpha, beta, lambda, true, y, q, mode, seed, offset, ws, ws_bytes, stream);
}

static mesa_status dequantize(const int8_t *q, mesa_layout L, const float *alpha, const float *beta, void *x_hat, mesa_dtype dt,
                              bool sym, void *stream)
{
    if (!valid_dtype(dt)) return MESA_ERR_INVALID_ARG;
    mesa_status st = check_layout(L);
    if (st != MESA_OK) return st;
    const int64_t numel = layout_numel(L);
    if (numel == 0) return MESA_OK;
    if (!q || !x_hat || !alpha || !aligned16(q) || !aligned16(x_hat) || !aligned4(alpha)) return MESA_ERR_INVALID_ARG;
    if (!sym && (!beta || !aligned4(beta))) return MESA_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int grid = stream_grid(numel, L.groups > 1 ? L.groups * L.inner : 0);
    GroupGeom gg = make_geom(L.groups, L.inner, int64_t(grid) * kThreads * kU * kVec);
    const size_t lds = size_t(gg.groups) * sizeof(float2);
#define MESA_LAUNCH_DQ(T) \
    do { \
        if (sym) hipLaunchKernelGGL((k_dequantize<T, kU, true>), dim3(grid), dim3(kThreads), lds, s, q, x_hat, numel, gg, alpha, beta); \
        else hipLaunchKernelGGL((k_dequantize<T, kU, false>), dim3(grid), dim3(kThreads), lds, s, q, x_hat, numel, gg, alpha, beta); \
    } while (0)
    MESA_FOR_DTYPE(dt, MESA_LAUNCH_DQ);
#undef MESA_LAUNCH_DQ
    return launch_status();
}

extern "C" MESA_EXPORT mesa_status mesa_dequantize(const int8_t *q, mesa_layout L, const float *alpha, const float *beta, void *x_hat,
                                       mesa_dtype dt, void *stream)
{
    return dequantize(q, L, alpha, beta, x_hat, dt, false, stream);
}

extern "C" MESA_EXPORT mesa_status mesa_dequantize_sym(const int8_t *q, mesa_layout L, const float *m, void *x_hat, mesa_dtype dt,
                                                       void *stream)
{
    return dequantize(q, L, m, nullptr, x_hat, dt, true, stream);
}

template <int ACT>
static mesa_status act_bwd_q(const int8_t *xq, mesa_layout L, const float *alpha, const float *beta, const void *dy, void *dx,
                             mesa_dtype dt, void *stream)
{
    if (!valid_dtype(dt)) return MESA_ERR_INVALID_ARG;
    mesa_status st = check_layout(L);
    if (st != MESA_OK) return st;
    const int64_t numel = layout_numel(L);
    if (numel == 0) return MESA_OK;
    if (!xq || !dy || !dx || !alpha || !beta || !aligned16(xq) || !aligned16(dy) || !aligned16(dx) || !aligned4(alpha) ||
        !aligned4(beta))
        return MESA_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool lut_fits = (L.groups <= 1 ? 1 : L.groups) <= kLutMaxGroups;
    // the table of a workgroup is paid for by two chunks, by four on the large tensors (measured: 2 / 4 / 8 chunks give
    // 0.61 / 0.71 / 0.71 of the HBM peak at 134 M elements, 0.65 / 0.63 / 0.62 at 39 M)
    const int grid = stream_grid(numel, L.groups > 1 ? L.groups * L.inner : 0, !lut_fits ? 1 : numel >= (int64_t(1) << 26) ? 4 : 2);
    GroupGeom gg = make_geom(L.groups, L.inner, int64_t(grid) * kThreads * kU * kVec);
    const bool lut = gg.groups <= uint32_t(kLutMaxGroups);
    const size_t lds = lut ? size_t(gg.groups) * 256 * sizeof(float) : size_t(gg.groups) * sizeof(float2);
#define MESA_LAUNCH_G(T, L_) \
    hipLaunchKernelGGL((k_gelu_bwd<T, kU, L_, ACT>), dim3(grid), dim3(kThreads), lds, s, xq, dy, dx, numel, gg, alpha, beta)
#define MESA_LAUNCH_G_T(T) do { if (lut) MESA_LAUNCH_G(T, true); else MESA_LAUNCH_G(T, false); } while (0)
    MESA_FOR_DTYPE(dt, MESA_LAUNCH_G_T);
#undef MESA_LAUNCH_G_T
#undef MESA_LAUNCH_G
    return launch_status();
}

extern "C" MESA_EXPORT mesa_status mesa_gelu_bwd_q(const int8_t *xq, mesa_layout L, const float *alpha, const float *beta, const void *dy,
                                       void *dx, mesa_dtype dt, void *stream)
{
    return act_bwd_q<kActGelu>(xq, L, alpha, beta, dy, dx, dt, stream);
}

extern "C" MESA_EXPORT mesa_status mesa_relu_bwd_q(const int8_t *xq, mesa_layout L, const float *alpha, const float *beta, const void *dy,
                                       void *dx, mesa_dtype dt, void *stream)
{
    return act_bwd_q<kActRelu>(xq, L, alpha, beta, dy, dx, dt, stream);
}

extern "C" MESA_EXPORT mesa_status mesa_stream_copy(const void *src, void *dst, size_t bytes, void *stream)
{
    if (bytes == 0) return MESA_OK;
    if (!src || !dst || !aligned16(src) || !aligned16(dst) || (bytes & 15u)) return MESA_ERR_INVALID_ARG;
    const int64_t n16 = int64_t(bytes / 16);
    const int grid = plan_grid(n16, int64_t(kThreads) * 4, 4 * kGridCap, 0);
    hipLaunchKernelGGL(k_copy, dim3(grid), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4 *>(src), static_cast<u32x4 *>(dst), n16);
    return launch_status();
}

extern "C" MESA_EXPORT mesa_status mesa_stream_read(const void *src, size_t bytes, void *sink, void *stream)
{
    if (bytes == 0) return MESA_OK;
    if (!src || !sink || !aligned16(src) || !aligned4(sink) || (bytes & 15u)) return MESA_ERR_INVALID_ARG;
    const int64_t n16 = int64_t(bytes / 16);
    const int grid = plan_grid(n16, int64_t(kThreads) * 4, 4 * kGridCap, 0);
    hipLaunchKernelGGL(k_read_probe, dim3(grid), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4 *>(src), n16, static_cast<uint32_t *>(sink));
    return launch_status();
}

extern "C" MESA_EXPORT mesa_status mesa_stream_fill(void *dst, size_t bytes, uint32_t word, void *stream)
{
    if (bytes == 0) return MESA_OK;
    if (!dst || !aligned16(dst) || (bytes & 15u)) return MESA_ERR_INVALID_ARG;
    const int64_t n16 = int64_t(bytes / 16);
    const int grid = plan_grid(n16, int64_t(kThreads) * 4, 4 * kGridCap, 0);
    hipLaunchKernelGGL(k_fill_probe, dim3(grid), dim3(kThreads), 0, static_cast<hipStream_t>(stream), static_cast<u32x4 *>(dst), n16,
                       word);
    return launch_status();
}

extern "C" MESA_EXPORT mesa_status mesa_event_create(void **event)
{
    if (!event) return MESA_ERR_INVALID_ARG;
    hipEvent_t ev;
    if (hipEventCreate(&ev) != hipSuccess) return MESA_ERR_LAUNCH;
    *event = ev;
    return MESA_OK;
}

extern "C" MESA_EXPORT mesa_status mesa_event_record(void *event, void *stream)
{
    if (!event) return MESA_ERR_INVALID_ARG;
    return hipEventRecord(static_cast<hipEvent_t>(event), static_cast<hipStream_t>(stream)) == hipSuccess ? MESA_OK
                                                                                                           : MESA_ERR_LAUNCH;
}

extern "C" MESA_EXPORT mesa_status mesa_event_elapsed_ms(void *start, void *stop, float *ms)
{
    if (!start || !stop || !ms) return MESA_ERR_INVALID_ARG;
    if (hipEventSynchronize(static_cast<hipEvent_t>(stop)) != hipSuccess) return MESA_ERR_LAUNCH;
    return hipEventElapsedTime(ms, static_cast<hipEvent_t>(start), static_cast<hipEvent_t>(stop)) == hipSuccess
               ? MESA_OK
               : MESA_ERR_LAUNCH;
}

extern "C" MESA_EXPORT mesa_status mesa_event_destroy(void *event)
{
    if (!event) return MESA_ERR_INVALID_ARG;
    return hipEventDestroy(static_cast<hipEvent_t>(event)) == hipSuccess ? MESA_OK : MESA_ERR_LAUNCH;
}

extern "C" MESA_EXPORT const char *mesa_status_string(mesa_status s)
{
    switch (s) {
    case MESA_OK: return "ok";
    case MESA_ERR_INVALID_ARG: return "invalid argument";
    case MESA_ERR_UNSUPPORTED: return "unsupported shape";
    case MESA_ERR_WORKSPACE: return "workspace missing or too small";
    case MESA_ERR_LAUNCH: return "HIP runtime error";
    }
    return "unknown status";
}

extern "C" MESA_EXPORT int mesa_version(void) { return 100; }

extern "C" MESA_EXPORT size_t mesa_workspace_bytes(mesa_op op, int64_t d0, int64_t d1, int64_t d2, mesa_dtype dt)
{
    switch (op) {
    case MESA_OP_UPDATE_RUNNING_PARAMS: return update_ws_bytes(d0, d1, d2);
    case MESA_OP_LAYERNORM_BWD_Q: return layernorm_ws_bytes(d0, d1);
    case MESA_OP_LINEAR_DW_Q: return linear_dw_ws_bytes(d0, d1, d2, dt);
    case MESA_OP_SOFTMAX_FWD_Q: return softmax_fwd_ws_bytes(d0, d1, d2);
    case MESA_OP_LAYERNORM_FWD_Q: return layernorm_fwd_ws_bytes(d0, d1, d2);
    }
    return 0;
}

// An upper bound of update_ws_bytes over every layout with this many elements and groups (for a caller that knows the
// tensor's size and groups but not how outer and inner share the rest): minmax_grid stays within its cap, rounded up to
// a multiple of at most 64, plus the at most 255 steps of its search.
size_t mesa::update_ws_bound(int64_t numel, int64_t groups)
{
    if (numel <= 0 || groups <= 0) return 16;
    int64_t worst = 0;
    const int caps[2] = {kMmGridCap, kFuGridCap};
    for (int v = 0; v < 2; ++v) {
        int64_t cap = caps[v];
        if (groups > 64) {
            const int64_t fixed = int64_t(caps[v]) * 64 / groups, paid = numel / (64 * groups);
            int64_t c = fixed > paid ? fixed : paid;
            if (c < 32) c = 32;
            if (c < cap) cap = c;
        }
        if (cap > worst) worst = cap;
    }
    return size_t(worst + 64 + 256) * 2 * size_t(groups) * sizeof(float);
}

// size of the min/max partials: enough for mesa_update_running_params and mesa_quantize_update_fused
size_t mesa::update_ws_bytes(int64_t outer, int64_t groups, int64_t inner)
{
    mesa_layout L = {outer, groups, inner};
    if (check_layout(L) != MESA_OK || layout_numel(L) == 0) return 16;
    const int g0 = minmax_grid(L), g1 = minmax_grid(L, kFuU, kFuGridCap);   // the two callers of this workspace
    return size_t(g0 > g1 ? g0 : g1) * 2 * size_t(groups < 1 ? 1 : groups) * sizeof(float);
}
