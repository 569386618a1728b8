// mfma_probe.hip -- a measurement helper, not part of the method: the rate at which this GPU sustains the weight
// gradient's matrix-core instruction stream when nothing else is asked of it.  One workgroup of four waves per CU (one
// wave per SIMD, as in k_dw_f16), every wave a 128 x 128 tile of sixteen 32 x 32 accumulators, sixteen
// v_mfma_f32_32x32x16_f16 per contraction step of 16.  Three forms:
//   0  operands stay in registers: the instruction alone;
//   1  the eight operand fragments of a step are read from LDS (16 bytes per lane and fragment, conflict-free, one
//      step ahead of their use), as a kernel that keeps its tiles in LDS must do;
//   2  form 1 plus three 16-byte global loads per lane and step whose data goes to LDS four steps later: 12 KB per
//      workgroup and step, the operand movement of k_dw_f16's 256 x 256 tile (per 32 rows 16 KB of binary16 values
//      and 8 KB of codes).  The loads walk `feed`, wrapping at its end; workgroup b reads vectors b * 256 .. + 255 of
//      every run of 65536, so an XCD (every eighth workgroup) keeps to its eighth of the feed: a feed of up to
//      8 x the L2 size stays in the L2s, which stands for tiles that neighbouring workgroups share.
// The operands are pseudo-random binary16 values of magnitude 1/2 .. 1 (what the datapath switches costs power, and
// the chip's clock follows the power).  The flop count is exact: launches x 256 workgroups x 4 waves x steps x 16
// instructions x 2 * 32 * 32 * 16.
#include <hip/hip_runtime.h>

#include "api_util.hpp"
#include "common.hpp"

namespace mesa {

typedef _Float16 mp_v8h __attribute__((ext_vector_type(8)));
typedef float mp_v16f __attribute__((ext_vector_type(16)));

constexpr int kProbeWorkgroups = 256;     // one per CU
constexpr int kProbePoolVecs = 4096;      // 64 KB of operands in LDS
constexpr int kProbeMaxSteps = 1 << 20;

__device__ __forceinline__ uint32_t probe_word(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return (x & 0x83ff83ffu) | 0x38003800u;      // two binary16 values: random sign and fraction, exponent of 1/2
}

template <int FORM>
__global__ __launch_bounds__(256, 1) void k_mfma_probe(int steps, const u32x4 *__restrict__ feed, int feed_vecs, float *__restrict__ sink)
{
    __shared__ __attribute__((aligned(16))) u32x4 pool[kProbePoolVecs];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int v = tid; v < kProbePoolVecs; v += 256) {
        const uint32_t s = (blockIdx.x * kProbePoolVecs + v) * 4u;
        pool[v] = u32x4{probe_word(s), probe_word(s + 1), probe_word(s + 2), probe_word(s + 3)};
    }
    __syncthreads();
    mp_v16f acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
    // a wave's fragments of step s: vectors ((8 s + f) * 64 + lane) of its quarter of the pool
    const u32x4 *mine = pool + wave * (kProbePoolVecs / 4);
    auto frag = [&](int s, int f) { return mine[((s * 8 + f) * 64 + lane) & (kProbePoolVecs / 4 - 1)]; };
    u32x4 cur[8], nxt[8];
#pragma unroll
    for (int f = 0; f < 8; ++f) cur[f] = frag(0, f);
    uint32_t at = (blockIdx.x * 256u + tid) % uint32_t(feed_vecs);     // walks the feed in strides of one vector per thread of the grid
    constexpr int kAhead = 4;                              // steps between a load's request and its store to LDS
    u32x4 fed[kAhead][3];
#pragma unroll
    for (int r = 0; r < kAhead; ++r)
#pragma unroll
        for (int k = 0; k < 3; ++k) fed[r][k] = u32x4{0u, 0u, 0u, 0u};
    auto step = [&](int s, int r, bool move) {
        if (FORM >= 1) {
#pragma unroll
            for (int f = 0; f < 8; ++f) nxt[f] = frag(s + 1, f);
        }
        if (FORM == 2 && move) {
            // the vectors requested kAhead steps ago go to LDS (over fragments this wave has just used); the next are requested
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                pool[wave * (kProbePoolVecs / 4) + (((s * 8 + k) * 64 + lane) & (kProbePoolVecs / 4 - 1))] = fed[r][k];
                fed[r][k] = feed[at];
                at += kProbeWorkgroups * 256;              // feed_vecs >= that: one subtraction brings it back
                at -= at >= uint32_t(feed_vecs) ? uint32_t(feed_vecs) : 0u;
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(mp_v8h, cur[i]), __builtin_bit_cast(mp_v8h, cur[4 + j]),
                                                                   acc[i][j], 0, 0, 0);
        if (FORM >= 1) {
#pragma unroll
            for (int f = 0; f < 8; ++f) cur[f] = nxt[f];
        }
    };
    int s = 0;
    for (; s + kAhead <= steps; s += kAhead) {
#pragma unroll
        for (int r = 0; r < kAhead; ++r) step(s + r, r, true);
    }
    for (; s < steps; ++s) step(s, 0, false);              // the last steps request nothing more
    uint32_t fold = 0u;
#pragma unroll
    for (int r = 0; r < kAhead; ++r)
#pragma unroll
        for (int k = 0; k < 3; ++k) fold ^= fed[r][k][0];
    float t = __builtin_bit_cast(float, fold & 0u);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) t += acc[i][j][v];
    sink[int64_t(blockIdx.x) * 256 + tid] = t;
}

// Form 3: the same work per workgroup and step as form 2 (a 256 x 256 tile, 64 instructions, 12 KB moved) shared out
// among EIGHT waves, two per SIMD: every wave a 128 x 64 tile of eight accumulators, eight instructions per step from
// four + two operand fragments, three 16-byte global loads per lane every second step.  What one wave cannot do --
// issue its vector, LDS and memory instructions while its own matrix instruction runs -- its neighbour on the SIMD does.
__global__ __launch_bounds__(512, 1) void k_mfma_probe8(int steps, const u32x4 *__restrict__ feed, int feed_vecs, float *__restrict__ sink)
{
    __shared__ __attribute__((aligned(16))) u32x4 pool[kProbePoolVecs];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int v = tid; v < kProbePoolVecs; v += 512) {
        const uint32_t s = (blockIdx.x * kProbePoolVecs + v) * 4u;
        pool[v] = u32x4{probe_word(s), probe_word(s + 1), probe_word(s + 2), probe_word(s + 3)};
    }
    __syncthreads();
    mp_v16f acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
    constexpr int kMine = kProbePoolVecs / 8;              // 512 vectors: eight fragments of 64 lanes
    u32x4 *mine = pool + wave * kMine;
    auto frag = [&](int s, int f) { return mine[((s * 6 + f) * 64 + lane) & (kMine - 1)]; };
    u32x4 cur[6], nxt[6];
#pragma unroll
    for (int f = 0; f < 6; ++f) cur[f] = frag(0, f);
    uint32_t at = (blockIdx.x * 512u + tid) % uint32_t(feed_vecs);
    constexpr int kAhead = 2;                              // pairs of steps between a load's request and its store to LDS
    u32x4 fed[kAhead][3];
#pragma unroll
    for (int r = 0; r < kAhead; ++r)
#pragma unroll
        for (int k = 0; k < 3; ++k) fed[r][k] = u32x4{0u, 0u, 0u, 0u};
    auto step = [&](int s, int r, bool move) {
#pragma unroll
        for (int f = 0; f < 6; ++f) nxt[f] = frag(s + 1, f);
        if (move) {
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                mine[((s * 6 + k) * 64 + lane) & (kMine - 1)] = fed[r][k];
                fed[r][k] = feed[at];
                at += kProbeWorkgroups * 512;              // feed_vecs >= that: one subtraction brings it back
                at -= at >= uint32_t(feed_vecs) ? uint32_t(feed_vecs) : 0u;
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(mp_v8h, cur[i]), __builtin_bit_cast(mp_v8h, cur[4 + j]),
                                                                   acc[i][j], 0, 0, 0);
#pragma unroll
        for (int f = 0; f < 6; ++f) cur[f] = nxt[f];
    };
    int s = 0;
    for (; s + 2 * kAhead <= steps; s += 2 * kAhead) {
#pragma unroll
        for (int r = 0; r < kAhead; ++r) {
            step(s + 2 * r, r, true);
            step(s + 2 * r + 1, r, false);
        }
    }
    for (; s < steps; ++s) step(s, 0, false);
    uint32_t fold = 0u;
#pragma unroll
    for (int r = 0; r < kAhead; ++r)
#pragma unroll
        for (int k = 0; k < 3; ++k) fold ^= fed[r][k][0];
    float t = __builtin_bit_cast(float, fold & 0u);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) t += acc[i][j][v];
    // two threads per slot of the sink: thread t and t + 256 of a workgroup add up in a fixed order
    __shared__ float half_sum[256];
    if (tid >= 256) half_sum[tid - 256] = t;
    __syncthreads();
    if (tid < 256) sink[int64_t(blockIdx.x) * 256 + tid] = t + half_sum[tid];
}

}  // namespace mesa

using namespace mesa;

extern "C" MESA_EXPORT mesa_status mesa_mfma_probe(int form, int64_t steps, const void *feed, size_t feed_bytes, float *sink, void *stream)
{
    if (form < 0 || form > 3 || steps < 0 || steps > kProbeMaxSteps || !sink || !aligned4(sink)) return MESA_ERR_INVALID_ARG;
    if (form >= 2 && (!feed || !aligned16(feed) || feed_bytes < (size_t(1) << 21) || (feed_bytes & 15u) || feed_bytes > (size_t(1) << 34)))
        return MESA_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const u32x4 *f = static_cast<const u32x4 *>(feed);
    const int fv = form >= 2 ? int(feed_bytes / 16) : 1;
    if (form == 0) hipLaunchKernelGGL(k_mfma_probe<0>, dim3(kProbeWorkgroups), dim3(256), 0, s, int(steps), f, fv, sink);
    else if (form == 1) hipLaunchKernelGGL(k_mfma_probe<1>, dim3(kProbeWorkgroups), dim3(256), 0, s, int(steps), f, fv, sink);
    else if (form == 2) hipLaunchKernelGGL(k_mfma_probe<2>, dim3(kProbeWorkgroups), dim3(256), 0, s, int(steps), f, fv, sink);
    else hipLaunchKernelGGL(k_mfma_probe8, dim3(kProbeWorkgroups), dim3(512), 0, s, int(steps), f, fv, sink);
    return launch_status();
}
