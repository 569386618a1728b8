// api_util.hpp -- argument checks and launch-shape planning shared by the entry points.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "host_math.hpp"
#include "mesa.h"

#define MESA_EXPORT __attribute__((visibility("default")))

namespace mesa {

// scratch sizes, each defined next to the launcher that uses the scratch
size_t update_ws_bytes(int64_t outer, int64_t groups, int64_t inner);
size_t update_ws_bound(int64_t numel, int64_t groups);
size_t layernorm_ws_bytes(int64_t M, int64_t D);
size_t linear_dw_ws_bytes(int64_t M, int64_t K, int64_t N, mesa_dtype dt);
size_t softmax_fwd_ws_bytes(int64_t total_rows, int64_t H, int64_t cols);
size_t layernorm_fwd_ws_bytes(int64_t M, int64_t D, int64_t G);

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool aligned4(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }
inline bool valid_dtype(mesa_dtype dt) { return dt == MESA_F32 || dt == MESA_F16 || dt == MESA_BF16; }
inline int dtype_bytes(mesa_dtype dt) { return dt == MESA_F32 ? 4 : 2; }

// expands X(T) with the element type that a valid dt names
#define MESA_FOR_DTYPE(dt, X) \
    do { \
        if ((dt) == MESA_F16) X(_Float16); \
        else if ((dt) == MESA_BF16) X(__bf16); \
        else X(float); \
    } while (0)

inline mesa_status check_layout(const mesa_layout &L)
{
    if (L.outer < 0 || L.groups < 0 || L.inner < 0) return MESA_ERR_INVALID_ARG;
    if (L.groups > 8192) return MESA_ERR_UNSUPPORTED;
    if (L.groups > 1 && L.inner >= (int64_t(1) << 30)) return MESA_ERR_UNSUPPORTED;
    // numel must stay below 2^53 (indices pass through binary64 once) -- far beyond any HBM
    if (L.outer > 0 && L.groups > 0 && L.inner > 0) {
        long double n = (long double)L.outer * (long double)L.groups * (long double)L.inner;
        if (n >= 9007199254740992.0L) return MESA_ERR_UNSUPPORTED;
    }
    return MESA_OK;
}

inline int64_t layout_numel(const mesa_layout &L) { return L.outer * L.groups * L.inner; }

inline mesa_status launch_status()
{
    return hipGetLastError() == hipSuccess ? MESA_OK : MESA_ERR_LAUNCH;
}

// Number of workgroups for a grid-stride streaming kernel in which every workgroup moves
// `per_wg_iter` elements per iteration: at most `cap` workgroups, iterations spread evenly, and --
// when it costs little -- a count that makes one grid step a whole number of rows of `row`
// elements, so that a thread keeps meeting the same channel group.
inline int plan_grid(int64_t numel, int64_t per_wg_iter, int cap, int64_t row)
{
    int64_t wgs_needed = ceil_div(numel, per_wg_iter);
    if (wgs_needed < 1) wgs_needed = 1;
    int64_t iters = ceil_div(wgs_needed, cap);
    int64_t n = ceil_div(wgs_needed, iters);
    if (row > 0) {
        int64_t a = per_wg_iter, b = row;
        while (b) { int64_t t = a % b; a = b; b = t; }
        int64_t mult = row / a;  // grid must be a multiple of this
        if (mult > 1 && mult <= 64) n = ceil_div(n, mult) * mult;
    }
    return int(n);
}

}  // namespace mesa
