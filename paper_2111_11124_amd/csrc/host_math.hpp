// host_math.hpp -- host-side integer helpers shared by the launchers: division by an invariant
// divisor through multiplication, and the per-launch constants of the group cursor.  Plain C++,
// no HIP types, so it can also be compiled and tested with a host compiler alone.
#pragma once
#include <stdint.h>

namespace mesa {

// q = n / d for 0 <= n < 2^31 and 1 <= d < 2^31:  q = (mulhi(n, mul) + n) >> shift.
// With l = ceil(log2 d), mul = floor(2^32 * (2^l - d) / d) + 1 is the low 32 bits of the 33-bit
// round-up reciprocal floor(2^(32+l)/d) + 1; the sum cannot overflow because mulhi(n, mul) < n.
struct FastDiv {
    uint32_t d;
    uint32_t mul;
    uint32_t shift;
};

inline FastDiv make_fastdiv(uint32_t d)
{
    FastDiv f;
    f.d = d;
    uint32_t l = 0;
    while ((uint64_t(1) << l) < d) ++l;
    f.shift = l;
    f.mul = uint32_t(((uint64_t(1) << 32) * ((uint64_t(1) << l) - d)) / d + 1);
    return f;
}

inline uint32_t fastdiv_host(uint32_t n, const FastDiv &f)
{
    uint32_t hi = uint32_t((uint64_t(n) * f.mul) >> 32);
    return (hi + n) >> f.shift;
}

// Where an element of a (outer, groups, inner) tensor sits: `rem` = position inside its slab of
// `inner` elements, `g` = group of that slab.  A thread that moves on by `step` elements per
// iteration updates both with adds and compares only; these are the per-launch constants.
struct GroupGeom {
    uint32_t inner;     // slab length (for groups == 1 a synthetic multiple of 16: the group is always 0)
    uint32_t groups;
    uint32_t step_rem;  // step % inner
    uint32_t step_g;    // (step / inner) % groups
    FastDiv div_inner;  // for the one-off placement of a thread's further vectors
    FastDiv div_groups;
};

inline GroupGeom make_geom(int64_t groups, int64_t inner, int64_t step)
{
    GroupGeom g;
    if (groups <= 1) {
        g.inner = 1u << 20;
        g.groups = 1;
    } else {
        g.inner = uint32_t(inner);
        g.groups = uint32_t(groups);
    }
    g.step_rem = uint32_t(step % int64_t(g.inner));
    g.step_g = uint32_t((step / int64_t(g.inner)) % int64_t(g.groups));
    g.div_inner = make_fastdiv(g.inner);
    g.div_groups = make_fastdiv(g.groups);
    return g;
}

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

}  // namespace mesa
