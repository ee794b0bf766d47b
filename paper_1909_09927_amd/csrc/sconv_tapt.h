// Entry points of the transposed-filter 3x3 kernel (sconv_tapt.hip), one pair per tile geometry; the
// candidate table of sconv_tap.hip lists them beside the staged kernel's geometries.
#pragma once

#include "sconv_internal.h"

namespace sconv {

struct TaptPlan {
    double cost;              // model clocks; negative: the geometry or the pinned decomposition does not apply
    int nwv, ncs, nt, nss;    // wavefronts per workgroup = nt tiles x ncs channel slices; workgroups per tile
};

#define SCONV_TAPT_DECLARE(NAME)                                                                               \
    TaptPlan tapt_plan_##NAME(const Problem& p, int split);                                                    \
    int tapt_launch_##NAME(const Problem& p, bool pooled, int split, const float* x, const float* w, float* y, \
                           hipStream_t stream);

SCONV_TAPT_DECLARE(5x7k1)
SCONV_TAPT_DECLARE(5x7k1n)
SCONV_TAPT_DECLARE(5x7k2)
SCONV_TAPT_DECLARE(7x7k1)
SCONV_TAPT_DECLARE(7x7k2)
SCONV_TAPT_DECLARE(p4x14k1)
SCONV_TAPT_DECLARE(p4x6k1)
SCONV_TAPT_DECLARE(p4x6k2)
SCONV_TAPT_DECLARE(p2x14k2)
SCONV_TAPT_DECLARE(p2x14k1)
SCONV_TAPT_DECLARE(p2x14hk1)
SCONV_TAPT_DECLARE(p2x14hk2)
SCONV_TAPT_DECLARE(s2_3x4k1)
SCONV_TAPT_DECLARE(s2_3x4k2)

}  // namespace sconv
