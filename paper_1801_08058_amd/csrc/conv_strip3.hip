// Rank-3 instantiations and launchers of the strip convolution kernels (see conv_strip_kernels.h): blocked output,
// two waves per SIMD, no channel sums.
#include "conv_strip_kernels.h"

namespace ngc {

template <int NF>
static hipError_t launch_strip_r3_nf(const StripParams &p, size_t lds_bytes, hipStream_t st)
{
    if (p.dbp) return hipErrorInvalidValue;
    if (p.ncolt > 1) return launch_strip_d<NF, 8, 0, false, true, true>(p, lds_bytes, st);
    return launch_strip_d<NF, 8, 0, false, true>(p, lds_bytes, st);
}

// p as launch_strip prepared it (XCD order decided); nf = 32-position fragments per SIMD (7, 4 or 2)
hipError_t launch_strip_r3(const StripParams &p, int nf, size_t lds_bytes, hipStream_t st)
{
    if (!p.r3 || p.out_mode != 0) return hipErrorInvalidValue;
    switch (nf) {
    case 7: return launch_strip_r3_nf<4>(p, lds_bytes, st);
    case 4: return launch_strip_r3_nf<2>(p, lds_bytes, st);
    case 2: return launch_strip_r3_nf<1>(p, lds_bytes, st);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_strip_multi_r3(const StripMulti &mp, int nf, size_t lds_bytes, hipStream_t st)
{
    switch (nf) {
    case 7: return launch_strip_multi_t<4, false, true>(mp, lds_bytes, st);
    case 4: return launch_strip_multi_t<2, false, true>(mp, lds_bytes, st);
    case 2: return launch_strip_multi_t<1, false, true>(mp, lds_bytes, st);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace ngc
