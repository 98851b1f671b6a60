// Instances of the zero-skipping FWD / BWI kernel for 1x1 layers.
#include "st_fwd_sparse_impl.hpp"

namespace st {
namespace fs {

// Without spatial reuse a non-zero input feeds only KPL multiply-adds per lane: as many output channels
// per lane as the layer has (Sec. 5.2 of the paper: T = Q/V for 1x1).
hipError_t launch_pw(const Geom &g, const float *in, const float *f, float *out, hipStream_t s)
{
    if (g.Ko % 256 == 0) return launch_cfg<1, 1, 2, 8, 4, 4>(g, in, f, out, s);
    if (g.Ko % 128 == 0) return launch_cfg<1, 1, 8, 8, 2, 2>(g, in, f, out, s);
    return launch_cfg<1, 1, 8, 8, 1, 4>(g, in, f, out, s);
}

}  // namespace fs
}  // namespace st
