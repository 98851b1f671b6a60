// Instances of the zero-skipping FWD / BWI kernel: 3x3, unit stride, one produced channel per lane.
#include "st_fwd_sparse_impl.hpp"

namespace st {
namespace fs {

// 64 accumulators per lane (8x8 pixels x 1 channel), for channel counts that are no multiple of 128.
hipError_t launch_s1_k1(const Geom &g, const float *in, const float *f, float *out, hipStream_t s)
{
    if (g.Wo % 8 != 0 && g.Wo % 7 == 0) return launch_cfg<3, 3, 8, 7, 1, 4>(g, in, f, out, s);
    return launch_cfg<3, 3, 8, 8, 1, 4>(g, in, f, out, s);
}

}  // namespace fs
}  // namespace st
