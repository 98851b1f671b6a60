// Instances of the zero-skipping FWD / BWI kernel: 3x3, unit stride, two produced channels per lane.
#include "st_fwd_sparse_impl.hpp"

namespace st {
namespace fs {

// 64 accumulators per lane (4x8 pixels x 2 channels).  7-wide tiles when the row length is a multiple
// of 7 but not of 8 (28, 14): no ragged tiles.
hipError_t launch_s1_k2(const Geom &g, const float *in, const float *f, float *out, hipStream_t s)
{
    if (g.Wo % 8 != 0 && g.Wo % 7 == 0) return launch_cfg<3, 3, 4, 7, 2, 4>(g, in, f, out, s);
    return launch_cfg<3, 3, 4, 8, 2, 4>(g, in, f, out, s);
}

}  // namespace fs
}  // namespace st
