// Instances of the zero-skipping FWD / BWI kernel: 3x3, unit stride, two produced channels per lane.
#include "st_fwd_sparse_impl.hpp"

namespace st {
namespace fs {

// 4x8 pixels x 2 channels = 64 accumulators per lane, four wavefronts per SIMD; 4x7 pixels = 56 accumulators,
// five.  The 7-wide tile is taken whenever the row length is a multiple of 7 (every image size of Table 1), also
// where 8 divides it too: measured on the 56- and 112-pixel layers of the VGG16 stack it is 2-8 % faster up to
// 80 % zeros, even at 0 %, and 6-8 % slower at 90 % (a seventh more filter bytes per pixel, which is what
// bounds the kernel there).
hipError_t launch_s1_k2(const Geom &g, const float *in, const float *f, float *out, hipStream_t s)
{
    if (g.Wo % 7 == 0) return launch_cfg<3, 3, 4, 7, 2, 4>(g, in, f, out, s);
    return launch_cfg<3, 3, 4, 8, 2, 4>(g, in, f, out, s);
}

}  // namespace fs
}  // namespace st
