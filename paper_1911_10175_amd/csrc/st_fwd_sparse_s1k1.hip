// Instances of the zero-skipping FWD / BWI kernel: 3x3, unit stride, one produced channel per lane.
#include "st_fwd_sparse_impl.hpp"

namespace st {
namespace fs {

// 64 accumulators per lane (8x8 pixels x 1 channel), for channel counts that are no multiple of 128.  Images
// whose sides are multiples of 7 get 7x7 tiles: 49 accumulators, 80 registers, six wavefronts per SIMD instead of
// five (measured: the BWI of 64->128 @112 488 -> 452 us at 50 % zeros, 313 -> 293 at 90 %; 64->64 @224 within
// 1.5 % either way; 4x7 tiles with eight wavefronts are 3-7 % slower: twice the filter bytes per pixel).
hipError_t launch_s1_k1(const Geom &g, const float *in, const float *f, float *out, hipStream_t s)
{
    if (g.Wo % 7 == 0 && g.Ho % 7 == 0) return launch_cfg<3, 3, 7, 7, 1, 4>(g, in, f, out, s);
    if (g.Wo % 8 != 0 && g.Wo % 7 == 0) return launch_cfg<3, 3, 8, 7, 1, 4>(g, in, f, out, s);
    return launch_cfg<3, 3, 8, 8, 1, 4>(g, in, f, out, s);
}

}  // namespace fs
}  // namespace st
