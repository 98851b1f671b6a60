// Instances of the zero-skipping FWD / BWI kernel for the 3x3 layers with stride 2.
#include "st_fwd_sparse_impl.hpp"

namespace st {
namespace fs {

// FWD: a 4x8 output tile is fed by a 9x17 input halo, 2.25 taps per tested element on average.
hipError_t launch_s2_fwd(const Geom &g, const float *in, const float *f, float *out, hipStream_t s)
{
    const bool seven = g.Wo % 8 != 0 && g.Wo % 7 == 0;
    if (g.Ko % 128 == 0) return seven ? launch_cfg<3, 3, 4, 7, 2, 4, 2, 1, 0>(g, in, f, out, s) : launch_cfg<3, 3, 4, 8, 2, 4, 2, 1, 0>(g, in, f, out, s);
    return seven ? launch_cfg<3, 3, 4, 7, 1, 4, 2, 1, 0>(g, in, f, out, s) : launch_cfg<3, 3, 4, 8, 1, 4, 2, 1, 0>(g, in, f, out, s);
}

// BWI: every tested element feeds all 9 taps; tiles have even sides so that the position of the input
// samples within a tile is the same for every tile.  One channel per lane and 64-pixel tiles: a dx tile
// receives only 2.25 taps per pixel and channel, so the filter registers of a channel must serve as many
// pixels as possible (two channels per lane on 4x8 tiles measured 20-45 % slower).
hipError_t launch_s2_bwi(const Geom &g, const float *in, const float *f, float *out, hipStream_t s)
{
    const bool fourteen = g.Wo % 8 != 0 && g.Wo % 14 == 0;
    return fourteen ? launch_cfg<3, 3, 4, 14, 1, 4, 1, 2, 1>(g, in, f, out, s) : launch_cfg<3, 3, 8, 8, 1, 4, 1, 2, 1>(g, in, f, out, s);
}

}  // namespace fs
}  // namespace st
