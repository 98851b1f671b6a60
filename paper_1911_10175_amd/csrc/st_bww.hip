// Filter-gradient kernels (BWW): zero-skipping and dense.
#include "st_common.hpp"

namespace st {

bool bww_fast_supported(const st_conv_desc &) { return false; }
size_t bww_sparse_workspace(const st_conv_desc &) { return 0; }
size_t bww_dense_workspace(const st_conv_desc &) { return 0; }

hipError_t launch_bww_sparse(const st_conv_desc &, const float *, const float *, float *, float *, hipStream_t)
{
    return hipErrorInvalidValue;
}

hipError_t launch_bww_dense(const st_conv_desc &, const float *, const float *, float *, float *, hipStream_t)
{
    return hipErrorInvalidValue;
}

}  // namespace st
