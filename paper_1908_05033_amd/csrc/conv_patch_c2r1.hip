// LDS-patch kernel variants for 2-bit containers, 1x1 filters.
#include "conv_patch_kernel.h"

hipError_t dsq_conv_patch_c2r1(const DsqConvArgs &a, const PatchPlan &pl, int which, int ks, int need, hipStream_t stream)
{
    return dispatch_variant<2, 1>(a, pl, which, ks, need, stream);
}
