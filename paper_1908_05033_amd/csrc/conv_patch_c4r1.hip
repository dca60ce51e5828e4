// LDS-patch kernel variants for 4-bit containers, 1x1 filters.
#include "conv_patch_kernel.h"

hipError_t dsq_conv_patch_c4r1(const DsqConvArgs &a, const PatchPlan &pl, int which, int ks, int need, hipStream_t stream)
{
    return dispatch_variant<4, 1>(a, pl, which, ks, need, stream);
}
