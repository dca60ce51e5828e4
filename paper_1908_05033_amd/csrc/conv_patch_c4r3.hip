// LDS-patch kernel variants for 4-bit containers, 3x3 filters.
#include "conv_patch_kernel.h"

hipError_t dsq_conv_patch_c4r3(const DsqConvArgs &a, const PatchPlan &pl, int which, int ks, int need, hipStream_t stream)
{
    return dispatch_variant<4, 3>(a, pl, which, ks, need, stream);
}
