// LDS-patch kernel variants for dense 3-bit activation codes, 1x1 filters.
#include "conv_patch_kernel.h"

hipError_t dsq_conv_patch_c3r1(const DsqConvArgs &a, const PatchPlan &pl, int which, int ks, int need, hipStream_t stream)
{
    return dispatch_variant<3, 1>(a, pl, which, ks, need, stream);
}
