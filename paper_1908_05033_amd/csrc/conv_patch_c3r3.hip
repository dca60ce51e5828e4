// LDS-patch kernel variants for dense 3-bit activation codes, 3x3 filters.
#include "conv_patch_kernel.h"

hipError_t dsq_conv_patch_c3r3(const DsqConvArgs &a, const PatchPlan &pl, int which, int ks, int need, hipStream_t stream)
{
    return dispatch_variant<3, 3>(a, pl, which, ks, need, stream);
}
