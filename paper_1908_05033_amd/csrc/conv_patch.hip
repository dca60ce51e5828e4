#include "conv_epilogue.h"
bool dsq_conv_patch_supported(const DsqConvArgs &) { return false; }
hipError_t dsq_launch_conv_patch(const DsqConvArgs &, hipStream_t) { return hipErrorNotSupported; }
