// Clears an int32 buffer with a kernel.  A memset node would do the same in an
// eager stream, but memset nodes replayed from a captured graph have not been
// reliable on this platform, so the library only ever uses kernels.
#include "dsq_kernels.h"

namespace {

__global__ __launch_bounds__(256) void fill_zero_kernel(int32_t *p, size_t n)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t n4 = n / 4;
    if (i < n4) reinterpret_cast<int4 *>(p)[i] = make_int4(0, 0, 0, 0);
    if (i < n - n4 * 4) p[n4 * 4 + i] = 0;
}

}  // namespace

hipError_t dsq_launch_fill_zero(int32_t *p, size_t n, hipStream_t stream)
{
    if (n == 0) return hipSuccess;
    const size_t threads = n / 4 > 4 ? n / 4 : 4;       // also covers the < 4 leftover words
    fill_zero_kernel<<<dim3((unsigned)((threads + 255) / 256)), 256, 0, stream>>>(p, n);
    return hipGetLastError();
}
