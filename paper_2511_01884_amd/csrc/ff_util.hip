// A plain device-to-device copy, 16 bytes per thread per step over a grid-stride loop.  It exists to
// calibrate hardware counters: a kernel whose HBM traffic is known exactly (bytes read = bytes
// written = the size) gives the factor by which a byte counter has to be scaled.
#include "ff_tile.hpp"

namespace ff {

namespace {

__global__ __launch_bounds__(256) void copy_kernel(const uintx4 *src, uintx4 *dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride)
        dst[i] = src[i];
}

}  // namespace

hipError_t launch_copy_kernel(const void *src, void *dst, size_t bytes, int num_cus, hipStream_t stream)
{
    const size_t n16 = bytes / 16;
    size_t blocks = (n16 + 255) / 256;
    const size_t cap = (size_t)num_cus * 16;
    if (blocks > cap)
        blocks = cap;
    if (blocks == 0)
        return hipSuccess;
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, stream,
                       reinterpret_cast<const uintx4 *>(src), reinterpret_cast<uintx4 *>(dst), n16);
    return hipGetLastError();
}

}  // namespace ff
