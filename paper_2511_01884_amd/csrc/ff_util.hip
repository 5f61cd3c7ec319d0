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

// ---- measured ceilings --------------------------------------------------------
// Two kernels that do nothing but the one thing a roofline is about, so that the fraction of the
// published peak a kernel reaches can be read next to what the chip sustains at all:
//   mfma_loop_kernel    a register-resident loop of independent bf16 32x32x16 MFMAs (no memory traffic)
//   stream_read_kernel  16-byte streaming loads over a buffer, eight in flight per thread
namespace ff {

namespace {

constexpr int kMfmaChains = 8;  // independent accumulators per wavefront: the matrix pipe never waits

__global__ __launch_bounds__(256) void mfma_loop_kernel(long long iters, float *sink)
{
    // operands with varied bit patterns (the power an MFMA draws depends on its data)
    const unsigned t = threadIdx.x + blockIdx.x * 256u;
    uintx4 a, b;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const unsigned h = (t * 2654435761u) ^ ((unsigned)i * 0x9e3779b9u);
        a[i] = ((h & 0x007f007fu) | 0x3f803f80u) ^ ((h >> 3) & 0x80008000u);          // bf16 pairs in +-[1, 2)
        b[i] = (((h >> 7) & 0x007f007fu) | 0x3f003f00u) ^ ((h >> 11) & 0x80008000u);  // bf16 pairs in +-[0.5, 1)
    }
    floatx16 acc[kMfmaChains];
#pragma unroll
    for (int c = 0; c < kMfmaChains; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            acc[c][r] = 0.0f;
    for (long long it = 0; it < iters; ++it) {
#pragma unroll
        for (int c = 0; c < kMfmaChains; ++c)
            acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                             __builtin_bit_cast(bf16x8, b), acc[c], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int c = 0; c < kMfmaChains; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            s += acc[c][r];
    sink[t] = s;
}

__global__ __launch_bounds__(256) void stream_read_kernel(const uintx4 *src, size_t n16, unsigned *sink)
{
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    uintx4 x = {0u, 0u, 0u, 0u};
    for (; i + 7 * stride < n16; i += 8 * stride) {
        uintx4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < 8; ++u)
            x ^= v[u];
    }
    for (; i < n16; i += stride)
        x ^= __builtin_nontemporal_load(src + i);
    sink[blockIdx.x * 256 + threadIdx.x] = x[0] ^ x[1] ^ x[2] ^ x[3];
}

}  // namespace

// one workgroup (four wavefronts) per compute unit; returns the flops the launch performs
hipError_t launch_mfma_loop(long long iters, float *sink, int num_cus, hipStream_t stream, double *flops)
{
    hipLaunchKernelGGL(mfma_loop_kernel, dim3(num_cus), dim3(256), 0, stream, iters, sink);
    *flops = (double)num_cus * 4.0 * (double)iters * kMfmaChains * (2.0 * 32 * 32 * 16);
    return hipGetLastError();
}

// two workgroups per compute unit (the count a streaming read is fastest with)
hipError_t launch_stream_read(const void *src, size_t bytes, unsigned *sink, int num_cus, hipStream_t stream)
{
    hipLaunchKernelGGL(stream_read_kernel, dim3(num_cus * 2), dim3(256), 0, stream,
                       reinterpret_cast<const uintx4 *>(src), bytes / 16, sink);
    return hipGetLastError();
}

}  // namespace ff
