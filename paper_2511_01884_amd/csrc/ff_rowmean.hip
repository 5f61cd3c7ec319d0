// Second fused chain (the paper's fused-epilogue case study, App. B.1):
//
//     Out[m][k] = X[m][k] + GELU( mean_n( X[m] . W[n] + b[n] - s[n] ) )
//
// The case study is about removing global-memory round trips from this chain
// (the GEMM output re-read, the second read of the original row).  On top of
// that, the mean over n of a linear layer is itself linear in the row:
//     mean_n( x . W[n] + b[n] - s[n] ) = x . wbar + c,
//     wbar[k] = mean_n W[n][k],  c = mean_n (b[n] - s[n]),
// so the M x N x K GEMM collapses to one read of W (column means) and one
// dot product per row: O(NK + MK) work, bound by HBM traffic
// (W + X read once, Out written once).  Three small kernels:
//   colsum_kernel    partial column sums of W over chunks of rows (fp32)
//   colmean_kernel   wbar = sum of the partials in chunk order / N, and c
//   rowdot_kernel    one wavefront per row: the row is read once and kept in
//                    registers (the case study's "cache original_x in registers"),
//                    dot with wbar from LDS, butterfly reduction, GELU, add, store.
// All sums run in fixed order: results are bitwise reproducible.
#include "ff_tile.hpp"

namespace ff {

namespace {

constexpr int kColThreads = 128;   // colsum: threads per workgroup, 16 bytes of a row each
constexpr int kRowThreads = 256;   // rowdot: 4 wavefronts = 4 rows in flight per workgroup
constexpr int kMaxChunks = 16;     // 16-byte chunks of a row one lane keeps in registers

template <typename T> struct Vec16 { static constexpr int n = 16 / (int)sizeof(T); };

__device__ __forceinline__ void unpack(const uintx4 &v, float (&f)[8], const __bf16 *)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = __uint_as_float(v[i] << 16);
        f[2 * i + 1] = __uint_as_float(v[i] & 0xffff0000u);
    }
}
__device__ __forceinline__ void unpack(const uintx4 &v, float (&f)[8], const float *)
{
#pragma unroll
    for (int i = 0; i < 4; ++i)
        f[i] = __uint_as_float(v[i]);
}

// partial[chunk][k] = sum over the chunk's rows of W[n][k]; grid (column strips, row chunks)
template <typename T>
__global__ __launch_bounds__(kColThreads) void colsum_kernel(const T *W, float *partial, int N, int K,
                                                             int rows_per_chunk)
{
    constexpr int E = Vec16<T>::n;
    const int k0 = (blockIdx.x * kColThreads + threadIdx.x) * E;
    if (k0 >= K)
        return;
    const int n_begin = blockIdx.y * rows_per_chunk;
    const int n_end = (n_begin + rows_per_chunk < N) ? n_begin + rows_per_chunk : N;
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    const T *w = W + (size_t)n_begin * K + k0;
    int n = n_begin;
    for (; n + 8 <= n_end; n += 8) {  // eight rows in flight
        uintx4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            v[u] = __builtin_nontemporal_load(reinterpret_cast<const uintx4 *>(w + (size_t)u * K));
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            float f[8];
            unpack(v[u], f, (const T *)nullptr);
#pragma unroll
            for (int e = 0; e < E; ++e)
                acc[e] += f[e];
        }
        w += (size_t)8 * K;
    }
    for (; n < n_end; ++n) {
        const uintx4 v = __builtin_nontemporal_load(reinterpret_cast<const uintx4 *>(w));
        float f[8];
        unpack(v, f, (const T *)nullptr);
#pragma unroll
        for (int e = 0; e < E; ++e)
            acc[e] += f[e];
        w += K;
    }
    float *dst = partial + (size_t)blockIdx.y * K + k0;
#pragma unroll
    for (int e = 0; e < E; ++e)
        dst[e] = acc[e];
}

// wbar[k] = (sum of partials in chunk order) / N;  wbar[K] = c = mean(b - s)
template <typename T>
__global__ __launch_bounds__(256) void colmean_kernel(const float *partial, const T *b, const T *s,
                                                      float *wbar, int N, int K, int chunks)
{
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k < K) {
        float acc = 0.0f;
        for (int c = 0; c < chunks; ++c)
            acc += partial[(size_t)c * K + k];
        wbar[k] = acc / (float)N;
    }
    if (blockIdx.x == 0) {
        // c = mean(b - s): one workgroup, fixed-order tree
        __shared__ float red[256];
        float acc = 0.0f;
        for (int n = threadIdx.x; n < N; n += 256)
            acc += (b ? load_as_float(b + n) : 0.0f) - (s ? load_as_float(s + n) : 0.0f);
        red[threadIdx.x] = acc;
        __syncthreads();
        for (int off = 128; off >= 1; off >>= 1) {
            if ((int)threadIdx.x < off)
                red[threadIdx.x] += red[threadIdx.x + off];
            __syncthreads();
        }
        if (threadIdx.x == 0)
            wbar[K] = red[0] / (float)N;
    }
}

// Out[m] = X[m] + GELU(X[m] . wbar + c); one wavefront per row, rows strided over the grid
template <typename T>
__global__ __launch_bounds__(kRowThreads) void rowdot_kernel(const T *X, const float *wbar, T *Out,
                                                            int M, int K)
{
    constexpr int E = Vec16<T>::n;
    extern __shared__ float s_w[];  // K floats
    for (int k = threadIdx.x; k < K; k += kRowThreads)
        s_w[k] = wbar[k];
    const float c = wbar[K];
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int nchunks = K / E;                       // 16-byte chunks per row
    const int per_lane = (nchunks + 63) / 64;        // chunks per lane, interleaved by lane
    for (int m = blockIdx.x * 4 + wave; m < M; m += gridDim.x * 4) {
        const T *x = X + (size_t)m * K;
        T *o = Out + (size_t)m * K;
        uintx4 keep[kMaxChunks];
        float dot = 0.0f;
#pragma unroll
        for (int u = 0; u < kMaxChunks; ++u) {
            const int ch = u * 64 + lane;
            if (u < per_lane && ch < nchunks)
                keep[u] = *reinterpret_cast<const uintx4 *>(x + (size_t)ch * E);
        }
#pragma unroll
        for (int u = 0; u < kMaxChunks; ++u) {
            const int ch = u * 64 + lane;
            if (u < per_lane && ch < nchunks) {
                float f[8];
                unpack(keep[u], f, (const T *)nullptr);
#pragma unroll
                for (int e = 0; e < E; ++e)
                    dot = fmaf(f[e], s_w[ch * E + e], dot);
            }
        }
        // rows longer than the register budget: the rest is read here and again below
        for (int u = kMaxChunks; u < per_lane; ++u) {
            const int ch = u * 64 + lane;
            if (ch < nchunks) {
                float f[8];
                unpack(*reinterpret_cast<const uintx4 *>(x + (size_t)ch * E), f, (const T *)nullptr);
#pragma unroll
                for (int e = 0; e < E; ++e)
                    dot = fmaf(f[e], s_w[ch * E + e], dot);
            }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1)
            dot += __shfl_xor(dot, off);             // every lane ends with the same sum
        const float g = gelu_erf(dot + c);
        auto emit = [&](const uintx4 &v, int ch) {
            float f[8];
            unpack(v, f, (const T *)nullptr);
            uintx4 r;
            if (sizeof(T) == 2) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    r[i] = pack_bf16x2(f[2 * i] + g, f[2 * i + 1] + g);
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    r[i] = __float_as_uint(f[i] + g);
            }
            *reinterpret_cast<uintx4 *>(o + (size_t)ch * E) = r;
        };
#pragma unroll
        for (int u = 0; u < kMaxChunks; ++u) {
            const int ch = u * 64 + lane;
            if (u < per_lane && ch < nchunks)
                emit(keep[u], ch);
        }
        for (int u = kMaxChunks; u < per_lane; ++u) {
            const int ch = u * 64 + lane;
            if (ch < nchunks)
                emit(*reinterpret_cast<const uintx4 *>(x + (size_t)ch * E), ch);
        }
    }
}

template <typename T>
hipError_t launch_t(const RowMeanParams &p, hipStream_t stream)
{
    constexpr int E = Vec16<T>::n;
    const int strips = (p.K + kColThreads * E - 1) / (kColThreads * E);
    hipLaunchKernelGGL(colsum_kernel<T>, dim3(strips, p.chunks), dim3(kColThreads), 0, stream,
                       reinterpret_cast<const T *>(p.W), p.partial, p.N, p.K, p.rows_per_chunk);
    hipLaunchKernelGGL(colmean_kernel<T>, dim3((p.K + 255) / 256), dim3(256), 0, stream, p.partial,
                       reinterpret_cast<const T *>(p.b), reinterpret_cast<const T *>(p.s), p.wbar, p.N,
                       p.K, p.chunks);
    const size_t lds_bytes = (size_t)p.K * sizeof(float);
    if (lds_bytes > 64 * 1024) {  // beyond the default dynamic-LDS limit
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&rowdot_kernel<T>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess)
            return e;
    }
    hipLaunchKernelGGL(rowdot_kernel<T>, dim3(p.row_grid), dim3(kRowThreads), lds_bytes,
                       stream, reinterpret_cast<const T *>(p.X), p.wbar, reinterpret_cast<T *>(p.Out), p.M,
                       p.K);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_rowmean_chain(bool bf16, const RowMeanParams &p, hipStream_t stream)
{
    return bf16 ? launch_t<__bf16>(p, stream) : launch_t<float>(p, stream);
}

}  // namespace ff
