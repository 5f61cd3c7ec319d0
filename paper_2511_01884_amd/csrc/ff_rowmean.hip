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
//   colsum_kernel    partial column sums of W over chunks of rows (fp32); one extra workgroup computes c
//   colmean_kernel   wbar = sum of the partials in chunk order / N
//   rowdot_kernel    one wavefront per row: the row is read once and kept in
//                    registers (the case study's "cache original_x in registers"),
//                    dot with wbar from LDS, butterfly reduction, GELU, add, store.
// All sums run in fixed order: results are bitwise reproducible.
#include "ff_tile.hpp"

namespace ff {

namespace {

constexpr int kColThreads = 128;   // colsum: threads across a strip of columns, 16 bytes of a row each
constexpr int kColSub = kRowMeanColSub;  // colsum: groups of rows per workgroup
constexpr int kRowWaves = kRowMeanWaves;  // rowdot: wavefronts = rows in flight per workgroup
constexpr int kRowThreads = kRowWaves * 64;
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

// partial[chunk][k] = sum over the chunk's rows of W[n][k]; grid (column strips, row chunks + 1).
// A workgroup is kColSub groups of kColThreads threads: a group adds a quarter of the chunk's rows,
// 16 bytes of each row per thread, and group 0 then adds the group sums in order.
template <typename T>
__global__ __launch_bounds__(kColThreads * kColSub) void colsum_kernel(const T *W, const T *b, const T *s,
                                                                       float *partial, float *c_out, int N,
                                                                       int K, int rows_per_chunk)
{
    constexpr int E = Vec16<T>::n;
    constexpr int kThreads = kColThreads * kColSub;
    __shared__ float red[kColSub][E][kColThreads];
    if (blockIdx.y == gridDim.y - 1) {
        // one extra workgroup: c = mean(b - s), strided sums and a fixed-order tree
        if (blockIdx.x != 0)
            return;
        float acc = 0.0f;
        if (b)
            for (int n = threadIdx.x; n < N; n += kThreads)
                acc += load_as_float(b + n);
        if (s)
            for (int n = threadIdx.x; n < N; n += kThreads)
                acc -= load_as_float(s + n);
        float *flat = &red[0][0][0];
        flat[threadIdx.x] = acc;
        __syncthreads();
        for (int off = kThreads / 2; off >= 1; off >>= 1) {
            if ((int)threadIdx.x < off)
                flat[threadIdx.x] += flat[threadIdx.x + off];
            __syncthreads();
        }
        if (threadIdx.x == 0)
            *c_out = flat[0] / (float)N;
        return;
    }
    const int col = threadIdx.x % kColThreads;
    const int sub = threadIdx.x / kColThreads;
    const int k0 = (blockIdx.x * kColThreads + col) * E;
    const int rows_per_sub = rows_per_chunk / kColSub;
    int n = blockIdx.y * rows_per_chunk + sub * rows_per_sub;
    int n_end = n + rows_per_sub;
    n_end = n_end < N ? n_end : N;
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (k0 < K) {
        const T *w = W + (size_t)n * K + k0;
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
    }
#pragma unroll
    for (int e = 0; e < E; ++e)
        red[sub][e][col] = acc[e];
    __syncthreads();
    if (sub == 0 && k0 < K) {
        float *dst = partial + (size_t)blockIdx.y * K + k0;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            float t = red[0][e][col];
#pragma unroll
            for (int g = 1; g < kColSub; ++g)
                t += red[g][e][col];
            dst[e] = t;
        }
    }
}

// wbar[k] = (sum of the chunk partials) / N;  wbar[K] = c = mean(b - s).
// A workgroup owns 64 columns: 16 lanes x float4 across, 16 groups of chunks down.  A thread adds
// its group's chunks in order, then thread k adds the 16 group sums in order.
__global__ __launch_bounds__(256) void colmean_kernel(const float *partial, float *wbar, int N, int K,
                                                      int chunks)
{
    __shared__ float red[16][65];
    const int col4 = threadIdx.x & 15;
    const int grp = threadIdx.x >> 4;
    const int k = blockIdx.x * 64 + col4 * 4;
    const int per_grp = (chunks + 15) / 16;
    const int c_begin = grp * per_grp;
    const int c_end = (c_begin + per_grp < chunks) ? c_begin + per_grp : chunks;
    floatx4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
    if (k < K) {
        const float *src = partial + (size_t)c_begin * K + k;
#pragma unroll 8
        for (int c = c_begin; c < c_end; ++c) {
            acc += *reinterpret_cast<const floatx4 *>(src);
            src += K;
        }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e)
        red[grp][col4 * 4 + e] = acc[e];
    __syncthreads();
    const int kk = blockIdx.x * 64 + threadIdx.x;
    if (threadIdx.x < 64 && kk < K) {
        float t = 0.0f;
#pragma unroll
        for (int g = 0; g < 16; ++g)
            t += red[g][threadIdx.x];
        wbar[kk] = t / (float)N;
    }
}

// Out[m] = X[m] + GELU(X[m] . wbar + c); one wavefront per row, rows strided over the grid.
// PL = 16-byte chunks of the row a lane keeps in registers between the dot product and the add.
template <typename T, int PL>
__global__ __launch_bounds__(kRowThreads) void rowdot_kernel(const T *X, const float *wbar, T *Out,
                                                            int M, int K)
{
    constexpr int E = Vec16<T>::n;
    extern __shared__ __align__(16) float s_w[];  // K floats
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int nchunks = K / E;                       // 16-byte chunks per row
    const int per_lane = (nchunks + 63) / 64;        // chunks per lane, interleaved by lane
    uintx4 keep[PL];
    // loads never branch: a lane past the row's end re-reads the last chunk and masks it out later
    auto load_row = [&](int m) {
        const T *x = X + (size_t)m * K;
#pragma unroll
        for (int u = 0; u < PL; ++u) {
            int ch = u * 64 + lane;
            ch = ch < nchunks ? ch : nchunks - 1;
            keep[u] = __builtin_nontemporal_load(reinterpret_cast<const uintx4 *>(x + (size_t)ch * E));
        }
    };
    int m = blockIdx.x * kRowWaves + wave;
    if (m < M)
        load_row(m);  // the first row is in flight while the column means move into LDS
    for (int k = threadIdx.x * 4; k < K; k += kRowThreads * 4)
        *reinterpret_cast<floatx4 *>(s_w + k) = *reinterpret_cast<const floatx4 *>(wbar + k);
    const float c = wbar[K];
    __syncthreads();
    bool loaded = true;
    for (; m < M; m += gridDim.x * kRowWaves) {
        if (!loaded)
            load_row(m);
        loaded = false;
        const T *x = X + (size_t)m * K;
        T *o = Out + (size_t)m * K;
        float dot = 0.0f;
#pragma unroll
        for (int u = 0; u < PL; ++u) {
            const int ch_raw = u * 64 + lane;
            const bool live = ch_raw < nchunks;
            const int ch = live ? ch_raw : nchunks - 1;
            float f[8];
            unpack(keep[u], f, (const T *)nullptr);
            float part = 0.0f;
#pragma unroll
            for (int e = 0; e < E; ++e)
                part = fmaf(f[e], s_w[ch * E + e], part);
            dot += live ? part : 0.0f;
        }
        // rows longer than the register budget: the rest is read here and again below
        for (int u = PL; u < per_lane; ++u) {
            const int ch = u * 64 + lane;
            if (ch < nchunks) {
                float f[8];
                unpack(*reinterpret_cast<const uintx4 *>(x + (size_t)ch * E), f, (const T *)nullptr);
                float part = 0.0f;
#pragma unroll
                for (int e = 0; e < E; ++e)
                    part = fmaf(f[e], s_w[ch * E + e], part);
                dot += part;
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
            __builtin_nontemporal_store(r, reinterpret_cast<uintx4 *>(o + (size_t)ch * E));
        };
#pragma unroll
        for (int u = 0; u < PL; ++u) {
            const int ch = u * 64 + lane;
            if (ch < nchunks)
                emit(keep[u], ch);
        }
        for (int u = PL; u < per_lane; ++u) {
            const int ch = u * 64 + lane;
            if (ch < nchunks)
                emit(*reinterpret_cast<const uintx4 *>(x + (size_t)ch * E), ch);
        }
    }
}

template <typename T, int PL>
hipError_t launch_rowdot(const RowMeanParams &p, hipStream_t stream)
{
    const size_t lds_bytes = (size_t)p.K * sizeof(float);
    if (lds_bytes > 64 * 1024) {  // beyond the default dynamic-LDS limit
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&rowdot_kernel<T, PL>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess)
            return e;
    }
    hipLaunchKernelGGL((rowdot_kernel<T, PL>), dim3(p.row_grid), dim3(kRowThreads), lds_bytes, stream,
                       reinterpret_cast<const T *>(p.X), p.wbar, reinterpret_cast<T *>(p.Out), p.M, p.K);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_t(const RowMeanParams &p, hipStream_t stream)
{
    constexpr int E = Vec16<T>::n;
    const int strips = (p.K + kColThreads * E - 1) / (kColThreads * E);
    hipLaunchKernelGGL(colsum_kernel<T>, dim3(strips, p.chunks + 1), dim3(kColThreads * kColSub), 0, stream,
                       reinterpret_cast<const T *>(p.W), reinterpret_cast<const T *>(p.b),
                       reinterpret_cast<const T *>(p.s), p.partial, p.wbar + p.K, p.N, p.K, p.rows_per_chunk);
    hipLaunchKernelGGL(colmean_kernel, dim3((p.K + 63) / 64), dim3(256), 0, stream, p.partial, p.wbar, p.N,
                       p.K, p.chunks);
    const int per_lane = (p.K / E + 63) / 64;
    if (per_lane <= 1) return launch_rowdot<T, 1>(p, stream);
    if (per_lane <= 2) return launch_rowdot<T, 2>(p, stream);
    if (per_lane <= 4) return launch_rowdot<T, 4>(p, stream);
    if (per_lane <= 8) return launch_rowdot<T, 8>(p, stream);
    return launch_rowdot<T, kMaxChunks>(p, stream);
}

}  // namespace

hipError_t launch_rowmean_chain(bool bf16, const RowMeanParams &p, hipStream_t stream)
{
    return bf16 ? launch_t<__bf16>(p, stream) : launch_t<float>(p, stream);
}

}  // namespace ff
