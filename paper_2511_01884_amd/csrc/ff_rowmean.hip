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
// (W + X read once, Out written once).
//
// One launch of one workgroup per compute unit, three phases separated by two
// grid-wide arrivals (counters in the control region, bounded waits):
//   1  column sums of W over chunks of rows (fp32 partials, written through);
//      one workgroup also computes c.  Then every wavefront requests its first
//      row of X, which travels while the grid meets.
//   2  the first K/64 workgroups add the partials in chunk order: wbar.
//   3  wbar moves into LDS; one wavefront per row: the row is read once and kept
//      in registers (the case study's "cache the original row in registers"),
//      dotted with wbar, butterfly-reduced, GELU, broadcast add, store.
// All sums run in fixed order: results are bitwise reproducible on a device.
#include "ff_tile.hpp"

namespace ff {

namespace {

constexpr int kColThreads = kRowMeanColThreads;  // phase 1: threads across a strip of columns, 16 bytes of a row each
constexpr int kColSub = kRowMeanColSub;          // phase 1: groups of rows per workgroup
constexpr int kThreads = kColThreads * kColSub;  // 512
constexpr int kWaves = kThreads / 64;            // phase 3: rows in flight per workgroup
constexpr int kMaxChunks = 16;                   // 16-byte chunks of a row one lane keeps in registers

// a plain value another workgroup (on another XCD, behind another L2) reads later in this launch
__device__ __forceinline__ void store_through(float *p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

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

// PL = 16-byte chunks of a row a lane keeps in registers; R = rows a wavefront requests ahead of phase 3.
template <typename T, int PL, int R>
__global__ __launch_bounds__(kThreads) void rowmean_kernel(const RowMeanParams p)
{
    constexpr int E = Vec16<T>::n;
    __shared__ float red[kColSub][8 * kColThreads];  // 16 KiB; phases 2 and the c sum reuse it
    extern __shared__ __align__(16) float s_w[];    // K floats (phase 3)
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int K = p.K, N = p.N, M = p.M;
    const int G = gridDim.x;
    const T *W = reinterpret_cast<const T *>(p.W);
    const T *X = reinterpret_cast<const T *>(p.X);
    T *Out = reinterpret_cast<T *>(p.Out);

    // ---- phase 1: partial[chunk][k] = sum over the chunk's rows of W[n][k] ----
    // item = (column strip, row chunk); a workgroup is kColSub groups of kColThreads threads, a group
    // adds a quarter of the chunk's rows (16 bytes of each row per thread), group 0 adds the groups
    {
        const int col = tid % kColThreads;
        const int sub = tid / kColThreads;
        const int rows_per_sub = p.rows_per_chunk / kColSub;
        for (int item = blockIdx.x; item < p.strips * p.chunks; item += G) {
            const int strip = item % p.strips;
            const int chunk = item / p.strips;
            const int k0 = (strip * kColThreads + col) * E;
            int n = chunk * p.rows_per_chunk + sub * rows_per_sub;
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
            __syncthreads();  // the previous item's readers are done with red
#pragma unroll
            for (int e = 0; e < E; ++e)
                red[sub][col * E + e] = acc[e];
            __syncthreads();
            // consecutive threads write consecutive columns: whole lines go out, written through
            for (int cidx = tid; cidx < kColThreads * E; cidx += kThreads) {
                const int k = strip * kColThreads * E + cidx;
                if (k < K) {
                    float t = red[0][cidx];
#pragma unroll
                    for (int g = 1; g < kColSub; ++g)
                        t += red[g][cidx];
                    store_through(p.partial + (size_t)chunk * K + k, t);
                }
            }
        }
    }

    // ---- arrival A: every partial is written ----
    wait_published();
    __syncthreads();
    const int way = blockIdx.x % kSyncWays;
    if (tid == 0)
        atomic_add_device(p.counters + (size_t)way * kSyncStride, 1u);

    // ---- the first R rows of every wavefront: requested now, they travel while the grid meets ----
    const int nchunks = K / E;                       // 16-byte chunks per row
    const int per_lane = (nchunks + 63) / 64;        // chunks per lane, interleaved by lane
    const int row_step = G * kWaves;
    uintx4 keep[R][PL];
    // loads never branch: a lane past the row's end re-reads the last chunk and masks it out later
    auto load_row = [&](int m, uintx4 (&dst)[PL]) {
        const T *x = X + (size_t)m * K;
#pragma unroll
        for (int u = 0; u < PL; ++u) {
            int ch = u * 64 + lane;
            ch = ch < nchunks ? ch : nchunks - 1;
            dst[u] = __builtin_nontemporal_load(reinterpret_cast<const uintx4 *>(x + (size_t)ch * E));
        }
    };
    const int m_first = blockIdx.x * kWaves + wave;
#pragma unroll
    for (int r = 0; r < R; ++r)
        if (m_first + r * row_step < M)
            load_row(m_first + r * row_step, keep[r]);

    if (wave == 0) {
        const int l = lane < kSyncWays ? lane : 0;
        const unsigned target = (unsigned)(G + kSyncWays - 1 - l) / kSyncWays + (l == 0 ? (unsigned)p.extra_arrivals : 0u);
        if (!wait_counters_wave(p.counters, target, p.wait_ticks) && lane == 0)
            atomic_store_device(p.err, 1u);
    }
    __syncthreads();

    // ---- phase 2: wbar[k] = (sum of the chunk partials in chunk order) / N ----
    // a workgroup item owns 64 columns: 16 lanes x float4 across, 16 groups of chunks down; a thread adds
    // its group's chunks in order, then thread k adds the 16 group sums in order
    const int mean_items = (K + 63) / 64;
    {
        float(*red2)[65] = reinterpret_cast<float(*)[65]>(&red[0][0]);
        for (int item = blockIdx.x; item < mean_items; item += G) {
            if (tid < 256) {
                const int col4 = tid & 15;
                const int grp = tid >> 4;
                const int k = item * 64 + col4 * 4;
                const int per_grp = (p.chunks + 15) / 16;
                const int c_begin = grp * per_grp;
                const int c_end = (c_begin + per_grp < p.chunks) ? c_begin + per_grp : p.chunks;
                floatx4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
                if (k < K) {
                    const float *src = p.partial + (size_t)c_begin * K + k;
#pragma unroll 8
                    for (int c = c_begin; c < c_end; ++c) {
                        acc += *reinterpret_cast<const floatx4 *>(src);
                        src += K;
                    }
                }
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    red2[grp][col4 * 4 + e] = acc[e];
            }
            __syncthreads();
            const int kk = item * 64 + tid;
            if (tid < 64 && kk < K) {
                float t = 0.0f;
#pragma unroll
                for (int g = 0; g < 16; ++g)
                    t += red2[g][tid];
                store_through(p.wbar + kk, t / (float)N);
            }
            __syncthreads();
        }
    }

    // ---- c = mean(b - s), by the workgroup after the last one that had phase-2 items ----
    const int b_wgs = mean_items + 1 < G ? mean_items + 1 : G;   // workgroups that arrive at B
    if ((int)blockIdx.x == b_wgs - 1) {
        const T *b = reinterpret_cast<const T *>(p.b);
        const T *sv = reinterpret_cast<const T *>(p.s);
        float acc = 0.0f;
        if (b)
            for (int n = tid; n < N; n += kThreads)
                acc += load_as_float(b + n);
        if (sv)
            for (int n = tid; n < N; n += kThreads)
                acc -= load_as_float(sv + n);
        float *flat = &red[0][0];
        flat[tid] = acc;
        __syncthreads();
        for (int off = kThreads / 2; off >= 1; off >>= 1) {
            if (tid < off)
                flat[tid] += flat[tid + off];
            __syncthreads();
        }
        if (tid == 0)
            store_through(p.wbar + K, flat[0] / (float)N);
    }

    // ---- arrival B: wbar and c are complete (only the workgroups that wrote them arrive) ----
    if ((int)blockIdx.x < b_wgs) {
        wait_published();
        __syncthreads();
        if (tid == 0)
            atomic_add_device(p.counters + (size_t)way * kSyncStride + 3, 1u);
    }
    if (wave == 0) {
        const int l = lane < kSyncWays ? lane : 0;
        const unsigned target = l < b_wgs ? (unsigned)(b_wgs + kSyncWays - 1 - l) / kSyncWays : 0u;
        if (!wait_counters_wave(p.counters + 3, target + (l == 0 ? (unsigned)p.extra_arrivals : 0u), p.wait_ticks) &&
            lane == 0)
            atomic_store_device(p.err, 1u);
    }
    __syncthreads();

    // ---- phase 3: Out[m] = X[m] + GELU(X[m] . wbar + c), one wavefront per row ----
    for (int k = tid * 4; k < K; k += kThreads * 4)
        *reinterpret_cast<floatx4 *>(s_w + k) = *reinterpret_cast<const floatx4 *>(p.wbar + k);
    const float c = p.wbar[K];
    __syncthreads();
    auto finish_row = [&](int m, const uintx4 (&row)[PL]) {
        const T *x = X + (size_t)m * K;
        T *o = Out + (size_t)m * K;
        float dot = 0.0f;
#pragma unroll
        for (int u = 0; u < PL; ++u) {
            const int ch_raw = u * 64 + lane;
            const bool live = ch_raw < nchunks;
            const int ch = live ? ch_raw : nchunks - 1;
            float f[8];
            unpack(row[u], f, (const T *)nullptr);
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
                emit(row[u], ch);
        }
        for (int u = PL; u < per_lane; ++u) {
            const int ch = u * 64 + lane;
            if (ch < nchunks)
                emit(*reinterpret_cast<const uintx4 *>(x + (size_t)ch * E), ch);
        }
    };
#pragma unroll
    for (int r = 0; r < R; ++r)
        if (m_first + r * row_step < M)
            finish_row(m_first + r * row_step, keep[r]);
    for (int m = m_first + R * row_step; m < M; m += row_step) {
        load_row(m, keep[0]);
        finish_row(m, keep[0]);
    }

    // ---- departure: the last workgroup of the last way re-arms every counter ----
    // (only then has every workgroup left both waits, so no poller can see a counter go back to zero)
    if (tid == 0) {
        const unsigned in_way = (unsigned)(G + kSyncWays - 1 - way) / kSyncWays;
        const unsigned ways = G < kSyncWays ? (unsigned)G : (unsigned)kSyncWays;
        if (atomic_add_device(p.counters + (size_t)way * kSyncStride + 1, 1u) == in_way - 1u) {
            if (atomic_add_device(p.counters + 2, 1u) == ways - 1u) {
                for (int w = 0; w < kSyncWays; ++w) {
                    atomic_store_device(p.counters + (size_t)w * kSyncStride, 0u);
                    atomic_store_device(p.counters + (size_t)w * kSyncStride + 1, 0u);
                    atomic_store_device(p.counters + (size_t)w * kSyncStride + 3, 0u);
                }
                atomic_store_device(p.counters + 2, 0u);
            }
        }
    }
}

template <typename T, int PL, int R>
hipError_t launch_plr(const RowMeanParams &p, hipStream_t stream)
{
    const size_t lds_bytes = (size_t)p.K * sizeof(float);
    if (lds_bytes > 32 * 1024) {  // static + dynamic beyond the default limit
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&rowmean_kernel<T, PL, R>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess)
            return e;
    }
    hipLaunchKernelGGL((rowmean_kernel<T, PL, R>), dim3(p.grid), dim3(kThreads), lds_bytes, stream, p);
    return hipGetLastError();
}

// two rows ahead when a wavefront has at least two rows and both fit the register budget
template <typename T, int PL>
hipError_t launch_pl(const RowMeanParams &p, hipStream_t stream)
{
    const bool two = PL <= 8 && (int64_t)p.M > (int64_t)p.grid * kWaves;
    return two ? launch_plr<T, PL, (PL <= 8 ? 2 : 1)>(p, stream) : launch_plr<T, PL, 1>(p, stream);
}

template <typename T>
hipError_t launch_t(const RowMeanParams &p, hipStream_t stream)
{
    constexpr int E = Vec16<T>::n;
    const int per_lane = (p.K / E + 63) / 64;
    if (per_lane <= 1) return launch_pl<T, 1>(p, stream);
    if (per_lane <= 2) return launch_pl<T, 2>(p, stream);
    if (per_lane <= 4) return launch_pl<T, 4>(p, stream);
    if (per_lane <= 8) return launch_pl<T, 8>(p, stream);
    return launch_pl<T, kMaxChunks>(p, stream);
}

}  // namespace

hipError_t launch_rowmean_chain(bool bf16, const RowMeanParams &p, hipStream_t stream)
{
    return bf16 ? launch_t<__bf16>(p, stream) : launch_t<float>(p, stream);
}

}  // namespace ff
