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
// One launch of one workgroup per compute unit, two phases separated by one
// grid-wide arrival (counters in the control region, bounded wait):
//   1  column sums of W: a work item is a 128-byte strip of columns times a chunk
//      of rows, 8 lanes per row piece and 64 rows per step, reduced by shuffles and
//      once through LDS; fp32 partials [chunks][K] are written through.  Every
//      workgroup also sums its slice of b - s.  Then every wavefront requests its
//      first rows of X, which travel while the grid meets.
//   2  each workgroup adds the few chunk partials in chunk order into LDS: wbar;
//      one wavefront per row: the row is read once and kept in registers (the
//      case study's "cache the original row in registers"), dotted with wbar,
//      butterfly-reduced, GELU, broadcast add, store.
// All sums run in fixed order: results are bitwise reproducible on a device.
#include "ff_tile.hpp"

namespace ff {

namespace {

constexpr int kThreads = kRowMeanThreads;         // 512
constexpr int kWaves = kThreads / 64;             // phase 2: rows in flight per workgroup
constexpr int kPieces = 8;                        // 16-byte pieces of a 128-byte strip
constexpr int kRowsPerStep = kRowMeanRowsPerStep; // phase 1: rows of W one load instruction of the workgroup covers
constexpr int kInFlight = 8;                      // phase 1: load instructions a thread keeps in flight
constexpr int kMaxChunks = 16;                    // 16-byte chunks of a row of X one lane keeps in registers
static_assert(kRowsPerStep * kPieces == kThreads, "one 16-byte piece per thread per step");

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

// PL = 16-byte chunks of a row a lane keeps in registers; R = rows a wavefront requests ahead of phase 2.
template <typename T, int PL, int R>
__global__ __launch_bounds__(kThreads) void rowmean_kernel(const RowMeanParams p)
{
    constexpr int E = Vec16<T>::n;
    constexpr int kStripElems = kPieces * E;        // columns of a strip
    __shared__ float red[kWaves][kPieces * 8];
    extern __shared__ __align__(16) float s_w[];    // K floats (phase 2)
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int K = p.K, N = p.N, M = p.M;
    const int G = gridDim.x;
    const T *W = reinterpret_cast<const T *>(p.W);
    const T *X = reinterpret_cast<const T *>(p.X);
    T *Out = reinterpret_cast<T *>(p.Out);

    // ---- phase 1: partial[chunk][k] = sum over the chunk's rows of W[n][k] ----
    {
        const int piece = tid % kPieces;
        const int r = tid / kPieces;
        for (int item = blockIdx.x; item < p.strips * p.chunks; item += G) {
            const int strip = item % p.strips;
            const int chunk = item / p.strips;
            const int k0 = strip * kStripElems + piece * E;
            const int n_begin = chunk * p.rows_per_chunk;
            const int n_end = n_begin + p.rows_per_chunk < N ? n_begin + p.rows_per_chunk : N;
            float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            if (k0 < K) {
                const T *w = W + k0;
                int n = n_begin + r;
                for (; n + (kInFlight - 1) * kRowsPerStep < n_end; n += kInFlight * kRowsPerStep) {
                    uintx4 v[kInFlight];
#pragma unroll
                    for (int u = 0; u < kInFlight; ++u)
                        v[u] = __builtin_nontemporal_load(
                            reinterpret_cast<const uintx4 *>(w + (size_t)(n + u * kRowsPerStep) * K));
#pragma unroll
                    for (int u = 0; u < kInFlight; ++u) {
                        float f[8];
                        unpack(v[u], f, (const T *)nullptr);
#pragma unroll
                        for (int e = 0; e < E; ++e)
                            acc[e] += f[e];
                    }
                }
                for (; n < n_end; n += kRowsPerStep) {
                    const uintx4 v = __builtin_nontemporal_load(reinterpret_cast<const uintx4 *>(w + (size_t)n * K));
                    float f[8];
                    unpack(v, f, (const T *)nullptr);
#pragma unroll
                    for (int e = 0; e < E; ++e)
                        acc[e] += f[e];
                }
            }
            // the 8 rows of a wavefront (lane / 8), fixed butterfly; lanes 0..7 end with the piece sums
#pragma unroll
            for (int off = 8; off <= 32; off <<= 1)
#pragma unroll
                for (int e = 0; e < E; ++e)
                    acc[e] += __shfl_xor(acc[e], off);
            __syncthreads();  // the previous item's readers are done with red
            if (lane < kPieces)
#pragma unroll
                for (int e = 0; e < E; ++e)
                    red[wave][lane * E + e] = acc[e];
            __syncthreads();
            if (tid < kStripElems) {
                float t = red[0][tid];
#pragma unroll
                for (int w8 = 1; w8 < kWaves; ++w8)
                    t += red[w8][tid];
                // the partial rows are padded to whole strips: columns at or beyond K hold zeros
                store_through(p.partial + (size_t)chunk * p.k_pad + strip * kStripElems + tid, t);
            }
        }
        // this workgroup's slice of sum(b - s): wavefront 0, lanes stride the slice, fixed butterfly
        if (wave == 0) {
            const T *b = reinterpret_cast<const T *>(p.b);
            const T *sv = reinterpret_cast<const T *>(p.s);
            const int per = (N + G - 1) / G;
            const int s_begin = blockIdx.x * per < N ? blockIdx.x * per : N;
            const int s_end = s_begin + per < N ? s_begin + per : N;
            float acc = 0.0f;
            for (int n = s_begin + lane; n < s_end; n += 64)
                acc += (b ? load_as_float(b + n) : 0.0f) - (sv ? load_as_float(sv + n) : 0.0f);
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1)
                acc += __shfl_xor(acc, off);
            if (lane == 0)
                store_through(p.cpart + blockIdx.x, acc);
        }
    }

    // ---- arrival: every partial is written ----
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

    // ---- phase 2: wbar into LDS (chunk partials added in chunk order), c, then one wavefront per row ----
    // two blocks of columns per pass, so that all of a thread's loads are in flight together
    for (int k = tid * 4; k < K; k += kThreads * 8) {
        const int k2 = k + kThreads * 4;
        const bool two = k2 < K;
        const float *src0 = p.partial + k;
        const float *src1 = p.partial + (two ? k2 : k);
        floatx4 t0 = {0.0f, 0.0f, 0.0f, 0.0f};
        floatx4 t1 = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll 4
        for (int ch = 0; ch < p.chunks; ++ch) {
            t0 += *reinterpret_cast<const floatx4 *>(src0);
            t1 += *reinterpret_cast<const floatx4 *>(src1);
            src0 += p.k_pad;
            src1 += p.k_pad;
        }
        *reinterpret_cast<floatx4 *>(s_w + k) = t0 / (float)N;
        if (two)
            *reinterpret_cast<floatx4 *>(s_w + k2) = t1 / (float)N;
    }
    float c = 0.0f;  // every wavefront adds the workgroups' slices in the same order
    for (int j = lane; j < G; j += 64)
        c += p.cpart[j];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1)
        c += __shfl_xor(c, off);
    c /= (float)N;
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
    // (only then has every workgroup left its wait, so no poller can see a counter go back to zero)
    if (tid == 0) {
        const unsigned in_way = (unsigned)(G + kSyncWays - 1 - way) / kSyncWays;
        const unsigned ways = G < kSyncWays ? (unsigned)G : (unsigned)kSyncWays;
        if (atomic_add_device(p.counters + (size_t)way * kSyncStride + 1, 1u) == in_way - 1u) {
            if (atomic_add_device(p.counters + 2, 1u) == ways - 1u) {
                for (int w = 0; w < kSyncWays; ++w) {
                    atomic_store_device(p.counters + (size_t)w * kSyncStride, 0u);
                    atomic_store_device(p.counters + (size_t)w * kSyncStride + 1, 0u);
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
