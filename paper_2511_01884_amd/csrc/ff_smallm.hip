// Small-M path (M <= 32, bf16) of the fused linear + erf-GELU + LayerNorm
// operator: a streamer, not a tiled GEMM.  The cost is reading W once, so each
// workgroup owns a strip of 32 output columns, its 8 wavefronts split K, and
// every wave streams its share of the strip's W rows with 16-byte loads, many
// in flight, straight into 16x16x32 MFMA operands (M = 16 fills the MFMA's row
// block exactly; the tiny X comes from L2).  The row statistics span all
// workgroups, so they are exchanged as 8-byte (mean, M2) partials through
// global memory with an arrival counter inside the same launch — a second
// launch would cost a visible fraction of the ~17 us the stream itself takes.
// This is the paper's bandwidth-bound diagnosis pattern (App. B.1: a kernel at
// DRAM peak is fixed by removing passes over memory, not by more arithmetic).
#include "ff_tile.hpp"

namespace ff {

namespace {

constexpr int kWaves = 8;
constexpr int kThreads = 64 * kWaves;
constexpr int kStripTiles = kSmallMStripCols / 16;  // 16-column MFMA tiles per strip
constexpr int kUnroll = 4;                          // MFMA k-steps (32 elements) per batch

__device__ __forceinline__ uintx4 load16_nt(const void *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const uintx4 *>(p));
}

// MT = number of 16-row blocks of X (1: M <= 16, 2: M <= 32).
template <int MT>
__global__ __launch_bounds__(kThreads) void smallm_kernel(const SmallMParams p)
{
    __shared__ float s_part[kWaves][kStripTiles][MT][4][64];  // per-wave accumulators
    __shared__ float s_g[MT * 16][kSmallMStripCols];          // G of the current strip
    __shared__ floatx2 s_chunk[32][MT * 16];                  // merged statistics per chunk
    __shared__ floatx2 s_rst[MT * 16];                        // (mean, rstd) per row

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15;
    const int kg = lane >> 4;  // which 8-element group of a 32-element k-step
    const int M = p.M, N = p.N, K = p.K;
    const __bf16 *X = reinterpret_cast<const __bf16 *>(p.X);
    const __bf16 *W = reinterpret_cast<const __bf16 *>(p.W);

    // K range of this wave, in k-steps of 32 elements
    const int ksteps = (K + 31) / 32;
    const int per_wave = (ksteps + kWaves - 1) / kWaves;
    const int ks_begin = wave * per_wave;
    const int ks_end = (ks_begin + per_wave < ksteps) ? ks_begin + per_wave : ksteps;

    // Final-store ownership: thread `tid` owns elements e = tid + i * 512, i < MT, of a
    // strip's [16 MT][32] block of G (row e / 32, column e % 32).
    float g_keep[kSmallMMaxStripsPerGroup][MT];  // my G values of each strip this group owns

    int owned = 0;
    for (int strip = blockIdx.x; strip < p.strips; strip += gridDim.x, ++owned) {
        const int n0 = strip * kSmallMStripCols;
        floatx4 acc[kStripTiles][MT];
#pragma unroll
        for (int t = 0; t < kStripTiles; ++t)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                acc[t][mt] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};

        // per-lane row pointers: W rows n0 + t*16 + l16 (clamped), X rows mt*16 + l16
        const __bf16 *wrow[kStripTiles];
#pragma unroll
        for (int t = 0; t < kStripTiles; ++t) {
            int n = n0 + t * 16 + l16;
            n = n < N ? n : N - 1;
            wrow[t] = W + (size_t)n * K;
        }
        // X rows beyond M are clamped, not zeroed: they only feed output rows that
        // are never stored, and every row's statistics are independent.
        const __bf16 *xrow[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int m = mt * 16 + l16;
            xrow[mt] = X + (size_t)(m < M ? m : M - 1) * K;
        }

        auto load_batch = [&](int ks0, uintx4 (&wf)[kUnroll][kStripTiles], uintx4 (&xf)[kUnroll][MT]) {
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int k = (ks0 + u) * 32 + kg * 8;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    xf[u][mt] = *reinterpret_cast<const uintx4 *>(xrow[mt] + k);
#pragma unroll
                for (int t = 0; t < kStripTiles; ++t)
                    wf[u][t] = load16_nt(wrow[t] + k);
            }
        };
        auto mma_batch = [&](const uintx4 (&wf)[kUnroll][kStripTiles], const uintx4 (&xf)[kUnroll][MT]) {
#pragma unroll
            for (int u = 0; u < kUnroll; ++u)
#pragma unroll
                for (int t = 0; t < kStripTiles; ++t)
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        // A operand = W rows (register index runs along n),
                        // B operand = X rows (lane index runs along m)
                        acc[t][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            __builtin_bit_cast(bf16x8, wf[u][t]),
                            __builtin_bit_cast(bf16x8, xf[u][mt]), acc[t][mt], 0, 0, 0);
        };

        // Full batches of kUnroll k-steps, software-pipelined two deep so that a
        // batch of loads is always in flight behind the one being multiplied.
        const int full_end = (ks_end < K / 32) ? ks_end : K / 32;  // k-steps with all 32 elements
        const int nb = full_end > ks_begin ? (full_end - ks_begin) / kUnroll : 0;
        uintx4 wf0[kUnroll][kStripTiles], xf0[kUnroll][MT];
        uintx4 wf1[kUnroll][kStripTiles], xf1[kUnroll][MT];
        if (nb > 0)
            load_batch(ks_begin, wf0, xf0);
        int bi = 0;
        for (; bi + 2 <= nb; bi += 2) {
            load_batch(ks_begin + (bi + 1) * kUnroll, wf1, xf1);
            mma_batch(wf0, xf0);
            if (bi + 2 < nb)
                load_batch(ks_begin + (bi + 2) * kUnroll, wf0, xf0);
            mma_batch(wf1, xf1);
        }
        if (bi < nb)
            mma_batch(wf0, xf0);
        // remaining k-steps one at a time; the last one may be cut by K
        for (int ks = ks_begin + nb * kUnroll; ks < ks_end; ++ks) {
            const int k = ks * 32 + kg * 8;
            const unsigned keep = k < K ? 0xffffffffu : 0u;
            const int kc = k < K ? k : 0;
#pragma unroll
            for (int t = 0; t < kStripTiles; ++t) {
                uintx4 w = load16_nt(wrow[t] + kc);
                w &= keep;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const uintx4 x = *reinterpret_cast<const uintx4 *>(xrow[mt] + kc);
                    acc[t][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        __builtin_bit_cast(bf16x8, w), __builtin_bit_cast(bf16x8, x), acc[t][mt], 0, 0, 0);
                }
            }
        }

        // ---- sum the 8 waves' partial products in wave order ----
        __syncthreads();  // s_part / s_g of the previous strip are no longer read
#pragma unroll
        for (int t = 0; t < kStripTiles; ++t)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    s_part[wave][t][mt][r][lane] = acc[t][mt][r];
        __syncthreads();
        // kStripTiles * MT * 4 * 64 outputs over 512 threads
        constexpr int kOutputs = kStripTiles * MT * 4 * 64;
        for (int o = tid; o < kOutputs; o += kThreads) {
            const int ol = o & 63;
            const int r = (o >> 6) & 3;
            const int mt = (o >> 8) % MT;
            const int t = (o >> 8) / MT;
            float z = 0.0f;
#pragma unroll
            for (int w = 0; w < kWaves; ++w)
                z += s_part[w][t][mt][r][ol];
            // element (m, n): lane index runs along m, register along n
            const int m = mt * 16 + (ol & 15);
            const int nl = t * 16 + 4 * (ol >> 4) + r;
            const int n = n0 + nl;
            float g = 0.0f;
            if (n < N) {
                const float bias = p.b ? load_as_float(reinterpret_cast<const __bf16 *>(p.b) + n) : 0.0f;
                g = gelu_erf(z + bias);
            }
            s_g[m][nl] = g;
        }
        __syncthreads();
        // ---- per-row (mean, M2) of the strip; keep my G value in a register ----
        const int nvalid = (N - n0 < kSmallMStripCols) ? (N - n0) : kSmallMStripCols;
        if (tid < MT * 16) {
            float s = 0.0f;
            for (int c = 0; c < nvalid; ++c)
                s += s_g[tid][c];
            const float mean = s / (float)nvalid;
            float m2 = 0.0f;
            for (int c = 0; c < nvalid; ++c) {
                const float d = s_g[tid][c] - mean;
                m2 = fmaf(d, d, m2);
            }
            floatx2 o = {mean, m2};
            publish_pair(p.partials + (size_t)strip * (MT * 16) + tid, o);
        }
#pragma unroll
        for (int e = 0; e < MT; ++e) {
            const int el = tid + e * kThreads;
            const float gv = s_g[el / kSmallMStripCols][el % kSmallMStripCols];
#pragma unroll
            for (int i = 0; i < kSmallMMaxStripsPerGroup; ++i)
                if (i == owned)
                    g_keep[i][e] = gv;
        }
    }

    // ---- exchange the strip statistics across the whole grid ----
    wait_published();
    __syncthreads();
    if (tid == 0) {
        atomic_add_device(p.counters, 1u);
        if (!wait_counter(p.counters, gridDim.x, p.wait_ticks))
            atomic_store_device(p.err, 1u);
    }
    __syncthreads();
    {
        // 32 chunks of consecutive strips per row, merged in order, then the
        // 32 chunk results merged in order by one thread per row.
        const int row = tid % (MT * 16);
        const int chunk = tid / (MT * 16);  // 0 .. 512/(16 MT) - 1
        constexpr int kChunks = kThreads / (MT * 16);
        const int per = (p.strips + kChunks - 1) / kChunks;
        float na = 0.0f, mean_a = 0.0f, m2a = 0.0f;
        for (int s = chunk * per; s < (chunk + 1) * per && s < p.strips; ++s) {
            const int cnt = (N - s * kSmallMStripCols < kSmallMStripCols) ? (N - s * kSmallMStripCols)
                                                                           : kSmallMStripCols;
            const floatx2 u = read_pair(p.partials + (size_t)s * (MT * 16) + row);
            merge_stats(na, mean_a, m2a, (float)cnt, u[0], u[1]);
        }
        // chunk counts are implied by position; pass them through LDS as (mean, M2)
        // and recompute the count when merging
        if (chunk < 32) {
            floatx2 o = {mean_a, m2a};
            s_chunk[chunk][row] = o;
        }
        __syncthreads();
        if (tid < MT * 16) {
            float nb_total = 0.0f, mean_t = 0.0f, m2_t = 0.0f;
            for (int c = 0; c < kChunks; ++c) {
                int first = c * per;
                int last = (c + 1) * per < p.strips ? (c + 1) * per : p.strips;
                if (first >= last)
                    break;
                int cols_first = first * kSmallMStripCols;
                int cols_last = last * kSmallMStripCols < N ? last * kSmallMStripCols : N;
                const floatx2 u = s_chunk[c][tid];
                merge_stats(nb_total, mean_t, m2_t, (float)(cols_last - cols_first), u[0], u[1]);
            }
            floatx2 o = {mean_t, 1.0f / sqrtf(m2_t / (float)N + p.eps)};
            s_rst[tid] = o;
        }
        __syncthreads();
    }
    if (tid == 0) {
        if (atomic_add_device(p.counters + 1, 1u) == gridDim.x - 1u) {
            atomic_store_device(p.counters, 0u);
            atomic_store_device(p.counters + 1, 0u);
        }
    }

    // ---- normalise and store ----
    owned = 0;
    for (int strip = blockIdx.x; strip < p.strips; strip += gridDim.x, ++owned) {
#pragma unroll
        for (int e = 0; e < MT; ++e) {
            float gv = 0.0f;
#pragma unroll
            for (int i = 0; i < kSmallMMaxStripsPerGroup; ++i)
                if (i == owned)
                    gv = g_keep[i][e];
            const int el = tid + e * kThreads;
            const int m = el / kSmallMStripCols;
            const int n = strip * kSmallMStripCols + el % kSmallMStripCols;
            if (m < M && n < N) {
                const floatx2 ms = s_rst[m];
                const float ga = p.gamma ? load_as_float(reinterpret_cast<const __bf16 *>(p.gamma) + n) : 1.0f;
                const float be = p.beta ? load_as_float(reinterpret_cast<const __bf16 *>(p.beta) + n) : 0.0f;
                const float y = fmaf((gv - ms[0]) * ms[1], ga, be);
                const float y_other = __shfl_xor(y, 1);
                // even lanes store two adjacent bf16 values (N is a multiple of 8)
                if ((tid & 1) == 0)
                    reinterpret_cast<unsigned *>(p.Y)[((size_t)m * N + n) >> 1] = pack_bf16x2(y, y_other);
            }
        }
    }
}

}  // namespace

hipError_t launch_smallm_kernel(int mt, const SmallMParams &p, int grid, hipStream_t stream)
{
    if (mt == 1)
        hipLaunchKernelGGL(smallm_kernel<1>, dim3(grid), dim3(kThreads), 0, stream, p);
    else
        hipLaunchKernelGGL(smallm_kernel<2>, dim3(grid), dim3(kThreads), 0, stream, p);
    return hipGetLastError();
}

}  // namespace ff
