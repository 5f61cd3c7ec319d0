// Small-M path (M <= 32, bf16) of the fused linear + erf-GELU + LayerNorm
// operator: a streamer, not a tiled GEMM.  The cost is reading W once, so each
// workgroup owns a strip of 32 output columns (32 rows of W, one contiguous
// block), its 8 wavefronts split K, and every wave streams its share with 16-byte
// loads arranged so that eight lanes cover one whole 128-byte line of a row — the
// pattern that reaches the same HBM rate as a linear copy.  The loaded registers
// are MFMA operands as they are: a load instruction covers 8 rows x 64 k, which a
// 16x16x32 MFMA sees as 16 "virtual" rows (row r with k 0..31, row r+8 with k
// 32..63); multiplying once by X[k 0..31] and once by X[k 32..63] leaves the wanted
// products in the lower and upper half of two accumulators, which are added when
// the waves' partial sums are combined in LDS.  M = 16 fills the MFMA's other
// dimension exactly; the tiny X comes from L2.
// The row statistics span all workgroups, so they are exchanged as 8-byte
// (mean, M2) partials through global memory with an arrival counter inside the
// same launch — a second launch would cost a visible fraction of the ~20 us the
// stream itself takes.  This is the paper's bandwidth-bound diagnosis pattern
// (App. B.1: a kernel at DRAM peak is fixed by removing passes over memory, not
// by more arithmetic).
#include "ff_tile.hpp"

namespace ff {

namespace {

constexpr int kWaves = 8;
constexpr int kThreads = 64 * kWaves;
constexpr int kRowGroups = kSmallMStripCols / 8;  // load instructions cover 8 rows of W
constexpr int kSegElems = 64;                     // one 128-byte line of a row
constexpr int kUnroll = 2;                        // segments per batch of loads

__device__ __forceinline__ uintx4 load16_nt(const void *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const uintx4 *>(p));
}

__device__ __forceinline__ floatx4 mfma16(const uintx4 &a, const uintx4 &b, const floatx4 &c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// MT = number of 16-row blocks of X (1: M <= 16, 2: M <= 32).
template <int MT>
__global__ __launch_bounds__(kThreads) void smallm_kernel(const SmallMParams p)
{
    // per-wave partial products, already in (row m, column) order; the row pitch of 33
    // keeps both the scattered writes and the row-wise reads free of bank conflicts
    __shared__ float s_part[kWaves][2][MT * 16][kSmallMStripCols + 1];
    __shared__ floatx2 s_wave[kWaves][MT * 16];       // merged statistics per wave
    __shared__ floatx2 s_rst[MT * 16];                // (mean, rstd) per row

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int M = p.M, N = p.N, K = p.K;
    const __bf16 *X = reinterpret_cast<const __bf16 *>(p.X);
    const __bf16 *W = reinterpret_cast<const __bf16 *>(p.W);

    // W operand: lane -> (row of the 8-row group, 16-byte chunk of the 128-byte segment).
    // MFMA row i = lane & 15 is physical row i & 7 with chunk (i >> 3) * 4 + (lane >> 4).
    const int w_row = lane & 7;
    const int w_chunk = ((lane >> 3) & 1) * 4 + (lane >> 4);
    // X operand: lane -> (row m = lane & 15, k group lane >> 4), lower and upper k half
    const int x_row = lane & 15;
    const int x_kg = lane >> 4;

    // K range of this wave, in 64-element segments
    const int segs = (K + kSegElems - 1) / kSegElems;
    const int per_wave = (segs + kWaves - 1) / kWaves;
    const int sg_begin = wave * per_wave;
    const int sg_end = (sg_begin + per_wave < segs) ? sg_begin + per_wave : segs;
    const int full_end = (sg_end < K / kSegElems) ? sg_end : K / kSegElems;  // whole segments only

    // Final-store ownership: thread `tid` owns elements e = tid + i * 512, i < MT, of a
    // strip's [16 MT][32] block of G (row e / 32, column e % 32).
    // Column e % 32 is the same for every i (512 % 32 == 0), so one bias / gamma / beta
    // value per strip serves all of a thread's elements.
    float g_keep[kSmallMMaxStripsPerGroup][MT];  // my G values of each strip this group owns
    float ga_keep[kSmallMMaxStripsPerGroup], be_keep[kSmallMMaxStripsPerGroup];
    const int my_col = tid % kSmallMStripCols;

    // X rows beyond M are clamped, not zeroed: they only feed output rows that are
    // never stored, and every row's statistics are independent.
    const __bf16 *xrow[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = mt * 16 + x_row;
        xrow[mt] = X + (size_t)(m < M ? m : M - 1) * K + x_kg * 8;
    }

    // Phase timestamps (test hook): thread 0 writes the wall clock at the phase boundaries into
    // timeline[workgroup * kTimelineSlots + k]: 0 start, 1 the first wavefront has streamed its share
    // of K (last strip), 2 all have, 3 statistics published, 4 every workgroup has arrived, 5 statistics
    // merged, 6 stores issued.
    auto stamp = [&](int k) {
        if (p.timeline != nullptr && tid == 0)
            p.timeline[(size_t)blockIdx.x * kTimelineSlots + k] = wall_clock64();
    };
    stamp(0);

    int owned = 0;
    for (int strip = blockIdx.x; strip < p.strips; strip += gridDim.x, ++owned) {
        const int n0 = strip * kSmallMStripCols;
        // this thread's column vectors, requested before the stream so that their
        // latency hides behind it
        const int my_n = n0 + my_col;
        const bool my_ok = my_n < N;
        const __bf16 *vb = reinterpret_cast<const __bf16 *>(p.b);
        const __bf16 *vg = reinterpret_cast<const __bf16 *>(p.gamma);
        const __bf16 *ve = reinterpret_cast<const __bf16 *>(p.beta);
        const float my_bias = (vb && my_ok) ? load_as_float(vb + my_n) : 0.0f;
        const float my_gamma = (vg && my_ok) ? load_as_float(vg + my_n) : 1.0f;
        const float my_beta = (ve && my_ok) ? load_as_float(ve + my_n) : 0.0f;
#pragma unroll
        for (int i = 0; i < kSmallMMaxStripsPerGroup; ++i)
            if (i == owned) {
                ga_keep[i] = my_gamma;
                be_keep[i] = my_beta;
            }
        floatx4 acc[kRowGroups][MT][2];
#pragma unroll
        for (int rg = 0; rg < kRowGroups; ++rg)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                acc[rg][mt][0] = acc[rg][mt][1] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};

        const __bf16 *wrow[kRowGroups];
#pragma unroll
        for (int rg = 0; rg < kRowGroups; ++rg) {
            int n = n0 + rg * 8 + w_row;
            n = n < N ? n : N - 1;
            wrow[rg] = W + (size_t)n * K + w_chunk * 8;
        }

        auto load_batch = [&](int sg0, uintx4 (&wf)[kUnroll][kRowGroups], uintx4 (&xf)[kUnroll][MT][2]) {
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int k = (sg0 + u) * kSegElems;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    xf[u][mt][0] = *reinterpret_cast<const uintx4 *>(xrow[mt] + k);
                    xf[u][mt][1] = *reinterpret_cast<const uintx4 *>(xrow[mt] + k + 32);
                }
#pragma unroll
                for (int rg = 0; rg < kRowGroups; ++rg)
                    wf[u][rg] = load16_nt(wrow[rg] + k);
            }
        };
        auto mma_batch = [&](const uintx4 (&wf)[kUnroll][kRowGroups], const uintx4 (&xf)[kUnroll][MT][2]) {
#pragma unroll
            for (int u = 0; u < kUnroll; ++u)
#pragma unroll
                for (int rg = 0; rg < kRowGroups; ++rg)
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        // A operand = W (register index of the result runs along n),
                        // B operand = X (lane index of the result runs along m)
                        acc[rg][mt][0] = mfma16(wf[u][rg], xf[u][mt][0], acc[rg][mt][0]);
                        acc[rg][mt][1] = mfma16(wf[u][rg], xf[u][mt][1], acc[rg][mt][1]);
                    }
        };

        // Whole segments in batches of kUnroll, software-pipelined two deep so that a
        // batch of loads is always in flight behind the one being multiplied.
        const int nb = full_end > sg_begin ? (full_end - sg_begin) / kUnroll : 0;
        uintx4 wf0[kUnroll][kRowGroups], xf0[kUnroll][MT][2];
        uintx4 wf1[kUnroll][kRowGroups], xf1[kUnroll][MT][2];
        if (nb > 0)
            load_batch(sg_begin, wf0, xf0);
        int bi = 0;
        for (; bi + 2 <= nb; bi += 2) {
            load_batch(sg_begin + (bi + 1) * kUnroll, wf1, xf1);
            mma_batch(wf0, xf0);
            if (bi + 2 < nb)
                load_batch(sg_begin + (bi + 2) * kUnroll, wf0, xf0);
            mma_batch(wf1, xf1);
        }
        if (bi < nb)
            mma_batch(wf0, xf0);
        // remaining segments one at a time; the last one may be cut by K (K % 8 == 0,
        // so 16-byte chunks are whole): chunks of W at or beyond K are zeroed
        for (int sg = sg_begin + nb * kUnroll; sg < sg_end; ++sg) {
            const int k = sg * kSegElems;
            const bool w_in = k + w_chunk * 8 < K;
            const unsigned keep = w_in ? 0xffffffffu : 0u;
            uintx4 x[MT][2];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                x[mt][0] = *reinterpret_cast<const uintx4 *>(xrow[mt] + (k + x_kg * 8 < K ? k : 0));
                x[mt][1] = *reinterpret_cast<const uintx4 *>(xrow[mt] + (k + 32 + x_kg * 8 < K ? k + 32 : 0));
            }
#pragma unroll
            for (int rg = 0; rg < kRowGroups; ++rg) {
                uintx4 w = load16_nt(wrow[rg] + (w_in ? k : 0));
                w &= keep;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    acc[rg][mt][0] = mfma16(w, x[mt][0], acc[rg][mt][0]);
                    acc[rg][mt][1] = mfma16(w, x[mt][1], acc[rg][mt][1]);
                }
            }
        }

        // ---- sum the 8 waves' partial products in wave order ----
        stamp(1);
        __syncthreads();  // s_part / s_g of the previous strip are no longer read
        stamp(2);
        // Result layout of a 16x16 MFMA: lane (j = lane & 15, g = lane >> 4), register t
        // holds result row 4 g + t, column j.  Rows 0..7 of the lower-k accumulator and
        // rows 8..15 of the upper-k accumulator are the wanted products of W row
        // (4 g + t) & 7, so lane groups 0,1 store the former and 2,3 the latter.
        {
            const int j = lane & 15, g = lane >> 4;
            const int hf = g >> 1;
#pragma unroll
            for (int rg = 0; rg < kRowGroups; ++rg)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const float v = hf ? acc[rg][mt][1][t] : acc[rg][mt][0][t];
                        s_part[wave][hf][mt * 16 + j][rg * 8 + 4 * (g & 1) + t] = v;
                    }
        }
        __syncthreads();
        const int nvalid = (N - n0 < kSmallMStripCols) ? (N - n0) : kSmallMStripCols;
#pragma unroll
        for (int e = 0; e < MT; ++e) {
            const int el = tid + e * kThreads;
            const int m = el / kSmallMStripCols;
            const int nl = my_col;
            float z = 0.0f;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) {
                z += s_part[w][0][m][nl];
                z += s_part[w][1][m][nl];
            }
            const float g = my_ok ? gelu_erf(z + my_bias) : 0.0f;
#pragma unroll
            for (int i = 0; i < kSmallMMaxStripsPerGroup; ++i)
                if (i == owned)
                    g_keep[i][e] = g;
            // per-row (mean, M2) of the strip: the 32 columns of a row sit in one half
            // of a wave, reduced with a fixed butterfly (every lane ends with the sums)
            float sum = g;
#pragma unroll
            for (int off = 16; off >= 1; off >>= 1)
                sum += __shfl_xor(sum, off);
            const float mean = sum / (float)nvalid;
            const float d = my_ok ? g - mean : 0.0f;
            float m2 = d * d;
#pragma unroll
            for (int off = 16; off >= 1; off >>= 1)
                m2 += __shfl_xor(m2, off);
            if (nl == 0) {
                floatx2 o = {mean, m2};
                publish_pair(p.partials + (size_t)strip * (MT * 16) + m, o);
            }
        }
    }

    // ---- exchange the strip statistics across the whole grid ----
    stamp(3);
    wait_published();
    __syncthreads();
    const int way = blockIdx.x % kSyncWays;
    if (tid == 0)
        atomic_add_device(p.counters + (size_t)way * kSyncStride, 1u);
    if (wave == 0) {
        // lane l polls way l: workgroups l, l + kSyncWays, ... arrive there
        const int l = lane < kSyncWays ? lane : 0;
        const unsigned target = (gridDim.x + kSyncWays - 1 - l) / kSyncWays + (l == 0 ? (unsigned)p.extra_arrivals : 0u);
        if (!wait_counters_wave(p.counters, target, p.wait_ticks) && lane == 0)
            atomic_store_device(p.err, 1u);
    }
    __syncthreads();
    stamp(4);
    {
        // Every workgroup merges all strips' partials itself, in strip order: thread ->
        // (row, chunk of consecutive strips); chunks of a wave are then folded with
        // directed shuffles (earlier strips on the left), the waves' results through
        // LDS.  Plain loads: the lines were written through by their single owner
        // before the counter could reach its target, and no cache of this XCD can
        // hold an older copy within this launch; workgroups of one XCD share them
        // in its L2 instead of all hitting the same lines in memory.
        constexpr int kRows = MT * 16;
        constexpr int kChunks = kThreads / kRows;       // chunks per workgroup
        constexpr int kChunksPerWave = 64 / kRows;      // 4 (MT = 1) or 2 (MT = 2)
        const int row = tid % kRows;
        const int chunk = tid / kRows;
        const int per = (p.strips + kChunks - 1) / kChunks;
        auto cols_of = [&](int first, int last) {       // columns covered by strips [first, last)
            const int a = first * kSmallMStripCols < N ? first * kSmallMStripCols : N;
            const int b = last * kSmallMStripCols < N ? last * kSmallMStripCols : N;
            return (float)(b - a);
        };
        const int s_begin = chunk * per < p.strips ? chunk * per : p.strips;
        const int s_end = (chunk + 1) * per < p.strips ? (chunk + 1) * per : p.strips;
        float na = 0.0f, mean_a = 0.0f, m2a = 0.0f;
        for (int s0 = s_begin; s0 < s_end; s0 += 8) {
            floatx2 u[8];  // eight loads issued together (never branching: past the end the last
                           // strip is read again and enters the merge with zero columns), merged in order
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int sj = s0 + j < s_end ? s0 + j : s_end - 1;
                u[j] = p.partials[(size_t)sj * kRows + row];
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const bool live = s0 + j < s_end;
                merge_stats(na, mean_a, m2a, live ? cols_of(s0 + j, s0 + j + 1) : 0.0f, u[j][0],
                            live ? u[j][1] : 0.0f);
            }
        }
        // fold the wave's chunks: lane takes the later chunk from lane + kRows * step
#pragma unroll
        for (int step = 1; step < kChunksPerWave; step <<= 1) {
            const float nb = __shfl_down(na, kRows * step);
            const float mb = __shfl_down(mean_a, kRows * step);
            const float qb = __shfl_down(m2a, kRows * step);
            merge_stats(na, mean_a, m2a, nb, mb, qb);
        }
        if (lane < kRows) {
            floatx2 o = {mean_a, m2a};
            s_wave[wave][row] = o;
        }
        __syncthreads();
        if (tid < kRows) {
            floatx2 u[kWaves];
#pragma unroll
            for (int w = 0; w < kWaves; ++w)
                u[w] = s_wave[w][tid];
            float nt = 0.0f, mean_t = 0.0f, m2_t = 0.0f;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) {
                const int first = w * kChunksPerWave * per;
                const int last = (w + 1) * kChunksPerWave * per;
                merge_stats(nt, mean_t, m2_t, cols_of(first, last), u[w][0], u[w][1]);
            }
            floatx2 o = {mean_t, 1.0f / sqrtf(m2_t / (float)N + p.eps)};
            s_rst[tid] = o;
        }
        __syncthreads();
    }
    stamp(5);
    // ---- normalise and store ----
    owned = 0;
    for (int strip = blockIdx.x; strip < p.strips; strip += gridDim.x, ++owned) {
        float ga = 1.0f, be = 0.0f;
#pragma unroll
        for (int i = 0; i < kSmallMMaxStripsPerGroup; ++i)
            if (i == owned) {
                ga = ga_keep[i];
                be = be_keep[i];
            }
#pragma unroll
        for (int e = 0; e < MT; ++e) {
            float gv = 0.0f;
#pragma unroll
            for (int i = 0; i < kSmallMMaxStripsPerGroup; ++i)
                if (i == owned)
                    gv = g_keep[i][e];
            const int el = tid + e * kThreads;
            const int m = el / kSmallMStripCols;
            const int n = strip * kSmallMStripCols + my_col;
            if (m < M && n < N) {
                const floatx2 ms = s_rst[m];
                const float y = fmaf((gv - ms[0]) * ms[1], ga, be);
                const float y_other = __shfl_xor(y, 1);
                // even lanes store two adjacent bf16 values (N is a multiple of 8)
                if ((tid & 1) == 0)
                    reinterpret_cast<unsigned *>(p.Y)[((size_t)m * N + n) >> 1] = pack_bf16x2(y, y_other);
            }
        }
    }

    stamp(6);
    // ---- departure: the last workgroup of the last way re-arms every counter ----
    // (only then has every workgroup left its wait, so no poller can see a counter go back to zero)
    if (tid == 0) {
        const unsigned in_way = (gridDim.x + kSyncWays - 1 - way) / kSyncWays;
        const unsigned ways = gridDim.x < (unsigned)kSyncWays ? gridDim.x : (unsigned)kSyncWays;
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
