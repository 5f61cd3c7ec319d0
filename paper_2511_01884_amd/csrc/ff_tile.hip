// Tiled MFMA path of the fused linear + erf-GELU + LayerNorm operator (gfx950).
//
// One workgroup (4 wavefronts) owns a BM x BN tile of the output and walks K in
// 64-byte slabs.  X and W slabs go HBM -> LDS with 16-byte direct-to-LDS loads
// into a ring of four stages (loads run three slabs ahead of the MFMAs, one
// barrier per slab), and are read back as MFMA fragments one k-step ahead of
// their use, so the matrix pipe does not wait on LDS latency after a barrier.  The MFMA is issued
// "transposed" (A operand = W rows, B operand = X rows), so that a lane's 16
// accumulator registers of a 32x32 block run along N — the LayerNorm reduction
// axis — and the row statistics need only one cross-lane step.
//
// The epilogue never leaves the registers (the fused-epilogue pattern of the
// paper's App. B.1 case, with the "cross-tile aggregation" it names as the hard
// part): bias + GELU in place, per-row (mean, M2) of the tile, exchange of those
// 8-byte partials with the other tiles of the same rows through global memory
// and an arrival counter, merge in fixed order, normalise, convert, and store Y
// through an LDS transpose in 16-byte coalesced rows.  G is never written to
// global memory (Sec. 4: removing the second global read).
//
// Modes: kFused (above), kTwoPass (writes fp32 G and the partials; a second
// kernel normalises — used when a row has more tiles than co-resident
// workgroups), kLinearOnly (test hook: fp32 Z = X W^T + b).
#include "ff_tile.hpp"

namespace ff {

namespace {

constexpr int kWavesN = 2;
constexpr int kWavesM = 2;
constexpr int kThreads = 64 * kWavesN * kWavesM;
constexpr int kRowBytes = 64;   // bytes of one tile row per K slab (4 chunks of 16 B)
constexpr int kChunksPerRow = kRowBytes / 16;
constexpr int kStepsPerSlab = kChunksPerRow / 2;  // a k-step consumes two chunks (one per lane half)
constexpr int kStages = 4;
constexpr int kRowsPerDma = 1024 / kRowBytes;     // one direct-to-LDS instruction fills 1 KiB

template <typename T>
struct Mma;

template <>
struct Mma<__bf16> {
    // One 16-byte fragment per lane holds 8 bf16 along K: one 32x32x16 MFMA.
    static __device__ __forceinline__ void step(const uintx4 &a, const uintx4 &b, floatx16 &c)
    {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                    __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};

template <>
struct Mma<float> {
    // One 16-byte fragment per lane holds 4 floats along K: four 32x32x2 MFMAs.
    static __device__ __forceinline__ void step(const uintx4 &a, const uintx4 &b, floatx16 &c)
    {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[e]), __uint_as_float(b[e]),
                                                     c, 0, 0, 0);
    }
};

// Compiler-level ordering of LDS traffic inside one wavefront (the LDS itself
// serves a wave's requests in issue order).
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Workgroup barrier for the K loop.  Unlike __syncthreads() it carries no fence,
// so it does not wait for outstanding global loads: direct-to-LDS loads of later
// slabs stay in flight across it (their completion is awaited explicitly with
// vmcnt).  It waits for this wave's own LDS reads and writes, and the barrier
// instruction itself is a compiler-level ordering point for memory operations.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0) only
    __builtin_amdgcn_s_barrier();
}

// Ordering point for the instruction scheduler: the listed accumulators must have
// been produced before it, and no memory operation moves across it.
__device__ __forceinline__ void pin_order(floatx16 &c0) { asm volatile("" : "+a"(c0) : : "memory"); }
__device__ __forceinline__ void pin_order(floatx16 &c0, floatx16 &c1)
{
    asm volatile("" : "+a"(c0), "+a"(c1) : : "memory");
}

// LDS placement of 16-byte chunk `c` (0..3) of tile row `row`: chunks are XORed
// with row bits so that the 16 consecutive rows a fragment read touches per pass
// (stride 64 B) spread over all 64 banks.
__device__ __forceinline__ int swizzle_of_row(int row) { return (row >> 2) & 3; }

// MFMA instructions one fragment pair costs per k-step (scheduling hints only).
template <typename T> struct MmaCount { static constexpr int value = 1; };
template <> struct MmaCount<float> { static constexpr int value = 4; };

template <typename T, int WTN, int WTM, int MODE>
__global__ __launch_bounds__(kThreads) void tile_kernel(const TileParams p)
{
    constexpr int BN = kWavesN * WTN * 32;
    constexpr int BM = kWavesM * WTM * 32;
    constexpr int kChunkElems = 16 / (int)sizeof(T);
    constexpr int kSlabElems = kRowBytes / (int)sizeof(T);
    constexpr int kABytes = BN * kRowBytes;
    constexpr int kBBytes = BM * kRowBytes;
    constexpr int kStageBytes = kABytes + kBBytes;
    // direct-to-LDS instructions per wave per slab
    constexpr int kDmaA = BN / kRowsPerDma / (kWavesN * kWavesM);
    constexpr int kDmaB = BM / kRowsPerDma / (kWavesN * kWavesM);
    constexpr int kDmaPerSlab = kDmaA + kDmaB;
    // epilogue LDS regions (reuse the stage buffers)
    using OutT = typename std::conditional<MODE == kFused, T, float>::type;
    constexpr int kOutRowBytes = WTN * 32 * (int)sizeof(OutT);
    constexpr int kOutPitch = kOutRowBytes + 16;
    constexpr int kOffPrm = 0;                               // 3 * BN floats
    constexpr int kOffWst = kOffPrm + 3 * BN * 4;            // kWavesN * BM float2
    constexpr int kOffRst = kOffWst + kWavesN * BM * 8;      // BM float2
    constexpr int kOffOut = (kOffRst + BM * 8 + 1023) & ~1023;
    constexpr int kEpiBytes = kOffOut + kWavesN * kWavesM * 32 * kOutPitch;
    constexpr int kSmemBytes = (kStages * kStageBytes > kEpiBytes) ? kStages * kStageBytes : kEpiBytes;

    __shared__ __attribute__((aligned(1024))) char smem[kSmemBytes];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn = wave % kWavesN;
    const int wm = wave / kWavesN;
    const int h = lane >> 5;
    const int l32 = lane & 31;

    const int M = p.M, N = p.N, K = p.K;
    const int slabs = (K + kSlabElems - 1) / kSlabElems;
    const bool k_ragged = (K % kSlabElems) != 0;
    const size_t row_stride = (size_t)K * sizeof(T);

    // fragment read offsets (bytes inside a stage); k-step s reads chunk (2s + h) ^ swizzle
    const int frag_swz = swizzle_of_row(l32);
    const int a_frag_base = (wn * WTN * 32 + l32) * kRowBytes;
    const int b_frag_base = kABytes + (wm * WTM * 32 + l32) * kRowBytes;

    // DMA lane geometry: lane -> (row within a 16-row group, stored chunk slot)
    const int dma_r = lane / kChunksPerRow;
    const int dma_cs = lane % kChunksPerRow;

    for (int t = blockIdx.x; t < p.rounds * (int)gridDim.x; t += gridDim.x) {
        // ---- tile coordinates (XCD-aware order inside a round when enabled) ----
        int rb, cb;
        if (p.swz_sc > 0) {
            const int round = t / (int)gridDim.x;
            const int xcd = blockIdx.x & 7;
            const int slot = blockIdx.x >> 3;
            const int sc = p.swz_sc, sr = 32 / sc;
            const int across = p.NT / sc;
            const int sbr = xcd / across, sbc = xcd % across;
            rb = round * ((int)gridDim.x / p.NT) + sbr * sr + slot / sc;
            cb = sbc * sc + slot % sc;
        } else {
            rb = t / p.NT;
            cb = t % p.NT;
        }
        if (rb >= p.RB)
            continue;  // uniform for the workgroup
        const int m0 = rb * BM;
        const int n0 = cb * BN;

        // ---- per-lane byte offsets of the DMA sources, relative to the tile's first row ----
        const char *w_tile = (const char *)p.W + (size_t)n0 * row_stride;
        const char *x_tile = (const char *)p.X + (size_t)m0 * row_stride;
        unsigned offa[kDmaA], offb[kDmaB];
#pragma unroll
        for (int j = 0; j < kDmaA; ++j) {
            const int row = wave * (BN / 4) + j * kRowsPerDma + dma_r;
            const int c = dma_cs ^ swizzle_of_row(row);
            const int rr = (n0 + row < N) ? row : (N - 1 - n0);  // clamp to the last valid row
            offa[j] = (unsigned)rr * (unsigned)row_stride + c * 16;
        }
#pragma unroll
        for (int j = 0; j < kDmaB; ++j) {
            const int row = wave * (BM / 4) + j * kRowsPerDma + dma_r;
            const int c = dma_cs ^ swizzle_of_row(row);
            const int rr = (m0 + row < M) ? row : (M - 1 - m0);
            offb[j] = (unsigned)rr * (unsigned)row_stride + c * 16;
        }

        // full slab: direct-to-LDS, nothing passes through registers.  dma_one issues
        // the x-th of the wave's kDmaPerSlab instructions (W rows first, then X rows).
        auto dma_one = [&](int slab, int x) {
            const int stage = slab % kStages;
            if (x < kDmaA) {
                char *sa = smem + stage * kStageBytes + wave * (BN / 4) * kRowBytes;
                const char *wk = w_tile + (size_t)slab * kRowBytes;
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void *)(wk + offa[x < kDmaA ? x : 0]),
                    (__attribute__((address_space(3))) void *)(sa + x * 1024), 16, 0, 0);
            } else {
                const int y = x - kDmaA;
                char *sb = smem + stage * kStageBytes + kABytes + wave * (BM / 4) * kRowBytes;
                const char *xk = x_tile + (size_t)slab * kRowBytes;
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void *)(xk + offb[y >= 0 && y < kDmaB ? y : 0]),
                    (__attribute__((address_space(3))) void *)(sb + y * 1024), 16, 0, 0);
            }
        };
        auto issue_full = [&](int slab) {
#pragma unroll
            for (int x = 0; x < kDmaPerSlab; ++x)
                dma_one(slab, x);
        };
        // any slab: the last one may be cut by K, then chunks at or beyond K are zero-filled
        auto issue_any = [&](int slab) {
            if (!k_ragged || slab + 1 < slabs) {
                issue_full(slab);
                return;
            }
            const int stage = slab % kStages;
            char *sa = smem + stage * kStageBytes + wave * (BN / 4) * kRowBytes;
            char *sb = smem + stage * kStageBytes + kABytes + wave * (BM / 4) * kRowBytes;
            const char *wk = w_tile + (size_t)slab * kRowBytes;
            const char *xk = x_tile + (size_t)slab * kRowBytes;
#pragma unroll
            for (int j = 0; j < kDmaA; ++j) {
                const int row = wave * (BN / 4) + j * kRowsPerDma + dma_r;
                const int c = dma_cs ^ swizzle_of_row(row);
                const bool in = slab * kSlabElems + c * kChunkElems < K;
                uintx4 v = *reinterpret_cast<const uintx4 *>(in ? wk + offa[j] : w_tile);
                v &= in ? 0xffffffffu : 0u;
                *reinterpret_cast<uintx4 *>(sa + j * 1024 + lane * 16) = v;
            }
#pragma unroll
            for (int j = 0; j < kDmaB; ++j) {
                const int row = wave * (BM / 4) + j * kRowsPerDma + dma_r;
                const int c = dma_cs ^ swizzle_of_row(row);
                const bool in = slab * kSlabElems + c * kChunkElems < K;
                uintx4 v = *reinterpret_cast<const uintx4 *>(in ? xk + offb[j] : x_tile);
                v &= in ? 0xffffffffu : 0u;
                *reinterpret_cast<uintx4 *>(sb + j * 1024 + lane * 16) = v;
            }
        };

        floatx16 acc[WTN][WTM];
#pragma unroll
        for (int i = 0; i < WTN; ++i)
#pragma unroll
            for (int j = 0; j < WTM; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    acc[i][j][r] = 0.0f;

        uintx4 fa[2][WTN], fb[2][WTM];  // fragment registers, double-buffered by k-step
        // x-th fragment read of (slab, k-step s): W fragments first, then X fragments
        auto read_one = [&](int slab, int s, int x, uintx4 (&a)[WTN], uintx4 (&b)[WTM]) {
            const char *sbase = smem + (slab % kStages) * kStageBytes;
            const int coff = ((2 * s + h) ^ frag_swz) << 4;
            if (x < WTN)
                a[x < WTN ? x : 0] = *reinterpret_cast<const uintx4 *>(
                    sbase + a_frag_base + x * 32 * kRowBytes + coff);
            else
                b[x >= WTN ? x - WTN : 0] = *reinterpret_cast<const uintx4 *>(
                    sbase + b_frag_base + (x - WTN) * 32 * kRowBytes + coff);
        };
        auto load_frags = [&](int slab, int s, uintx4 (&a)[WTN], uintx4 (&b)[WTM]) {
#pragma unroll
            for (int x = 0; x < WTN + WTM; ++x)
                read_one(slab, s, x, a, b);
        };
        // the MFMAs are issued in kGroups groups of kPerGroup fragment pairs
        constexpr int kGroups = WTN + WTM;
        constexpr int kPerGroup = WTN * WTM / kGroups;
        static_assert(kPerGroup * kGroups == WTN * WTM, "pairs must split evenly over the groups");
        static_assert(kPerGroup == 1 || kPerGroup == 2, "pin_order takes one or two accumulators");
        auto mma_group = [&](int g, const uintx4 (&a)[WTN], const uintx4 (&b)[WTM]) {
#pragma unroll
            for (int q = 0; q < kPerGroup; ++q) {
                const int pair = g * kPerGroup + q;
                Mma<T>::step(a[pair / WTM], b[pair % WTM], acc[pair / WTM][pair % WTM]);
            }
        };
        auto pin_group = [&](int g) {
            const int p0 = g * kPerGroup;
            if (kPerGroup == 2)
                pin_order(acc[p0 / WTM][p0 % WTM], acc[(p0 + 1) / WTM][(p0 + 1) % WTM]);
            else
                pin_order(acc[p0 / WTM][p0 % WTM]);
        };
        auto mma_all = [&](const uintx4 (&a)[WTN], const uintx4 (&b)[WTM]) {
#pragma unroll
            for (int g = 0; g < kGroups; ++g)
                mma_group(g, a, b);
        };

        // ---- main loop over K slabs ----
        // Invariant at the top of iteration i (after barrier B_i): slabs <= i+1 are
        // visible in LDS to every wave, every wave has finished reading slab i-1, and
        // the fragments of (slab i, k-step 0) are already on their way to registers.
        static_assert(kStepsPerSlab == 2, "the loop body below is written for two k-steps per slab");
        static_assert(kDmaPerSlab <= kGroups, "one DMA instruction per MFMA group at most");
        __syncthreads();  // previous tile's epilogue is done with the LDS
        for (int sl = 0; sl < 3 && sl < slabs; ++sl)
            issue_any(sl);
        if (slabs > 2)
            __builtin_amdgcn_s_waitcnt(0x0f70 | (kDmaPerSlab & 15) | ((kDmaPerSlab >> 4) << 14));
        else
            __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0)
        lds_barrier();
        load_frags(0, 0, fa[0], fb[0]);

        // steady iterations: the slab issued (i+3) exists and is a full one.  The
        // instruction order below is the intended issue order (one DMA and one LDS
        // read in the shadow of each group of MFMAs); the scheduling fences keep it.
        const int n_steady = slabs - 3 - (k_ragged ? 1 : 0);
        int i = 0;
        for (; i < n_steady; ++i) {
#pragma unroll
            for (int g = 0; g < kGroups; ++g) {
                if (g < kDmaPerSlab)
                    dma_one(i + 3, g);
                read_one(i, 1, g, fa[1], fb[1]);
                mma_group(g, fa[0], fb[0]);
                pin_group(g);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int g = 0; g < kGroups; ++g) {
                mma_group(g, fa[1], fb[1]);
                read_one(i + 1, 0, g, fa[0], fb[0]);
                pin_group(g);
                __builtin_amdgcn_sched_barrier(0);
            }
            // all but the newest slab's loads have landed; then B_{i+1}
            __builtin_amdgcn_s_waitcnt(0x0f70 | (kDmaPerSlab & 15) | ((kDmaPerSlab >> 4) << 14));
            lds_barrier();
        }
        // last (up to four) iterations: nothing, or a K-cut slab, left to issue
        for (; i < slabs; ++i) {
            if (i + 3 < slabs)
                issue_any(i + 3);
            load_frags(i, 1, fa[1], fb[1]);
            mma_all(fa[0], fb[0]);
            if (i + 1 < slabs)
                load_frags(i + 1, 0, fa[0], fb[0]);
            mma_all(fa[1], fb[1]);
            __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0)
            lds_barrier();
        }
        __syncthreads();  // all fragment reads done: LDS becomes epilogue scratch

        // ---- epilogue ----
        float *s_b = reinterpret_cast<float *>(smem + kOffPrm);
        float *s_g = s_b + BN;
        float *s_be = s_g + BN;
        floatx2 *s_wst = reinterpret_cast<floatx2 *>(smem + kOffWst);
        floatx2 *s_rst = reinterpret_cast<floatx2 *>(smem + kOffRst);
        char *s_out = smem + kOffOut + wave * 32 * kOutPitch;

        for (int c = tid; c < BN; c += kThreads) {
            const int n = n0 + c;
            const bool ok = n < N;
            s_b[c] = (ok && p.b) ? load_as_float(reinterpret_cast<const T *>(p.b) + n) : 0.0f;
            s_g[c] = (ok && p.gamma) ? load_as_float(reinterpret_cast<const T *>(p.gamma) + n) : 1.0f;
            s_be[c] = (ok && p.beta) ? load_as_float(reinterpret_cast<const T *>(p.beta) + n) : 0.0f;
        }
        __syncthreads();

        const int ncol_wave = wn * WTN * 32;            // wave's first column inside the tile
        const int nvalid_tile = (N - n0 < BN) ? (N - n0) : BN;
        const bool ragged_n = nvalid_tile < BN;

        // bias + GELU, in place in the accumulators
#pragma unroll
        for (int i = 0; i < WTN; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int cl = ncol_wave + i * 32 + q * 8 + h * 4;
                const floatx4 bb = *reinterpret_cast<const floatx4 *>(s_b + cl);
#pragma unroll
                for (int j = 0; j < WTM; ++j)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float z = acc[i][j][q * 4 + e] + bb[e];
                        float g = (MODE == kLinearOnly) ? z : gelu_erf(z);
                        if (MODE != kLinearOnly && ragged_n && cl + e >= nvalid_tile)
                            g = 0.0f;
                        acc[i][j][q * 4 + e] = g;
                    }
            }

        if (MODE != kLinearOnly) {
            // per-row (mean, M2) over this wave's columns, then over the tile
            int cntw_i = nvalid_tile - ncol_wave;
            cntw_i = cntw_i < 0 ? 0 : (cntw_i > WTN * 32 ? WTN * 32 : cntw_i);
            const float cntw = (float)cntw_i;
#pragma unroll
            for (int j = 0; j < WTM; ++j) {
                float s = 0.0f;
#pragma unroll
                for (int i = 0; i < WTN; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        s += acc[i][j][r];
                s += __shfl_xor(s, 32);
                const float mean = cntw_i > 0 ? s / cntw : 0.0f;
                float m2 = 0.0f;
#pragma unroll
                for (int i = 0; i < WTN; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        float d = acc[i][j][r] - mean;
                        if (ragged_n) {
                            const int cl = ncol_wave + i * 32 + (r >> 2) * 8 + h * 4 + (r & 3);
                            d = cl < nvalid_tile ? d : 0.0f;
                        }
                        m2 = fmaf(d, d, m2);
                    }
                m2 += __shfl_xor(m2, 32);
                if (h == 0) {
                    floatx2 v = {mean, m2};
                    s_wst[wn * BM + wm * WTM * 32 + j * 32 + l32] = v;
                }
            }
            __syncthreads();
            if (tid < BM) {
                int c0 = nvalid_tile < WTN * 32 ? nvalid_tile : WTN * 32;
                float na = (float)c0;
                floatx2 v = s_wst[tid];
                float mean_a = v[0], m2a = v[1];
#pragma unroll
                for (int w = 1; w < kWavesN; ++w) {
                    int cw = nvalid_tile - w * WTN * 32;
                    cw = cw < 0 ? 0 : (cw > WTN * 32 ? WTN * 32 : cw);
                    const floatx2 u = s_wst[w * BM + tid];
                    merge_stats(na, mean_a, m2a, (float)cw, u[0], u[1]);
                }
                floatx2 o = {mean_a, m2a};
                if (MODE == kFused)
                    publish_pair(p.partials + ((size_t)rb * p.NT + cb) * BM + tid, o);
                else
                    p.partials[((size_t)rb * p.NT + cb) * BM + tid] = o;
            }
        }

        if (MODE == kFused) {
            // exchange with the other tiles of these rows
            wait_published();
            __syncthreads();
            if (tid == 0) {
                unsigned *arrive = p.counters + 2 * (size_t)rb;
                atomic_add_device(arrive, 1u);
                if (!wait_counter(arrive, (unsigned)p.NT, p.wait_ticks))
                    atomic_store_device(p.err, 1u);
            }
            __syncthreads();
            if (tid < BM) {
                float na = 0.0f, mean_a = 0.0f, m2a = 0.0f;
                for (int c = 0; c < p.NT; ++c) {
                    const int cnt = (N - c * BN < BN) ? (N - c * BN) : BN;
                    const floatx2 u = read_pair(p.partials + ((size_t)rb * p.NT + c) * BM + tid);
                    merge_stats(na, mean_a, m2a, (float)cnt, u[0], u[1]);
                }
                const float var = m2a / (float)N;
                floatx2 o = {mean_a, 1.0f / sqrtf(var + p.eps)};
                s_rst[tid] = o;
            }
            __syncthreads();
            if (tid == 0) {
                // the last tile to have read the partials re-arms the counters
                unsigned *cnt = p.counters + 2 * (size_t)rb;
                if (atomic_add_device(cnt + 1, 1u) == (unsigned)p.NT - 1u) {
                    atomic_store_device(cnt, 0u);
                    atomic_store_device(cnt + 1, 0u);
                }
            }
        }

        // ---- (normalise,) convert, transpose through LDS, store 16-byte rows ----
        OutT *out_base = (MODE == kFused) ? reinterpret_cast<OutT *>(p.Y)
                                          : reinterpret_cast<OutT *>(p.F);
#pragma unroll
        for (int j = 0; j < WTM; ++j) {
            float mu = 0.0f, rstd = 1.0f;
            if (MODE == kFused) {
                const floatx2 ms = s_rst[wm * WTM * 32 + j * 32 + l32];
                mu = ms[0];
                rstd = ms[1];
            }
#pragma unroll
            for (int i = 0; i < WTN; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int cw = i * 32 + q * 8 + h * 4;  // column inside the wave's strip
                    float y[4];
                    if (MODE == kFused) {
                        const floatx4 ga4 = *reinterpret_cast<const floatx4 *>(s_g + ncol_wave + cw);
                        const floatx4 be4 = *reinterpret_cast<const floatx4 *>(s_be + ncol_wave + cw);
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            y[e] = fmaf((acc[i][j][q * 4 + e] - mu) * rstd, ga4[e], be4[e]);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            y[e] = acc[i][j][q * 4 + e];
                    }
                    char *dst = s_out + l32 * kOutPitch + cw * (int)sizeof(OutT);
                    if (sizeof(OutT) == 2) {
                        uintx2 v = {pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3])};
                        *reinterpret_cast<uintx2 *>(dst) = v;
                    } else {
                        floatx4 v = {y[0], y[1], y[2], y[3]};
                        *reinterpret_cast<floatx4 *>(dst) = v;
                    }
                }
            wave_lds_sync();
            constexpr int kCpr = kOutRowBytes / 16;  // 16-byte chunks per row
            constexpr int kIters = 32 * kCpr / 64;
            constexpr int kChunkOut = 16 / (int)sizeof(OutT);
#pragma unroll
            for (int it = 0; it < kIters; ++it) {
                const int idx = it * 64 + lane;
                const int r = idx / kCpr;
                const int c = idx % kCpr;
                const uintx4 v = *reinterpret_cast<const uintx4 *>(s_out + r * kOutPitch + c * 16);
                const int gm = m0 + wm * WTM * 32 + j * 32 + r;
                const int gn = n0 + ncol_wave + c * kChunkOut;
                if (gm < M && gn < N)
                    *reinterpret_cast<uintx4 *>(out_base + (size_t)gm * N + gn) = v;
            }
            wave_lds_sync();
        }
    }
}

// Second kernel of the two-pass variant: one workgroup per row.  Merges the
// row's per-tile (mean, M2) in a fixed order, then normalises the fp32 G row.
template <typename T>
__global__ __launch_bounds__(256) void finalize_kernel(const FinalizeParams p)
{
    __shared__ float s_stat[2];
    const int m = blockIdx.x;
    const int tid = threadIdx.x;
    const int rb = m / p.BM;
    const int r = m % p.BM;
    if (tid < 64) {
        float na = 0.0f, mean_a = 0.0f, m2a = 0.0f;
        for (int c = tid; c < p.NT; c += 64) {
            const int cnt = (p.N - c * p.BN < p.BN) ? (p.N - c * p.BN) : p.BN;
            const floatx2 u = p.partials[((size_t)rb * p.NT + c) * p.BM + r];
            merge_stats(na, mean_a, m2a, (float)cnt, u[0], u[1]);
        }
        for (int off = 32; off >= 1; off >>= 1) {
            const float nb = __shfl_down(na, off);
            const float mb = __shfl_down(mean_a, off);
            const float qb = __shfl_down(m2a, off);
            merge_stats(na, mean_a, m2a, nb, mb, qb);
        }
        if (tid == 0) {
            s_stat[0] = mean_a;
            s_stat[1] = 1.0f / sqrtf(m2a / (float)p.N + p.eps);
        }
    }
    __syncthreads();
    const float mu = s_stat[0], rstd = s_stat[1];
    const float *g = p.G + (size_t)m * p.N;
    T *y = reinterpret_cast<T *>(p.Y) + (size_t)m * p.N;
    const T *gamma = reinterpret_cast<const T *>(p.gamma);
    const T *beta = reinterpret_cast<const T *>(p.beta);
    for (int n = tid * 4; n < p.N; n += 256 * 4) {
        const floatx4 gv = *reinterpret_cast<const floatx4 *>(g + n);
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float ga = gamma ? load_as_float(gamma + n + e) : 1.0f;
            const float be = beta ? load_as_float(beta + n + e) : 0.0f;
            o[e] = fmaf((gv[e] - mu) * rstd, ga, be);
        }
        if (sizeof(T) == 2) {
            uintx2 v = {pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3])};
            *reinterpret_cast<uintx2 *>(y + n) = v;
        } else {
            floatx4 v = {o[0], o[1], o[2], o[3]};
            *reinterpret_cast<floatx4 *>(y + n) = v;
        }
    }
}

template <typename T, int WT, int MODE>
hipError_t launch_tile(const TileParams &p, int grid, hipStream_t stream)
{
    hipLaunchKernelGGL((tile_kernel<T, WT, WT, MODE>), dim3(grid), dim3(kThreads), 0, stream, p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_tile_kernel(bool bf16, int tile, int mode, const TileParams &p, int grid,
                              hipStream_t stream)
{
#define FF_DISPATCH(T, WT)                                              \
    switch (mode) {                                                     \
    case kFused: return launch_tile<T, WT, kFused>(p, grid, stream);    \
    case kTwoPass: return launch_tile<T, WT, kTwoPass>(p, grid, stream); \
    default: return launch_tile<T, WT, kLinearOnly>(p, grid, stream);   \
    }
    if (bf16) {
        if (tile == 256) { FF_DISPATCH(__bf16, 4) }
        FF_DISPATCH(__bf16, 2)
    }
    if (tile == 256) { FF_DISPATCH(float, 4) }
    FF_DISPATCH(float, 2)
#undef FF_DISPATCH
}

hipError_t launch_finalize_kernel(bool bf16, const FinalizeParams &p, hipStream_t stream)
{
    if (bf16)
        hipLaunchKernelGGL(finalize_kernel<__bf16>, dim3(p.M), dim3(256), 0, stream, p);
    else
        hipLaunchKernelGGL(finalize_kernel<float>, dim3(p.M), dim3(256), 0, stream, p);
    return hipGetLastError();
}

}  // namespace ff
