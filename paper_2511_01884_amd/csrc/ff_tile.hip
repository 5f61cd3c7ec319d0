// Tiled MFMA path of the fused linear + erf-GELU + LayerNorm operator (gfx950).
//
// One workgroup (4 or 8 wavefronts) owns a BM x BN tile of the output and walks K in
// 128-byte slabs (whole cache lines: one L2 request per line).  X and W slabs go
// HBM -> LDS with 16-byte direct-to-LDS loads into two stages; the loads of the
// next slab are issued in the shadow of the MFMAs, the single barrier per slab
// sits before the last k-step, and MFMA fragments are read one k-step ahead of
// their use, so the matrix pipe does not wait on LDS latency after the barrier.  The MFMA is issued
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

constexpr int kRowBytes = 128;  // bytes of one tile row per K slab (8 chunks of 16 B)
constexpr int kChunksPerRow = kRowBytes / 16;
constexpr int kStepsPerSlab = kChunksPerRow / 2;  // a k-step consumes two chunks (one per lane half)
constexpr int kStages = 2;
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

// Ordering point for the instruction scheduler: the listed accumulators must have
// been produced before it, and no memory operation moves across it.
__device__ __forceinline__ void pin_order(floatx16 &c0) { asm volatile("" : "+a"(c0) : : "memory"); }
__device__ __forceinline__ void pin_order(floatx16 &c0, floatx16 &c1)
{
    asm volatile("" : "+a"(c0), "+a"(c1) : : "memory");
}

// The lane index, computed where it is asked for: the compiler can neither move the computation out
// of a loop nor keep its result across one (values that the K loop does not use would have to be
// carried across it in scratch memory).
__device__ __forceinline__ int opaque_lane()
{
    int l;
    asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(l));
    return l;
}
// The value of a uniform integer, hidden from the optimiser in the same way.
__device__ __forceinline__ int opaque_uniform(int v)
{
    int r;
    asm volatile("s_mov_b32 %0, %1" : "=s"(r) : "s"(v));
    return r;
}
// The other half-wave's value (lane ^ 32), through the LDS crossbar.
__device__ __forceinline__ float swap_halves(float v, int lane)
{
    return __int_as_float(__builtin_amdgcn_ds_bpermute((lane ^ 32) << 2, __float_as_int(v)));
}

// LDS placement of 16-byte chunk `c` (0..7) of tile row `row`: chunks are XORed
// with row bits so that the consecutive rows a fragment read touches per pass
// (stride 128 B) spread over all banks, for 8-lane and for 16-lane passes.
__device__ __forceinline__ int swizzle_of_row(int row) { return (row & 7) ^ ((row >> 3) & 1); }

// MFMA instructions one fragment pair costs per k-step (scheduling hints only).
template <typename T> struct MmaCount { static constexpr int value = 1; };
template <> struct MmaCount<float> { static constexpr int value = 4; };

// RAGGED_N: N is not a multiple of the tile width, so the last tile of each row
// masks the columns at or beyond N in the statistics (chosen on the host).
//
// Wave layout: kWavesN x kWavesM wavefronts, each owning WTN x WTM MFMA blocks of 32 x 32.  The
// 256-tile runs as 2 x 4 wavefronts of 4 x 2 blocks (two wavefronts per SIMD: 128 accumulator
// registers each, and eight wavefronts keep twice as many loads in flight on the L2 -> LDS path
// as four) or as 2 x 2 wavefronts of 4 x 4 blocks; the 128- and 64-tiles as 2 x 2 wavefronts, two
// workgroups per compute unit (second launch bound: two wavefronts per SIMD must fit).
//
// PIPE selects how the K slabs reach the LDS.  kPipeDma: W and X slabs both by direct-to-LDS loads
// into two stages (one workgroup per compute unit at 256 x 256; the whole LDS).  kPipeXReg: the W
// slab by direct-to-LDS loads into two stages, the X slab through registers into a single buffer
// (loaded a slab ahead, written between two barriers once everyone has read the previous one).
// That fits a 256-column x 128-row tile into half the LDS (2 x 32 KB + 16 KB), so that two
// workgroups can share a compute unit: while one is in its epilogue (vector ALU, exchange, stores) the
// other's K loop keeps the matrix pipe busy, and each covers the other's barrier stalls.  Measured, two
// such workgroups per unit lose to one 256 x 256 tile (1.5 times the L2 -> LDS bytes per flop); the
// shape earns its place one per unit, on problems whose 256 x 256 tiles would leave half the units idle.
template <typename T, int kWavesN, int kWavesM, int WTN, int WTM, int MODE, bool RAGGED_N, int PIPE>
__global__ __launch_bounds__(64 * kWavesN * kWavesM, (kWavesN * kWavesM * WTN * WTM <= 32) ? 2 : 1)
void tile_kernel(const TileParams p)
{
#if defined(__HIP_DEVICE_COMPILE__)  // the body uses device-only types (buffer descriptors)
    constexpr int kWaves = kWavesN * kWavesM;
    constexpr int kThreads = 64 * kWaves;
    constexpr int BN = kWavesN * WTN * 32;
    constexpr int BM = kWavesM * WTM * 32;
    constexpr int kChunkElems = 16 / (int)sizeof(T);
    constexpr int kSlabElems = kRowBytes / (int)sizeof(T);
    constexpr int kABytes = BN * kRowBytes;
    constexpr int kBBytes = BM * kRowBytes;
    // LDS placement of the slabs: W of slab s at (s % 2) * kWStride, X of slab s at kXBase + (s % 2) * kXStride
    constexpr bool kXReg = PIPE == kPipeXReg;
    constexpr int kStageBytes = kABytes + kBBytes;
    constexpr int kWStride = kXReg ? kABytes : kStageBytes;
    constexpr int kXBase = kXReg ? kStages * kABytes : kABytes;
    constexpr int kXStride = kXReg ? 0 : kStageBytes;
    constexpr int kSlabLdsBytes = kXReg ? kStages * kABytes + kBBytes : kStages * kStageBytes;
    // direct-to-LDS instructions per wave per slab
    constexpr int kDmaA = BN / kRowsPerDma / kWaves;
    constexpr int kDmaB = BM / kRowsPerDma / kWaves;
    constexpr int kDmaPerSlab = kDmaA + kDmaB;
    // epilogue LDS regions (reuse the stage buffers)
    using OutT = typename std::conditional<MODE == kFused, T, float>::type;
    constexpr int kOutRowBytes = WTN * 32 * (int)sizeof(OutT);
    constexpr int kOutPitch = kOutRowBytes + 16;
    constexpr int kOffPrm = 0;                               // 3 * BN floats
    constexpr int kOffWst = kOffPrm + 3 * BN * 4;            // kWavesN * BM float2
    constexpr int kOffRst = kOffWst + kWavesN * BM * 8;      // BM float2
    constexpr int kOffOut = (kOffRst + BM * 8 + 1023) & ~1023;
    constexpr int kEpiBytes = kOffOut + kWaves * 32 * kOutPitch;
    constexpr int kSmemBytes = (kSlabLdsBytes > kEpiBytes) ? kSlabLdsBytes : kEpiBytes;

    // One LDS object for everything: with a second one the compiler can no longer tell the DMA's LDS
    // writes from the fragment reads and waits for all loads in flight before every read.
    constexpr int kPrmEarlyBytes = (PIPE != kPipeXReg) ? 3 * BN * 4 : 0;
    __shared__ __attribute__((aligned(1024))) char smem[kSmemBytes + kPrmEarlyBytes];
    // Bias, gamma and beta of the tile's columns.  With both operands travelling by DMA the three
    // vectors are requested ahead of the first slab and parked in LDS of their own when it has
    // landed, so that the epilogue finds them there; the register-staged pipeline, whose two
    // workgroups per compute unit leave no LDS to spare, loads them when the K loop is over.
    constexpr bool kPrmEarly = !kXReg;
    constexpr int kPrmPerThread = (3 * BN + kThreads - 1) / kThreads;
    float *s_prm_early = reinterpret_cast<float *>(smem + kSmemBytes);

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wn = wave % kWavesN;
    const int wm = wave / kWavesN;

    // Phase timestamps (test hook): when a timeline buffer is bound, thread 0 of every workgroup writes
    // the wall clock at the phase boundaries of each of its first `timeline_rounds` tiles into
    // timeline[(round * grid + workgroup) * kTimelineSlots + k].
    int round = 0;
    bool stamper = false;  // thread 0 of the workgroup, decided per tile
    auto stamp = [&](int k) {
        if (p.timeline != nullptr && stamper && round < p.timeline_rounds)
            p.timeline[((size_t)round * gridDim.x + blockIdx.x) * kTimelineSlots + k] =
                k < kTimelineCycleSlot ? wall_clock64() : clock64();
    };

    // Two workgroups per compute unit started together would run their K loops and their epilogues
    // in step; the second half of the grid starts late by about an epilogue's length instead, so
    // that one workgroup's epilogue falls into the other's K loop from the first tile on.
    if (p.stagger_ticks > 0 && blockIdx.x >= (gridDim.x >> 1)) {
        const long long t0 = wall_clock64();
        while (wall_clock64() - t0 < p.stagger_ticks)
            __builtin_amdgcn_s_sleep(16);
    }

    bool first_tile = true;
    for (; round < p.rounds; ++round) {
        // ---- tile coordinates (XCD-aware order inside a round when enabled) ----
        int rb, cb;
        if (p.swz_sc_log2 >= 0) {
            // 8 XCDs x (grid / 8) workgroups, grid and NT powers of two: all quotients are shifts.
            // XCD x takes a block of sr x sc tiles (sc = 1 << swz_sc_log2 columns, sr = grid / 8 / sc
            // rows) of the round's (grid / NT) x NT tiles; the workgroups of the second half of the
            // grid take the lower rows of their XCD's block.
            const int xcd = blockIdx.x & 7;
            const int slot = blockIdx.x >> 3;
            const int scl = p.swz_sc_log2;
            const int across_log2 = p.nt_log2 - scl;
            const int sbr = xcd >> across_log2, sbc = xcd & ((1 << across_log2) - 1);
            rb = (round << (p.grid_log2 - p.nt_log2)) + (sbr << (p.grid_log2 - 3 - scl)) + (slot >> scl);
            cb = (sbc << scl) + (slot & ((1 << scl) - 1));
        } else {
            const int t = round * (int)gridDim.x + (int)blockIdx.x;
            rb = t / p.NT;
            cb = t - rb * p.NT;
        }
        if (rb >= p.RB)
            continue;  // uniform for the workgroup
        // Everything derived from the lane index and from the shape is computed here, per tile, where
        // it is used.
        const int lane = opaque_lane();
        const int M = opaque_uniform(p.M), N = opaque_uniform(p.N), K = opaque_uniform(p.K);
        const int slabs = (K + kSlabElems - 1) / kSlabElems;
        const bool k_ragged = (K % kSlabElems) != 0;
        const size_t row_stride = (size_t)K * sizeof(T);
        stamper = wave == 0 && lane == 0;
        stamp(0);
        const int m0 = rb * BM;
        const int n0 = cb * BN;
        const int h = lane >> 5;
        const int l32 = lane & 31;
        // fragment read offsets (bytes inside a stage); k-step s reads chunk (2s + h) ^ swizzle
        const int frag_swz = swizzle_of_row(l32);
        const int a_frag_base = (wn * WTN * 32 + l32) * kRowBytes;
        const int b_frag_base = kXBase + (wm * WTM * 32 + l32) * kRowBytes;
        // DMA lane geometry: lane -> (row within a 16-row group, stored chunk slot)
        const int dma_r = lane / kChunksPerRow;
        const int dma_cs = lane % kChunksPerRow;

        // ---- per-lane byte offsets of the DMA sources, relative to the tile's first row ----
        const char *w_tile = (const char *)p.W + (size_t)n0 * row_stride;
        const char *x_tile = (const char *)p.X + (size_t)m0 * row_stride;
        unsigned offa[kDmaA], offb[kDmaB];
#pragma unroll
        for (int j = 0; j < kDmaA; ++j) {
            const int row = wave * (BN / kWaves) + j * kRowsPerDma + dma_r;
            const int c = dma_cs ^ swizzle_of_row(row);
            const int rr = (n0 + row < N) ? row : (N - 1 - n0);  // clamp to the last valid row
            offa[j] = (unsigned)rr * (unsigned)row_stride + c * 16;
        }
#pragma unroll
        for (int j = 0; j < kDmaB; ++j) {
            const int row = wave * (BM / kWaves) + j * kRowsPerDma + dma_r;
            const int c = dma_cs ^ swizzle_of_row(row);
            const int rr = (m0 + row < M) ? row : (M - 1 - m0);
            offb[j] = (unsigned)rr * (unsigned)row_stride + c * 16;
        }

        // full slab: direct-to-LDS, nothing passes through registers.  dma_one issues
        // the x-th of the wave's kDmaPerSlab instructions (W rows first, then X rows).
        // Buffer descriptors over the tile's rows: the per-lane 32-bit byte offset is
        // the loop-invariant part of a load's address, the slab offset rides in a scalar
        // register, so a DMA instruction costs no vector ALU work.  All addresses are
        // clamped in-bounds above; the descriptors do not rely on range checking.
        const __amdgpu_buffer_rsrc_t w_rsrc =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(w_tile), 0, 0xffffffffu, 0x00020000);
        const __amdgpu_buffer_rsrc_t x_rsrc =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(x_tile), 0, 0xffffffffu, 0x00020000);
        auto dma_one = [&](int slab, int x) {
            const int stage = slab % kStages;
            if (x < kDmaA) {
                char *sa = smem + stage * kWStride + wave * (BN / kWaves) * kRowBytes;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    w_rsrc, (__attribute__((address_space(3))) void *)(sa + x * 1024), 16,
                    offa[x < kDmaA ? x : 0], slab * kRowBytes, 0, 0);
            } else {
                const int y = x - kDmaA;
                char *sb = smem + kXBase + stage * kXStride + wave * (BM / kWaves) * kRowBytes;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    x_rsrc, (__attribute__((address_space(3))) void *)(sb + y * 1024), 16,
                    offb[y >= 0 && y < kDmaB ? y : 0], slab * kRowBytes, 0, 0);
            }
        };
        // K-cut (last) slab: through registers, chunks at or beyond K are zero-filled
        auto issue_cut = [&](int slab, int half) {
            // lane geometry re-derived through an opaque move: this rarely taken path
            // must not have its masks precomputed (and spilled) at kernel entry
            const int lane_c = opaque_lane();
            const int dma_r = lane_c / kChunksPerRow;
            const int dma_cs = lane_c % kChunksPerRow;
            const int stage = slab % kStages;
            if (half == 0) {
                char *sa = smem + stage * kWStride + wave * (BN / kWaves) * kRowBytes;
                const char *wk = w_tile + (size_t)slab * kRowBytes;
#pragma unroll
                for (int j = 0; j < kDmaA; ++j) {
                    const int row = wave * (BN / kWaves) + j * kRowsPerDma + dma_r;
                    const int c = dma_cs ^ swizzle_of_row(row);
                    const bool in = slab * kSlabElems + c * kChunkElems < K;
                    uintx4 v = *reinterpret_cast<const uintx4 *>(in ? wk + offa[j] : w_tile);
                    v &= in ? 0xffffffffu : 0u;
                    *reinterpret_cast<uintx4 *>(sa + j * 1024 + lane_c * 16) = v;
                }
            } else {
                char *sb = smem + kXBase + stage * kXStride + wave * (BM / kWaves) * kRowBytes;
                const char *xk = x_tile + (size_t)slab * kRowBytes;
#pragma unroll
                for (int j = 0; j < kDmaB; ++j) {
                    const int row = wave * (BM / kWaves) + j * kRowsPerDma + dma_r;
                    const int c = dma_cs ^ swizzle_of_row(row);
                    const bool in = slab * kSlabElems + c * kChunkElems < K;
                    uintx4 v = *reinterpret_cast<const uintx4 *>(in ? xk + offb[j] : x_tile);
                    v &= in ? 0xffffffffu : 0u;
                    *reinterpret_cast<uintx4 *>(sb + j * 1024 + lane_c * 16) = v;
                }
            }
        };

        // The accumulators start from a zero the optimiser cannot see through: given a constant it
        // parks a block of sixteen zeros in scratch memory for the path that skips the steady iterations.
        float zero;
        asm volatile("v_mov_b32 %0, 0" : "=v"(zero));
        floatx16 acc[WTN][WTM];
#pragma unroll
        for (int i = 0; i < WTN; ++i)
#pragma unroll
            for (int j = 0; j < WTM; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    acc[i][j][r] = zero;

        uintx4 fa[2][WTN], fb[2][WTM];  // fragment registers, double-buffered by k-step
        // x-th fragment read of (slab, k-step s): W fragments first, then X fragments
        auto read_one = [&](int slab, int s, int x, uintx4 (&a)[WTN], uintx4 (&b)[WTM]) {
            const int coff = ((2 * s + h) ^ frag_swz) << 4;
            if (x < WTN)
                a[x < WTN ? x : 0] = *reinterpret_cast<const uintx4 *>(
                    smem + (slab % kStages) * kWStride + a_frag_base + x * 32 * kRowBytes + coff);
            else
                b[x >= WTN ? x - WTN : 0] = *reinterpret_cast<const uintx4 *>(
                    smem + (slab % kStages) * kXStride + b_frag_base + (x - WTN) * 32 * kRowBytes + coff);
        };
        auto load_frags = [&](int slab, int s, uintx4 (&a)[WTN], uintx4 (&b)[WTM]) {
#pragma unroll
            for (int x = 0; x < WTN + WTM; ++x)
                read_one(slab, s, x, a, b);
        };
        // the MFMAs of a k-step are issued in kGroups groups (one per fragment read); group g takes the
        // fragment pairs [g * kPairs / kGroups, (g + 1) * kPairs / kGroups): two each for 4 x 4 blocks per
        // wave, one each for 2 x 2, and for a single block the second group takes the only pair
        constexpr int kGroups = WTN + WTM;
        constexpr int kPairs = WTN * WTM;
        static_assert(kPairs <= 2 * kGroups, "pin_order takes at most two accumulators");
        auto mma_group = [&](int g, const uintx4 (&a)[WTN], const uintx4 (&b)[WTM]) {
#pragma unroll
            for (int pair = g * kPairs / kGroups; pair < (g + 1) * kPairs / kGroups; ++pair)
                Mma<T>::step(a[pair / WTM], b[pair % WTM], acc[pair / WTM][pair % WTM]);
        };
        auto pin_group = [&](int g) {
            const int p0 = g * kPairs / kGroups;
            const int n = (g + 1) * kPairs / kGroups - p0;
            if (n == 2)
                pin_order(acc[p0 / WTM][p0 % WTM], acc[(p0 + 1) / WTM][(p0 + 1) % WTM]);
            else if (n == 1)
                pin_order(acc[p0 / WTM][p0 % WTM]);
        };
        auto mma_all = [&](const uintx4 (&a)[WTN], const uintx4 (&b)[WTM]) {
#pragma unroll
            for (int g = 0; g < kGroups; ++g)
                mma_group(g, a, b);
        };

        // ---- main loop over K slabs ----
        // Per slab: four k-steps, each one group-interleaved stream of MFMAs with one
        // LDS fragment read (for the next k-step) and at most one DMA instruction in
        // the shadow of each MFMA group.  The W half of slab i+1 is issued during
        // k-step 3 of slab i-1... concretely, iteration i issues the X half of slab
        // i+1 in k-step 0 and the W half of slab i+2 in k-step 3; the barrier before
        // k-step 3 is the point where slab i+1 has landed for everyone and everyone
        // has finished reading slab i (its stage is then refilled).
        static_assert(kStepsPerSlab == 4 && kStages == 2, "loop body written for 4 k-steps, 2 stages");
        static_assert(kXReg || (kDmaA <= kGroups && kDmaB <= kGroups), "one DMA instruction per MFMA group at most");
        auto dma_half_any = [&](int slab, int half) {
            // half 0: W rows (x in [0, kDmaA)), half 1: X rows; K-cut slabs go through registers
            if (!k_ragged || slab + 1 < slabs) {
#pragma unroll
                for (int x = 0; x < (half == 0 ? kDmaA : kDmaB); ++x)
                    dma_one(slab, half == 0 ? x : kDmaA + x);
            } else {
                issue_cut(slab, half);
            }
        };
        if constexpr (kXReg) {
        // ---- main loop, X slabs through registers ----
        // Iteration i: the X slab i+1 is requested at the start (global -> registers); after the
        // first three k-steps barrier A says everyone has read slab i from the LDS; then the X
        // registers go to the single X buffer, the W slab i+2 is requested into the stage slab i
        // occupied, half of the last k-step's MFMAs cover the LDS writes, barrier B publishes the X
        // slab (every wave has waited for its own share of W slab i+1 before it), and the rest of the
        // last k-step covers the first fragment reads of slab i+1.  The other workgroup on the compute
        // unit fills the matrix pipe while this one stands at its barriers.
        uintx4 xr[kDmaB];
        auto x_load_full = [&](int slab) {
#pragma unroll
            for (int j = 0; j < kDmaB; ++j)
                xr[j] = __builtin_bit_cast(uintx4, __builtin_amdgcn_raw_buffer_load_b128(
                                                       x_rsrc, offb[j], slab * kRowBytes, 0));
        };
        auto x_load = [&](int slab) {
            if (!k_ragged || slab + 1 < slabs) {
                x_load_full(slab);
            } else {
                const int lane_c = opaque_lane();  // as in issue_cut
#pragma unroll
                for (int j = 0; j < kDmaB; ++j) {
                    const int row = wave * (BM / kWaves) + j * kRowsPerDma + lane_c / kChunksPerRow;
                    const int c = (lane_c % kChunksPerRow) ^ swizzle_of_row(row);
                    const bool in = slab * kSlabElems + c * kChunkElems < K;
                    uintx4 v = __builtin_bit_cast(uintx4, __builtin_amdgcn_raw_buffer_load_b128(
                                                              x_rsrc, in ? offb[j] : 0u, in ? slab * kRowBytes : 0, 0));
                    v &= in ? 0xffffffffu : 0u;
                    xr[j] = v;
                }
            }
        };
        auto x_store = [&]() {
            char *sb = smem + kXBase + wave * (BM / kWaves) * kRowBytes + lane * 16;
#pragma unroll
            for (int j = 0; j < kDmaB; ++j)
                *reinterpret_cast<uintx4 *>(sb + j * 1024) = xr[j];
        };
        lds_barrier();  // the previous tile's epilogue is done with the LDS
        dma_half_any(0, 0);
        x_load(0);
        if (slabs > 1)
            dma_half_any(1, 0);
        __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0)
        x_store();
        lds_barrier();
        stamp(1);
        stamp(kTimelineCycleSlot);
        load_frags(0, 0, fa[0], fb[0]);
        // steady iterations: slab i+1 and slab i+2 exist and are full ones
        const int n_steady = slabs - 2 - (k_ragged ? 1 : 0);
        int i = 0;
        for (; i < n_steady; ++i) {
            x_load_full(i + 1);
#pragma unroll
            for (int g = 0; g < kGroups; ++g) {  // k-step 0
                read_one(i, 1, g, fa[1], fb[1]);
                mma_group(g, fa[0], fb[0]);
                pin_group(g);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int g = 0; g < kGroups; ++g) {  // k-step 1
                mma_group(g, fa[1], fb[1]);
                read_one(i, 2, g, fa[0], fb[0]);
                pin_group(g);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int g = 0; g < kGroups; ++g) {  // k-step 2
                mma_group(g, fa[0], fb[0]);
                read_one(i, 3, g, fa[1], fb[1]);
                pin_group(g);
                __builtin_amdgcn_sched_barrier(0);
            }
            lds_barrier();                       // A: everyone has read slab i
            __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): X registers and this wave's W rows of slab i+1
            x_store();
#pragma unroll
            for (int x = 0; x < kDmaA; ++x)
                dma_one(i + 2, x);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int g = 0; g < kGroups / 2; ++g) {  // k-step 3, first half
                mma_group(g, fa[1], fb[1]);
                pin_group(g);
            }
            __builtin_amdgcn_sched_barrier(0);
            lds_barrier();                       // B: slab i+1 is complete in the LDS
            load_frags(i + 1, 0, fa[0], fb[0]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int g = kGroups / 2; g < kGroups; ++g) {  // k-step 3, second half
                mma_group(g, fa[1], fb[1]);
                pin_group(g);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // last iterations: slab i+1 or i+2 is missing or cut by K
        for (; i < slabs; ++i) {
            const bool more = i + 1 < slabs;
            if (more)
                x_load(i + 1);
            load_frags(i, 1, fa[1], fb[1]);
            mma_all(fa[0], fb[0]);
            load_frags(i, 2, fa[0], fb[0]);
            mma_all(fa[1], fb[1]);
            load_frags(i, 3, fa[1], fb[1]);
            mma_all(fa[0], fb[0]);
            if (more) {
                lds_barrier();                       // A
                __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0)
                x_store();
                if (i + 2 < slabs)
                    dma_half_any(i + 2, 0);
                __builtin_amdgcn_s_waitcnt(0x0f70);  // a K-cut W slab went through registers
                lds_barrier();                       // B
                load_frags(i + 1, 0, fa[0], fb[0]);
            }
            mma_all(fa[1], fb[1]);
        }
        } else {
        // The previous tile's epilogue is done with the LDS once every wave is here (its LDS reads
        // completed before its stores could issue).  No wait for those stores: they drain while the
        // first slab of this tile travels.
        // The parameter loads are the oldest loads in flight: every wait for a slab below covers them.
        // Entry c of [bias | gamma | beta] goes to thread c % kThreads; loads never branch (what has
        // no source reads the first element of W and is replaced by the default).
        float prm[kPrmPerThread];
#pragma unroll
        for (int u = 0; u < kPrmPerThread; ++u) {
            const int c = wave * 64 + lane + u * kThreads;
            const int which = c / BN;
            const int n = n0 + (c & (BN - 1));
            const T *src = reinterpret_cast<const T *>(which == 0 ? p.b : (which == 1 ? p.gamma : p.beta));
            const bool ok = which < 3 && n < N && src != nullptr;
            const float v = load_as_float(ok ? src + n : reinterpret_cast<const T *>(p.W));
            prm[u] = ok ? v : (which == 1 ? 1.0f : 0.0f);
        }
        lds_barrier();
        dma_half_any(0, 0);
        dma_half_any(0, 1);
        if (slabs > 1)
            dma_half_any(1, 0);
        if (first_tile && p.timeline == nullptr && slabs > 1 && !(k_ragged && slabs == 2))
            __builtin_amdgcn_s_waitcnt(0x0f70 | (kDmaA & 15) | ((kDmaA >> 4) << 14));  // slab 0 landed
        else
            __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): also the previous tile's stores, whose
                                                 // completion order relative to loads is not relied on
        first_tile = false;
        // the previous tile's last readers of the parameter region passed the barrier above
#pragma unroll
        for (int u = 0; u < kPrmPerThread; ++u) {
            const int c = wave * 64 + lane + u * kThreads;
            if (c < 3 * BN)
                s_prm_early[c] = prm[u];
        }
        lds_barrier();
        stamp(1);
        stamp(kTimelineCycleSlot);
        load_frags(0, 0, fa[0], fb[0]);

        // steady iterations: slab i+1 and slab i+2 exist and are full ones
        const int n_steady = slabs - 2 - (k_ragged ? 1 : 0);
        int i = 0;
        for (; i < n_steady; ++i) {
#pragma unroll
            for (int g = 0; g < kGroups; ++g) {  // k-step 0
                if (g < kDmaB)
                    dma_one(i + 1, kDmaA + g);
                read_one(i, 1, g, fa[1], fb[1]);
                mma_group(g, fa[0], fb[0]);
                pin_group(g);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int g = 0; g < kGroups; ++g) {  // k-step 1
                mma_group(g, fa[1], fb[1]);
                read_one(i, 2, g, fa[0], fb[0]);
                pin_group(g);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int g = 0; g < kGroups; ++g) {  // k-step 2
                mma_group(g, fa[0], fb[0]);
                read_one(i, 3, g, fa[1], fb[1]);
                pin_group(g);
                __builtin_amdgcn_sched_barrier(0);
            }
            __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): slab i+1 has landed
            lds_barrier();
#pragma unroll
            for (int g = 0; g < kGroups; ++g) {  // k-step 3
                if (g < kDmaA)
                    dma_one(i + 2, g);
                mma_group(g, fa[1], fb[1]);
                read_one(i + 1, 0, g, fa[0], fb[0]);
                pin_group(g);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // last iterations: slab i+1 or i+2 is missing or cut by K
        for (; i < slabs; ++i) {
            if (i + 1 < slabs)
                dma_half_any(i + 1, 1);
            load_frags(i, 1, fa[1], fb[1]);
            mma_all(fa[0], fb[0]);
            load_frags(i, 2, fa[0], fb[0]);
            mma_all(fa[1], fb[1]);
            load_frags(i, 3, fa[1], fb[1]);
            mma_all(fa[0], fb[0]);
            __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0)
            lds_barrier();
            if (i + 2 < slabs)
                dma_half_any(i + 2, 0);
            if (i + 1 < slabs)
                load_frags(i + 1, 0, fa[0], fb[0]);
            mma_all(fa[1], fb[1]);
        }
        }  // kPipeDma
        __syncthreads();  // all fragment reads done: LDS becomes epilogue scratch
        stamp(2);
        stamp(kTimelineCycleSlot + 1);

        // ---- epilogue ----
        // The lane index and the row length are taken afresh so that the epilogue's many
        // lane-dependent addresses and its float constants are computed here, once per tile,
        // instead of being hoisted out of the tile loop and carried (spilled) across the main loop.
        {
        const int lane = opaque_lane();
        const int M = opaque_uniform(p.M), N = opaque_uniform(p.N);
        const int h = lane >> 5;
        const int l32 = lane & 31;
        float *s_b = kPrmEarly ? s_prm_early : reinterpret_cast<float *>(smem + kOffPrm);
        float *s_g = s_b + BN;
        float *s_be = s_g + BN;
        floatx2 *s_wst = reinterpret_cast<floatx2 *>(smem + kOffWst);
        floatx2 *s_rst = reinterpret_cast<floatx2 *>(smem + kOffRst);
        char *s_out = smem + kOffOut + wave * 32 * kOutPitch;

        if (!kPrmEarly) {
            for (int c = wave * 64 + lane; c < BN; c += kThreads) {
                const int n = n0 + c;
                const bool ok = n < N;
                s_b[c] = (ok && p.b) ? load_as_float(reinterpret_cast<const T *>(p.b) + n) : 0.0f;
                s_g[c] = (ok && p.gamma) ? load_as_float(reinterpret_cast<const T *>(p.gamma) + n) : 1.0f;
                s_be[c] = (ok && p.beta) ? load_as_float(reinterpret_cast<const T *>(p.beta) + n) : 0.0f;
            }
            __syncthreads();
        }

        const int ncol_wave = wn * WTN * 32;            // wave's first column inside the tile
        const int nvalid_tile = (N - n0 < BN) ? (N - n0) : BN;

        // bias + GELU in place in the accumulators, and per-row (count, mean, M2) of
        // the tile.  A lane holds 16 WTN values of each of its WTM rows; their sums are
        // taken about the lane's first value (a shift that keeps sum-of-squares
        // cancellation harmless), merged with the other lane half, then across waves.
        {
            constexpr bool kRagged = RAGGED_N;
            int cnt_own = WTN * 16, cnt_other = WTN * 16;
            if (kRagged) {
                cnt_own = cnt_other = 0;
#pragma unroll
                for (int i = 0; i < WTN; ++i)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const int c0 = ncol_wave + i * 32 + q * 8 + e;
                            cnt_own += (c0 + h * 4 < nvalid_tile) ? 1 : 0;
                            cnt_other += (c0 + (h ^ 1) * 4 < nvalid_tile) ? 1 : 0;
                        }
            }
            int cntw_i = nvalid_tile - ncol_wave;
            cntw_i = cntw_i < 0 ? 0 : (cntw_i > WTN * 32 ? WTN * 32 : cntw_i);
            float shift[WTM], s1[WTM], s2[WTM];
#pragma unroll
            for (int j = 0; j < WTM; ++j)
                shift[j] = s1[j] = s2[j] = 0.0f;
#pragma unroll
            for (int i = 0; i < WTN; ++i) {
                floatx4 bb[4];  // bias of this lane's 16 columns of block row i
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    bb[q] = *reinterpret_cast<const floatx4 *>(s_b + ncol_wave + i * 32 + q * 8 + h * 4);
#pragma unroll
                for (int j = 0; j < WTM; ++j) {
                    // one 32x32 block at a time: read its 16 registers, write back 16 G values
                    floatx16 v = acc[i][j];
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float z = v[r] + bb[r >> 2][r & 3];
                        if (MODE == kLinearOnly) {
                            v[r] = z;
                            continue;
                        }
                        float g = gelu_erf(z);
                        if (i == 0 && r == 0)
                            shift[j] = g;  // column ncol_wave + 4h: valid whenever the lane has any
                        float d = g - shift[j];
                        if (kRagged && ncol_wave + i * 32 + (r >> 2) * 8 + h * 4 + (r & 3) >= nvalid_tile) {
                            g = 0.0f;
                            d = 0.0f;
                        }
                        v[r] = g;
                        s1[j] += d;
                        s2[j] = fmaf(d, d, s2[j]);
                    }
                    acc[i][j] = v;
                    pin_order(acc[i][j]);  // G goes back to the accumulator registers
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if (MODE != kLinearOnly) {
                // (the lane index is taken afresh after the pass over the accumulators and again
                // before the stores: values derived from it are not carried across those passes)
                const int lane = opaque_lane();
                const int h = lane >> 5;
                const int l32 = lane & 31;
#pragma unroll
                for (int j = 0; j < WTM; ++j) {
                    // lane statistics -> merged with the other half-wave (lower half first)
                    const float n_own = (float)cnt_own, n_oth = (float)cnt_other;
                    const float inv_own = cnt_own > 0 ? 1.0f / n_own : 0.0f;
                    float mean_own = fmaf(s1[j], inv_own, shift[j]);
                    float m2_own = fmaxf(s2[j] - s1[j] * s1[j] * inv_own, 0.0f);
                    if (kRagged && cnt_own == 0)
                        mean_own = 0.0f;
                    const float mean_oth = swap_halves(mean_own, lane);
                    const float m2_oth = swap_halves(m2_own, lane);
                    float na = h == 0 ? n_own : n_oth;
                    float mean_a = h == 0 ? mean_own : mean_oth;
                    float m2a = h == 0 ? m2_own : m2_oth;
                    merge_stats(na, mean_a, m2a, h == 0 ? n_oth : n_own,
                                h == 0 ? mean_oth : mean_own, h == 0 ? m2_oth : m2_own);
                    if (h == 0) {
                        floatx2 v = {mean_a, m2a};
                        s_wst[wn * BM + wm * WTM * 32 + j * 32 + l32] = v;
                    }
                }
            }
            (void)cntw_i;
        }

        const int tid = wave * 64 + opaque_lane();  // taken afresh: not carried across the pass above
        if (MODE != kLinearOnly) {
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

        stamp(3);
        if (MODE == kFused) {
            // exchange with the other tiles of these rows
            wait_published();
            __syncthreads();
            if (tid == 0) {
                unsigned *arrive = p.counters + 2 * (size_t)rb;
                atomic_add_device(arrive, 1u);
                if (!wait_counter(arrive, (unsigned)(p.NT + p.extra_arrivals), p.wait_ticks))
                    atomic_store_device(p.err, 1u);
            }
            __syncthreads();
            stamp(4);
            // Plain loads: each line was written through by its single owner before the counter
            // could reach its target, and no cache of this XCD can hold an older copy within this
            // launch.  Loads are issued 16 at a time, the merge runs in tile order.  Where the
            // workgroup has two threads per row and a row more than 16 tiles, each thread takes
            // half of the row's tiles (the load latency, not the arithmetic, is what the merge
            // costs) and the halves meet in LDS.
            constexpr int kParts = (64 * kWaves >= 2 * BM) ? 2 : 1;
            const bool split = kParts == 2 && p.NT > 16;
            const int row = tid & (BM - 1);
            const int per = split ? (p.NT + 1) / 2 : p.NT;
            float na = 0.0f, mean_a = 0.0f, m2a = 0.0f;
            if (tid < BM || (split && tid < kParts * BM)) {
                // Buffer loads: a row block's partials as the resource, the tile as the scalar
                // offset and the row as the one vector offset, so that no load needs a 64-bit
                // address of its own in vector registers.
                const int part = wave / (BM / 64);  // uniform in a wavefront
                const __amdgpu_buffer_rsrc_t st_rsrc = __builtin_amdgcn_make_buffer_rsrc(
                    reinterpret_cast<char *>(p.partials + (size_t)rb * p.NT * BM), 0,
                    (unsigned)(p.NT * BM * (int)sizeof(floatx2)), 0x00020000);
                const unsigned row_off = (unsigned)row * (unsigned)sizeof(floatx2);
                const int c_begin = part * per < p.NT ? part * per : p.NT;
                const int c_end = c_begin + per < p.NT ? c_begin + per : p.NT;
                for (int c0 = c_begin; c0 < c_end; c0 += 16) {
                    floatx2 u[16];
#pragma unroll
                    for (int j = 0; j < 16; ++j) {
                        const int c = c0 + j < c_end ? c0 + j : c_end - 1;  // unconditional loads
                        if (kParts == 2)
                            u[j] = __builtin_bit_cast(floatx2, __builtin_amdgcn_raw_buffer_load_b64(
                                                           st_rsrc, row_off, c * BM * (int)sizeof(floatx2), 0));
                        else  // one thread per row: plain addressing takes fewer registers there
                            u[j] = p.partials[((size_t)rb * p.NT + c) * BM + row];
                    }
#pragma unroll
                    for (int j = 0; j < 16; ++j)
                        if (c0 + j < c_end) {
                            const int c = c0 + j;
                            const int cnt = (N - c * BN < BN) ? (N - c * BN) : BN;
                            merge_stats(na, mean_a, m2a, (float)cnt, u[j][0], u[j][1]);
                        }
                }
                if (split && part == 1) {  // s_wst is free: its last readers passed the barriers above
                    floatx2 o = {mean_a, m2a};
                    s_wst[row] = o;
                }
            }
            if (split)
                __syncthreads();
            if (tid < BM) {
                if (split) {
                    const int rest = N - per * BN;  // columns of the second half's tiles
                    const floatx2 u = s_wst[row];
                    merge_stats(na, mean_a, m2a, rest > 0 ? (float)rest : 0.0f, u[0], u[1]);
                }
                const float var = m2a / (float)N;
                floatx2 o = {mean_a, 1.0f / sqrtf(var + p.eps)};
                s_rst[tid] = o;
            }
            __syncthreads();
        }

        stamp(5);
        // ---- (normalise,) convert, transpose through LDS, store 16-byte rows ----
        OutT *out_base = (MODE == kFused) ? reinterpret_cast<OutT *>(p.Y)
                                          : reinterpret_cast<OutT *>(p.F);
        const int lane_o = opaque_lane();
        {
        const int lane = lane_o;
        const int h = lane >> 5;
        const int l32 = lane & 31;
#pragma unroll
        for (int j = 0; j < WTM; ++j) {
            float rstd = 1.0f, shift = 0.0f;  // y = (g * rstd + shift) * gamma + beta
            if (MODE == kFused) {
                const floatx2 ms = s_rst[wm * WTM * 32 + j * 32 + l32];
                rstd = ms[1];
                shift = -ms[0] * ms[1];
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
                            y[e] = fmaf(fmaf(acc[i][j][q * 4 + e], rstd, shift), ga4[e], be4[e]);
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
                if (gm < M && gn < N)  // streaming store: Y is not read again by this launch
                    __builtin_nontemporal_store(v, reinterpret_cast<uintx4 *>(out_base + (size_t)gm * N + gn));
            }
            wave_lds_sync();
        }
        }
        if (MODE == kFused && tid == 0) {
            // Departure, after the stores have been issued so that the wait for the counter's old value
            // delays nothing: the last tile of the row-block to get here re-arms its counters (every
            // tile of the row-block has read the partials by then).
            unsigned *cnt = p.counters + 2 * (size_t)rb;
            if (atomic_add_device(cnt + 1, 1u) == (unsigned)p.NT - 1u) {
                atomic_store_device(cnt, 0u);
                atomic_store_device(cnt + 1, 0u);
            }
        }
        stamp(6);
        }  // epilogue scope
    }
#else
    (void)p;
#endif
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

template <typename T, int WN, int WM, int WTN, int WTM, int MODE, int PIPE>
hipError_t launch_tile(const TileParams &p, int grid, hipStream_t stream)
{
    constexpr int BN = WN * WTN * 32;
    constexpr int kThreads = 64 * WN * WM;
    if (p.N % BN != 0)
        hipLaunchKernelGGL((tile_kernel<T, WN, WM, WTN, WTM, MODE, true, PIPE>), dim3(grid), dim3(kThreads), 0,
                           stream, p);
    else
        hipLaunchKernelGGL((tile_kernel<T, WN, WM, WTN, WTM, MODE, false, PIPE>), dim3(grid), dim3(kThreads), 0,
                           stream, p);
    return hipGetLastError();
}

template <typename T, int WN, int WM, int WTN, int WTM, int MODE, int PIPE>
int max_blocks_per_cu()
{
    int a = 0, b = 0;
    constexpr int kThreads = 64 * WN * WM;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&a, tile_kernel<T, WN, WM, WTN, WTM, MODE, true, PIPE>,
                                                     kThreads, 0) != hipSuccess ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&b, tile_kernel<T, WN, WM, WTN, WTM, MODE, false, PIPE>,
                                                     kThreads, 0) != hipSuccess) {
        (void)hipGetLastError();
        return 0;
    }
    return a < b ? a : b;
}

}  // namespace

// Dispatch over (dtype, tile shape, mode): wave layout, blocks per wave and slab pipeline per shape.
#define FF_TILE_DISPATCH(CALL)                                                             \
    if (bf16) {                                                                            \
        switch (shape) {                                                                   \
        case kTile256x128: FF_MODES(__bf16, 2, 2, 4, 2, kPipeXReg, CALL)                   \
        case kTile256W8: FF_MODES(__bf16, 2, 4, 4, 2, kPipeDma, CALL)                      \
        case kTile256: FF_MODES(__bf16, 2, 2, 4, 4, kPipeDma, CALL)                        \
        case kTile128: FF_MODES(__bf16, 2, 2, 2, 2, kPipeDma, CALL)                        \
        default: FF_MODES(__bf16, 2, 2, 1, 1, kPipeDma, CALL)                              \
        }                                                                                  \
    }                                                                                      \
    switch (shape) {                                                                       \
    case kTile256x128: FF_MODES(float, 2, 2, 4, 2, kPipeXReg, CALL)                        \
    case kTile256W8: FF_MODES(float, 2, 4, 4, 2, kPipeDma, CALL)                           \
    case kTile256: FF_MODES(float, 2, 2, 4, 4, kPipeDma, CALL)                             \
    case kTile128: FF_MODES(float, 2, 2, 2, 2, kPipeDma, CALL)                             \
    default: FF_MODES(float, 2, 2, 1, 1, kPipeDma, CALL)                                   \
    }
#define FF_MODES(T, WN, WM, WTN, WTM, PIPE, CALL)                     \
    switch (mode) {                                                   \
    case kFused: return CALL(T, WN, WM, WTN, WTM, kFused, PIPE);      \
    case kTwoPass: return CALL(T, WN, WM, WTN, WTM, kTwoPass, PIPE);  \
    default: return CALL(T, WN, WM, WTN, WTM, kLinearOnly, PIPE);     \
    }

hipError_t launch_tile_kernel(bool bf16, int shape, int mode, const TileParams &p, int grid, hipStream_t stream)
{
#define FF_CALL(T, WN, WM, WTN, WTM, MODE, PIPE) launch_tile<T, WN, WM, WTN, WTM, MODE, PIPE>(p, grid, stream)
    FF_TILE_DISPATCH(FF_CALL)
#undef FF_CALL
}

// Workgroups of this kernel that fit one compute unit at once (registers, LDS), as the runtime
// reports it; 0 if the query fails.  A launch whose workgroups wait for one another inside the
// launch must not be larger than this many per compute unit.
int tile_kernel_blocks_per_cu(bool bf16, int shape, int mode)
{
#define FF_CALL(T, WN, WM, WTN, WTM, MODE, PIPE) max_blocks_per_cu<T, WN, WM, WTN, WTM, MODE, PIPE>()
    FF_TILE_DISPATCH(FF_CALL)
#undef FF_CALL
}
#undef FF_MODES
#undef FF_TILE_DISPATCH

hipError_t launch_finalize_kernel(bool bf16, const FinalizeParams &p, hipStream_t stream)
{
    if (bf16)
        hipLaunchKernelGGL(finalize_kernel<__bf16>, dim3(p.M), dim3(256), 0, stream, p);
    else
        hipLaunchKernelGGL(finalize_kernel<float>, dim3(p.M), dim3(256), 0, stream, p);
    return hipGetLastError();
}

}  // namespace ff
