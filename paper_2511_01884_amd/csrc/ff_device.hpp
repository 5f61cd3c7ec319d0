// Device-side building blocks shared by the gfx950 kernels: bf16 <-> fp32,
// erf-form GELU, pairwise merge of (count, mean, M2) row statistics, and the
// workspace layout the kernels and the host agree on.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ff {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));

// ---- workspace layout (bytes from the workspace base) ----------------------
// [0, 4)                error word: non-zero once a wait inside a launch gave up
// [256, CTRL_BYTES)     arrival / departure counters, two uint32 per row-block; zero between launches
// [CTRL_BYTES, ...)     per-tile row statistics (float2 mean, M2), then the
//                       two-pass variant's fp32 G; other entry points' scratch
constexpr size_t kCtrlBytes = 1u << 20;
constexpr size_t kCounterOffset = 256;
constexpr int64_t kMaxRowBlocks = (int64_t)((kCtrlBytes - kCounterOffset) / 8);

// Workgroup barrier that carries no fence: unlike __syncthreads() it does not wait for outstanding
// global loads, so loads requested ahead (registers or direct-to-LDS) stay in flight across it;
// their completion is awaited explicitly with vmcnt where it matters.  It waits for this wave's own
// LDS reads and writes, and the barrier instruction itself is a compiler-level ordering point for
// memory operations.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0) only
    __builtin_amdgcn_s_barrier();
}

// ---- bf16 <-> fp32 -----------------------------------------------------------
__device__ __forceinline__ float bf16_bits_to_float(unsigned short h)
{
    return __uint_as_float(((unsigned)h) << 16);
}
__device__ __forceinline__ float load_as_float(const float *p) { return *p; }
__device__ __forceinline__ float load_as_float(const __bf16 *p)
{
    return bf16_bits_to_float(*reinterpret_cast<const unsigned short *>(p));
}
// Round-to-nearest-even pack of two floats (hardware conversion on gfx950).
__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi)
{
    floatx2 v = {lo, hi};
    bf16x2 h = __builtin_convertvector(v, bf16x2);
    return *reinterpret_cast<unsigned *>(&h);
}

// ---- GELU, erf form -----------------------------------------------------------
// g = z * Phi(z), Phi the standard normal distribution function, Phi(z) = 0.5 * erfc(-z / sqrt 2).
// With q = Phi(-|z|) evaluated directly (no 1 + erf cancellation), g = max(z, 0) - |z| q for either
// sign of z.  q is smooth, positive and falls like exp(-z^2 / 2), so its base-2 logarithm is close to
// a low-degree polynomial: q ~ 2^P(|z|), P of degree 5, fitted (fit_gelu_tail.py beside this file) so
// that the error of |z| q, which is the error of g, is below 4.7e-7 for every z; P has a negative
// leading coefficient and no real stationary point, so 2^P decays to 0 for large |z|.  One hardware
// 2^x (1 ulp) and five multiply-adds: the epilogue's cost per element is what matters here, the
// matrix pipe is idle while it runs.
__device__ __forceinline__ float gelu_erf(float z)
{
    const float x = fabsf(z);
    float p = -0.000473293995f;
    p = fmaf(p, x, 0.00708446082f);
    p = fmaf(p, x, -0.051827167f);
    p = fmaf(p, x, -0.459992648f);
    p = fmaf(p, x, -1.15078777f);
    p = fmaf(p, x, -1.00003763f);
    const float q = __builtin_amdgcn_exp2f(p);
    return fmaf(-x, q, fmaxf(z, 0.0f));
}

// ---- (count, mean, M2) merge (Chan et al. pairwise update) ---------------------
// Folds block b into block a:  delta = mean_b - mean_a; n = n_a + n_b;
// mean = mean_a + delta * n_b / n;  M2 = M2_a + M2_b + delta^2 * n_a * n_b / n.
__device__ __forceinline__ void merge_stats(float &na, float &mean_a, float &m2a,
                                            float nb, float mean_b, float m2b)
{
    const float n = na + nb;
    if (n > 0.0f) {
        const float inv = 1.0f / n;
        const float delta = mean_b - mean_a;
        mean_a = fmaf(delta, nb * inv, mean_a);
        m2a = m2a + m2b + delta * delta * (na * nb * inv);
    }
    na = n;
}

// Cross-workgroup exchange of row statistics.  Workgroups of one launch run on
// different XCDs with separate L2 caches, so the 8-byte (mean, M2) partials are
// written and read with device-scope atomic accesses: the store writes through to
// the level all XCDs share, the load never takes a stale line of the local L2.
// A full fence (L2 write-back plus invalidate) would also be correct but costs
// tens of microseconds per launch.  Ordering: every publishing thread waits for
// its own stores to complete (vmcnt), the workgroup meets at a barrier, and only
// then one thread bumps the arrival counter; readers load the partials after they
// have seen the counter reach its target.
__device__ __forceinline__ void publish_pair(floatx2 *p, floatx2 v)
{
    __hip_atomic_store(reinterpret_cast<unsigned long long *>(p),
                       __builtin_bit_cast(unsigned long long, v), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ floatx2 read_pair(const floatx2 *p)
{
    const unsigned long long bits = __hip_atomic_load(
        reinterpret_cast<const unsigned long long *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return __builtin_bit_cast(floatx2, bits);
}
// This thread's published partials have reached the shared level.
__device__ __forceinline__ void wait_published()
{
    __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0)
}

__device__ __forceinline__ unsigned atomic_add_device(unsigned *p, unsigned v)
{
    return __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned atomic_load_device(const unsigned *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void atomic_store_device(unsigned *p, unsigned v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Wait (bounded) until *counter >= target.  Returns false if the bound expired.
// One thread calls this; the rest of the workgroup waits at a barrier.  The clock
// is read only every 256 polls: reading it costs as much as a poll.
__device__ __forceinline__ bool wait_counter(const unsigned *counter, unsigned target,
                                             long long limit_ticks)
{
    if (atomic_load_device(counter) >= target)
        return true;
    const long long t0 = wall_clock64();
    for (;;) {
        for (int i = 0; i < 256; ++i) {
            __builtin_amdgcn_s_sleep(1);
            if (atomic_load_device(counter) >= target)
                return true;
        }
        if (wall_clock64() - t0 > limit_ticks)
            return false;
    }
}

// Grid-wide arrival spread over several counters.  A few hundred workgroups bumping and polling one
// word queue up behind each other at the memory side; with kSyncWays words on different
// 4 KiB pages the queues are kSyncWays times shorter.  Way w of the control region's counter
// array: arrivals at [w * kSyncStride], departures at [w * kSyncStride + 1]; word [2] counts the
// ways whose workgroups have all departed.
constexpr int kSyncWays = 32;
constexpr int kSyncStride = 1024;  // uint32 words between ways

// Called by every lane of one wavefront; lane l < kSyncWays polls way l until it has seen
// `target` arrivals there (sticky: a way counts once seen).  False if the bound expired.
__device__ __forceinline__ bool wait_counters_wave(const unsigned *counters, unsigned target,
                                                   long long limit_ticks)
{
    const int lane = threadIdx.x & 63;
    const bool polls = lane < kSyncWays;
    const unsigned *mine = counters + (size_t)(polls ? lane : 0) * kSyncStride;
    bool seen = !polls || atomic_load_device(mine) >= target;
    if (__all(seen))
        return true;
    const long long t0 = wall_clock64();
    for (;;) {
        for (int i = 0; i < 256; ++i) {
            __builtin_amdgcn_s_sleep(1);
            if (!seen)
                seen = atomic_load_device(mine) >= target;
            if (__all(seen))
                return true;
        }
        if (wall_clock64() - t0 > limit_ticks)
            return false;
    }
}

}  // namespace ff
