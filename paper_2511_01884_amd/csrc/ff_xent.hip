// Row-wise cross-entropy: the row reduction of the paper's case study (Sec. 4),
//
//     loss[r] = log( sum_c exp(L[r][c]) ) - L[r][t[r]],    mean = (1/B) sum_r loss[r].
//
// The case study's kernel went from block-wide shared-memory reductions to
// shuffle reductions with a single cross-wavefront combine, and then removed the
// second global read of the logits by buffering the row on chip.  Here the
// second read is removed at the source instead: every lane keeps a running
// (maximum, sum of exp(x - maximum)) pair and rescales the sum whenever its
// maximum moves, so a row is read exactly once however long it is and nothing
// has to be buffered.  Lanes are combined with a shuffle butterfly; in the
// long-row variant the four wavefronts of a workgroup are then combined once
// through LDS.  The kernel is bound by the HBM read of L.
//
// The mean over rows is part of the same launch: each workgroup adds the losses
// of its rows in row order, publishes that one number, and the workgroup that
// arrives last adds the published numbers in workgroup order.  All orders are
// fixed by the launch shape, so results are bitwise reproducible.
#include "ff_tile.hpp"

namespace ff {

namespace {

constexpr int kThreads = 256;
constexpr int kInFlight = 8;  // chunk loads a lane issues back to back
constexpr float kLog2e = 1.44269504088896341f;
constexpr float kLn2 = 0.693147180559945309f;

__device__ __forceinline__ float exp2_hw(float x) { return __builtin_amdgcn_exp2f(x); }

// Reference point for the exponents: the maximum, or 0 while the maximum is still -inf
// (so that -inf - (-inf) never appears).
__device__ __forceinline__ float ref_of(float m) { return m == -INFINITY ? 0.0f : m; }

// (m, s) <- (m, s) combined with (mb, sb); s counts exp(x - m) over the values seen
__device__ __forceinline__ void combine(float &m, float &s, float mb, float sb)
{
    const float mn = fmaxf(m, mb);
    const float ref = ref_of(mn);
    s = s * exp2_hw((m - ref) * kLog2e) + sb * exp2_hw((mb - ref) * kLog2e);
    m = mn;
}

template <typename T, int VEC> struct Chunk;
template <> struct Chunk<float, 4> {
    uintx4 v;
    __device__ __forceinline__ void load(const float *p) { v = __builtin_nontemporal_load(reinterpret_cast<const uintx4 *>(p)); }
    __device__ __forceinline__ void get(float (&f)[4]) const
    {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            f[i] = __uint_as_float(v[i]);
    }
};
template <> struct Chunk<__bf16, 8> {
    uintx4 v;
    __device__ __forceinline__ void load(const __bf16 *p) { v = __builtin_nontemporal_load(reinterpret_cast<const uintx4 *>(p)); }
    __device__ __forceinline__ void get(float (&f)[8]) const
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(v[i] << 16);
            f[2 * i + 1] = __uint_as_float(v[i] & 0xffff0000u);
        }
    }
};
template <> struct Chunk<float, 1> {
    float v;
    __device__ __forceinline__ void load(const float *p) { v = *p; }
    __device__ __forceinline__ void get(float (&f)[1]) const { f[0] = v; }
};
template <> struct Chunk<__bf16, 1> {
    unsigned short v;
    __device__ __forceinline__ void load(const __bf16 *p) { v = *reinterpret_cast<const unsigned short *>(p); }
    __device__ __forceinline__ void get(float (&f)[1]) const { f[0] = bf16_bits_to_float(v); }
};

// Fold one chunk's values into the lane's running pair.
template <int VEC>
__device__ __forceinline__ void fold(float &m, float &s, const float (&f)[VEC])
{
    float cm = f[0];
#pragma unroll
    for (int e = 1; e < VEC; ++e)
        cm = fmaxf(cm, f[e]);
    const float mn = fmaxf(m, cm);
    const float ref = ref_of(mn);
    float add = 0.0f;
#pragma unroll
    for (int e = 0; e < VEC; ++e)
        add += exp2_hw((f[e] - ref) * kLog2e);
    s = fmaf(s, exp2_hw((m - ref) * kLog2e), add);
    m = mn;
}

// Fold a whole batch of chunks with one rescale: the batch's maximum first, then every element's
// exponential against it (per-chunk sums, added in chunk order).  Against folding chunk by chunk this
// saves one exponential and a few selects per chunk, which matters for bf16 rows: they carry twice the
// elements per byte and sit at the vector-ALU limit.
template <int VEC>
__device__ __forceinline__ void fold_batch(float &m, float &s, const float (&f)[kInFlight][VEC])
{
    float bm = f[0][0];
#pragma unroll
    for (int u = 0; u < kInFlight; ++u)
#pragma unroll
        for (int e = 0; e < VEC; ++e)
            bm = fmaxf(bm, f[u][e]);
    const float mn = fmaxf(m, bm);
    const float ref = ref_of(mn);
    float add = 0.0f;
#pragma unroll
    for (int u = 0; u < kInFlight; ++u) {
        float part = 0.0f;
#pragma unroll
        for (int e = 0; e < VEC; ++e)
            part += exp2_hw((f[u][e] - ref) * kLog2e);
        add += part;
    }
    s = fmaf(s, exp2_hw((m - ref) * kLog2e), add);
    m = mn;
}

// ROWT threads share a row: 64 (a wavefront per row, four rows per workgroup) or 256 (the
// workgroup per row).  VEC = elements per load: 16 bytes' worth, or 1 when C is not a multiple
// of that.
template <typename T, int VEC, int ROWT>
__global__ __launch_bounds__(kThreads) void xent_kernel(XentParams p)
{
    __shared__ float s_m[4], s_s[4], s_loss[4];
    __shared__ float s_red[kThreads];
    __shared__ unsigned s_last;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    constexpr int kGroupsPerWg = kThreads / ROWT;
    const int tl = threadIdx.x % ROWT;  // thread within the row's group
    const int group = (ROWT == 64) ? blockIdx.x * kGroupsPerWg + wave : blockIdx.x;
    const int ngroups = gridDim.x * kGroupsPerWg;
    const T *L = reinterpret_cast<const T *>(p.logits);
    const int nchunks = p.C / VEC;
    float loss_sum = 0.0f;  // losses of this group's rows, in row order (same in every lane)

    for (int r = group; r < p.B; r += ngroups) {
        const T *row = L + (size_t)r * (size_t)p.C;
        const long long t = p.targets[r];
        const bool t_ok = t >= 0 && t < (long long)p.C;
        const float xt = load_as_float(row + (t_ok ? t : 0));  // one more element, usually an L2 hit
        float m = -INFINITY, s = 0.0f;
        int ch = tl;
        // whole batches: all of this lane's loads are inside the row
        for (; ch + (kInFlight - 1) * ROWT < nchunks; ch += kInFlight * ROWT) {
            Chunk<T, VEC> c[kInFlight];
#pragma unroll
            for (int u = 0; u < kInFlight; ++u)
                c[u].load(row + (size_t)(ch + u * ROWT) * VEC);
            float f[kInFlight][VEC];
#pragma unroll
            for (int u = 0; u < kInFlight; ++u)
                c[u].get(f[u]);
            fold_batch<VEC>(m, s, f);
        }
        // the rest of the row, one chunk at a time
        for (; ch < nchunks; ch += ROWT) {
            Chunk<T, VEC> c;
            c.load(row + (size_t)ch * VEC);
            float f[VEC];
            c.get(f);
            fold<VEC>(m, s, f);
        }
        // lanes of a wavefront: butterfly; lane 0's result is the wavefront's
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const float mb = __shfl_xor(m, off);
            const float sb = __shfl_xor(s, off);
            combine(m, s, mb, sb);
        }
        m = __shfl(m, 0);
        s = __shfl(s, 0);
        if (ROWT == 256) {  // the single cross-wavefront combine, in wavefront order
            __syncthreads();  // the previous row's readers are done with s_m, s_s
            if (lane == 0) {
                s_m[wave] = m;
                s_s[wave] = s;
            }
            __syncthreads();
            m = s_m[0];
            s = s_s[0];
#pragma unroll
            for (int w = 1; w < 4; ++w)
                combine(m, s, s_m[w], s_s[w]);
        }
        float loss = (m - xt) + __builtin_amdgcn_logf(s) * kLn2;
        if (!t_ok)
            loss = __builtin_nanf("");
        if (p.row_loss && tl == 0)
            p.row_loss[r] = loss;
        loss_sum += loss;
    }

    // workgroup's number: its groups in order
    if (ROWT == 64) {
        if (lane == 0)
            s_loss[wave] = loss_sum;
        __syncthreads();
        loss_sum = ((s_loss[0] + s_loss[1]) + s_loss[2]) + s_loss[3];
    }
    if (threadIdx.x == 0) {
        publish_pair(p.partials + blockIdx.x, floatx2{loss_sum, 0.0f});
        wait_published();
        const unsigned before = atomic_add_device(p.counter, 1u);
        s_last = (before + 1u == gridDim.x) ? 1u : 0u;
    }
    __syncthreads();
    if (s_last == 0u)
        return;
    // last workgroup to arrive: every other workgroup's number is visible; add them in workgroup order
    float acc = 0.0f;
    for (int i = threadIdx.x; i < (int)gridDim.x; i += kThreads)
        acc += read_pair(p.partials + i)[0];
    s_red[threadIdx.x] = acc;
    __syncthreads();
    for (int off = kThreads / 2; off >= 1; off >>= 1) {
        if ((int)threadIdx.x < off)
            s_red[threadIdx.x] += s_red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        *p.mean_loss = s_red[0] / (float)p.B;
        atomic_store_device(p.counter, 0u);  // ready for the next launch
    }
}

template <typename T, int VEC>
hipError_t launch_v(const XentParams &p, hipStream_t stream)
{
    if (p.wg_per_row)
        hipLaunchKernelGGL((xent_kernel<T, VEC, 256>), dim3(p.grid), dim3(kThreads), 0, stream, p);
    else
        hipLaunchKernelGGL((xent_kernel<T, VEC, 64>), dim3(p.grid), dim3(kThreads), 0, stream, p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_xent_kernel(bool bf16, const XentParams &p, hipStream_t stream)
{
    if (bf16)
        return p.C % 8 == 0 ? launch_v<__bf16, 8>(p, stream) : launch_v<__bf16, 1>(p, stream);
    return p.C % 4 == 0 ? launch_v<float, 4>(p, stream) : launch_v<float, 1>(p, stream);
}

}  // namespace ff
