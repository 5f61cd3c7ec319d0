// Host side of the C ABI declared in include/ff.h: argument validation, variant
// selection by shape, workspace management and kernel launches.  Nothing here
// computes on tensors and nothing falls back to a library GEMM or LayerNorm.
#include <mutex>
#include <vector>
#include <algorithm>

#include "../../include/ff.h"
#include "ff_tile.hpp"

namespace {

using namespace ff;

constexpr int kMaxDevices = 64;

// Scratch memory of the entry point that allocates nothing: error word, arrival counters and per-tile
// row statistics of one call, laid out like a workspace.  One copy per device that loads the library,
// held until the process ends.  Host code never uses this name as an address: the per-device address
// comes from hipGetSymbolAddress (no_alloc_scratch below).
constexpr size_t kNoAllocBytes = 8u << 20;
static __device__ __align__(256) unsigned char scratch[kNoAllocBytes];

// Sets `words` 32-bit words at `dst` to `value` (a fill kernel, not a memset node, so that a caller
// may record it into a graph).
__global__ __launch_bounds__(256) void fill_words_kernel(unsigned *dst, size_t words, unsigned value)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < words; i += (size_t)gridDim.x * 256)
        dst[i] = value;
}

// The state a workspace must be in between launches: error word and counters zero.
hipError_t init_control_region(void *ws)
{
    hipError_t e = hipMemset(ws, 0, kCtrlBytes);
    if (e == hipSuccess)
        e = hipDeviceSynchronize();
    return e;
}

struct DeviceState {
    bool probed = false;
    int num_cus = 256;
    long long ticks_per_us = 100;
    void *ws = nullptr;       // bound or owned workspace; its control region is zeroed when it is bound or allocated
    size_t ws_bytes = 0;
    bool ws_owned = false;
    void *no_alloc_ptr = nullptr;            // this device's copy of `scratch`, once asked for
    bool no_alloc_used = false;
    unsigned long long *timeline = nullptr;  // test hook: phase timestamps of the tiled kernels
    size_t timeline_bytes = 0;
    signed char blocks_per_cu[2][kNumTileShapes][3] = {};  // cached occupancy answers [bf16][shape][mode], 0 = not asked
};

std::mutex g_mutex;
DeviceState g_dev[kMaxDevices];
int g_forced_variant = FF_VARIANT_AUTO;
long long g_wait_limit_us = 2000000;
int g_extra_arrivals = 0;
int g_forced_tile = 0;        // 0 = automatic, else 64, 128 or 256
int g_forced_wg_per_cu = 0;   // 0 = automatic (one workgroup per compute unit), else 1 or 2
int g_forced_waves = 0;       // 0 = automatic, else 4 or 8 wavefronts per workgroup of the 256 x 256 tile
int g_stagger_us = 12;        // start delay of the second workgroup per compute unit (256 x 128 tiles)
thread_local int t_last_variant = 0;

struct Plan {
    int variant = 0;
    int shape = 0;     // a TileShape
    int tile_m = 0, tile_n = 0;  // rows and columns of a tile
    int stagger_us = 0;
    int NT = 0, RB = 0;
    int grid = 0, rounds = 0, swz_sc_log2 = -1, nt_log2 = 0, grid_log2 = 0;
    int mt = 0, strips = 0;  // small-M
    size_t partial_off = 0, partial_bytes = 0;
    size_t g_off = 0, g_bytes = 0;
    size_t total_bytes = 0;
};

size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

int validate_shape(int64_t M, int64_t K, int64_t N, int dtype)
{
    if (dtype != FF_F32 && dtype != FF_BF16)
        return FF_ERR_DTYPE;
    if (M <= 0 || K <= 0 || N <= 0)
        return FF_ERR_SHAPE;
    // K is bounded so that 256 rows of X or W span less than 4 GiB (the kernels
    // address a tile's rows with 32-bit byte offsets)
    if (M > (int64_t)1 << 30 || K > (int64_t)1 << 21 || N > (int64_t)1 << 30)
        return FF_ERR_SHAPE;
    const int vec = dtype == FF_BF16 ? 8 : 4;
    if (K % vec != 0 || N % vec != 0)
        return FF_ERR_UNSUPPORTED;
    return FF_OK;
}

// Decides variant, tile size, grid and workspace layout for a shape.
// Workgroups of the chosen tile kernel that fit a compute unit at once, asked of the runtime once per
// kernel and device; 0 when unknown.
int resident_blocks_per_cu(DeviceState *st, bool bf16, int shape, int mode)
{
    if (st == nullptr)
        return 0;
    signed char &slot = st->blocks_per_cu[bf16 ? 1 : 0][shape][mode];
    if (slot == 0) {
        const int n = tile_kernel_blocks_per_cu(bf16, shape, mode);
        slot = (signed char)(n <= 0 ? -1 : (n > 100 ? 100 : n));
    }
    return slot < 0 ? 0 : slot;
}

int make_plan(int64_t M, int64_t K, int64_t N, int dtype, int num_cus, DeviceState *st, int forced,
              bool linear_only, Plan &pl)
{
    (void)K;
    const bool bf16 = dtype == FF_BF16;
    const int64_t strips = (N + kSmallMStripCols - 1) / kSmallMStripCols;
    const bool smallm_ok = bf16 && M <= 32 && strips <= (int64_t)num_cus * kSmallMMaxStripsPerGroup;

    int variant = forced;
    if (linear_only)
        variant = FF_VARIANT_TILED_TWOPASS;  // layout only; the launch uses the linear-only mode
    else if (variant == FF_VARIANT_AUTO)
        variant = smallm_ok ? FF_VARIANT_SMALL_M : 0;

    if (variant == FF_VARIANT_SMALL_M) {
        if (!smallm_ok)
            return FF_ERR_UNSUPPORTED;
        pl.variant = FF_VARIANT_SMALL_M;
        pl.mt = M <= 16 ? 1 : 2;
        pl.strips = (int)strips;
        pl.grid = (int)(strips < num_cus ? strips : num_cus);
        pl.partial_off = kCtrlBytes;
        pl.partial_bytes = round_up((size_t)strips * 16 * pl.mt * sizeof(float) * 2, 256);
        pl.total_bytes = pl.partial_off + pl.partial_bytes;
        return FF_OK;
    }

    // Tiled variants, by how many tiles of a shape there are per compute unit (measured on one device,
    // 1024 x 4096 x 8192, whole call: 256 x 256 tiles 108 us with half the units idle, 256 x 128 tiles
    // 82 us, 128 x 128 tiles two per unit 92 us, the same in two passes 84 us):
    //   more 256 x 256 tiles than half the compute units: 256 x 256 tiles, one workgroup of eight
    //     wavefronts per unit.  Eight wavefronts run the epilogue faster than four (two wavefronts per
    //     SIMD hide each other's latencies) and the K loop up to 4 % slower (half again as many LDS
    //     fragment reads per MFMA); the sum favours eight (4096^3 115.7 against 116.7 us; 65536 x 1024
    //     x 1024 159.5 against 170.7; 8192 x 4096 x 16384 950 against 966);
    //   else, in bf16, if the 128 x 128 tiles outnumber the units but the 256-column x 128-row tiles do
    //     not: 256 x 128 tiles, one per unit, in one round (14 to 20 % faster than 128 x 128 tiles two
    //     per unit on five such shapes; in fp32, where the K loop is eight times longer per slab and
    //     that kernel spills, 128 x 128 tiles win by a third).  Two of those per unit are never chosen: the
    //     overlap of one workgroup's epilogue with the other's K loop does not pay for the 1.5 times
    //     larger L2 -> LDS traffic per flop (4096^3: 148 us);
    //   else 128 x 128 tiles, up to two per unit, which finish in one round; and for at most a
    //     quarter of the units' worth of those, 64 x 64 tiles, which spread them further.
    const int64_t tiles256 = ((M + 255) / 256) * ((N + 255) / 256);
    const int64_t tiles256x128 = ((M + 127) / 128) * ((N + 255) / 256);
    const int64_t tiles128 = ((M + 127) / 128) * ((N + 127) / 128);
    if (tiles256 * 2 > num_cus)
        pl.shape = kTile256W8;
    else if (bf16 && tiles128 > num_cus && tiles256x128 <= num_cus)
        pl.shape = kTile256x128;
    else
        pl.shape = tiles128 * 4 > num_cus ? kTile128 : kTile64;
    if (g_forced_tile != 0) {
        pl.shape = g_forced_tile == 64 ? kTile64 : (g_forced_tile == 128 ? kTile128 : kTile256);
        if (g_forced_tile == 256 && g_forced_wg_per_cu == 2)
            pl.shape = kTile256x128;
    }
    if (g_forced_waves != 0) {
        if (tile_shape_cols(pl.shape) != 256)
            return FF_ERR_UNSUPPORTED;
        pl.shape = g_forced_waves == 8 ? kTile256W8 : kTile256;
    }
    pl.tile_m = tile_shape_rows(pl.shape);
    pl.tile_n = tile_shape_cols(pl.shape);
    const int64_t RB = (M + pl.tile_m - 1) / pl.tile_m;
    const int64_t NT = (N + pl.tile_n - 1) / pl.tile_n;
    if (RB > kMaxRowBlocks - 1 || RB * NT > (int64_t)1 << 30)  // the last counter pair belongs to the cross-entropy kernel
        return FF_ERR_SHAPE;
    pl.RB = (int)RB;
    pl.NT = (int)NT;
    const int64_t total = RB * NT;
    // workgroups per compute unit: a 256 x 256 tile takes a whole unit's LDS and registers, the other
    // shapes half or less
    int per_cu = (pl.shape == kTile256 || pl.shape == kTile256W8) ? 1 : 2;
    if (g_forced_wg_per_cu == 1)
        per_cu = 1;
    // The fused kernel's workgroups wait for one another inside the launch: never launch more of them
    // than the runtime says are resident at once.
    if (variant != FF_VARIANT_TILED_TWOPASS && !linear_only) {
        const int fit = resident_blocks_per_cu(st, bf16, pl.shape, kFused);
        if (fit > 0 && per_cu > fit)
            per_cu = fit;
    }
    const int64_t grid_cap = (int64_t)num_cus * per_cu;
    pl.grid = (int)(total < grid_cap ? total : grid_cap);
    pl.rounds = (int)((total + pl.grid - 1) / pl.grid);
    const bool fused_ok = NT <= pl.grid;
    if (variant == 0)
        variant = fused_ok ? FF_VARIANT_TILED_FUSED : FF_VARIANT_TILED_TWOPASS;
    if (variant == FF_VARIANT_TILED_FUSED && !fused_ok)
        return FF_ERR_UNSUPPORTED;
    if (variant != FF_VARIANT_TILED_FUSED && variant != FF_VARIANT_TILED_TWOPASS)
        return FF_ERR_UNSUPPORTED;
    pl.variant = variant;
    // XCD-aware tile order: needs 8 XCDs x 32 or 64 workgroups and NT a power of two that divides
    // the grid (the kernel's index arithmetic is then all shifts)
    pl.swz_sc_log2 = -1;
    pl.nt_log2 = 0;
    pl.grid_log2 = 0;
    if ((pl.grid == 256 || pl.grid == 512) && NT <= pl.grid && (NT & (NT - 1)) == 0) {
        int sc = (int)(NT / 8 > 8 ? NT / 8 : 8);
        if (sc > NT)
            sc = (int)NT;
        while ((1 << pl.nt_log2) < NT)
            ++pl.nt_log2;
        while ((1 << pl.grid_log2) < pl.grid)
            ++pl.grid_log2;
        pl.swz_sc_log2 = 0;
        while ((1 << pl.swz_sc_log2) < sc)
            ++pl.swz_sc_log2;
    }
    // start delay of the second workgroup of every compute unit (256 x 128 tiles, full grid only)
    pl.stagger_us = (pl.shape == kTile256x128 && per_cu == 2 && pl.grid == 2 * num_cus) ? g_stagger_us : 0;
    pl.partial_off = kCtrlBytes;
    pl.partial_bytes = round_up((size_t)total * pl.tile_m * sizeof(float) * 2, 256);
    pl.g_off = pl.partial_off + pl.partial_bytes;
    pl.g_bytes = (variant == FF_VARIANT_TILED_TWOPASS && !linear_only)
                     ? round_up((size_t)M * (size_t)N * sizeof(float), 256)
                     : 0;
    pl.total_bytes = pl.g_off + pl.g_bytes;
    return FF_OK;
}

DeviceState *current_device_state(int *dev_out = nullptr)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return nullptr;
    }
    DeviceState &st = g_dev[dev];
    if (!st.probed) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            st.num_cus = v;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeWallClockRate, dev) == hipSuccess && v > 0)
            st.ticks_per_us = v / 1000 > 0 ? v / 1000 : 1;
        (void)hipGetLastError();
        st.probed = true;
    }
    if (dev_out)
        *dev_out = dev;
    return &st;
}

// Makes sure a workspace of at least `bytes` exists.  The control region of a workspace is zeroed,
// synchronously, when it is allocated here or bound by ff_set_workspace, never on a caller's stream;
// the kernels leave it zero behind them.  Allocating, freeing and synchronising are illegal while a
// stream is being captured, so a call that would have to grow the library's own workspace during a
// capture is refused instead.
int prepare_workspace(DeviceState &st, size_t bytes, hipStream_t stream)
{
    if (st.ws != nullptr && st.ws_bytes >= bytes)
        return FF_OK;
    if (st.ws != nullptr && !st.ws_owned)
        return FF_ERR_WORKSPACE;  // the caller's workspace is too small
    hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &capture) != hipSuccess) {
        (void)hipGetLastError();
        return FF_ERR_WORKSPACE;
    }
    if (capture != hipStreamCaptureStatusNone)
        return FF_ERR_WORKSPACE;
    if (st.ws != nullptr) {
        if (hipDeviceSynchronize() != hipSuccess || hipFree(st.ws) != hipSuccess) {
            (void)hipGetLastError();
            return FF_ERR_LAUNCH;
        }
        st.ws = nullptr;
        st.ws_bytes = 0;
    }
    const size_t want = round_up(bytes + bytes / 4, 1 << 20);
    void *mem = nullptr;
    if (hipMalloc(&mem, want) != hipSuccess) {
        (void)hipGetLastError();
        return FF_ERR_WORKSPACE;
    }
    if (init_control_region(mem) != hipSuccess) {
        (void)hipGetLastError();
        (void)hipFree(mem);
        return FF_ERR_LAUNCH;
    }
    st.ws = mem;
    st.ws_bytes = want;
    st.ws_owned = true;
    return FF_OK;
}

bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// This device's copy of the static scratch array (asked of the runtime once per device, with that
// device current), or null if the runtime refuses.
void *no_alloc_scratch(DeviceState &st)
{
    if (st.no_alloc_ptr == nullptr) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
            (void)hipGetLastError();
            return nullptr;
        }
        st.no_alloc_ptr = ptr;
    }
    return st.no_alloc_ptr;
}

int run(const void *X, const void *W, const void *b, const void *gamma, const void *beta, float eps,
        int64_t M, int64_t K, int64_t N, int dtype, void *Y, float *Z, bool linear_only,
        hipStream_t stream, bool no_alloc = false)
{
    int rc = validate_shape(M, K, N, dtype);
    if (rc != FF_OK)
        return rc;
    if (!X || !W || (!linear_only && !Y) || (linear_only && !Z))
        return FF_ERR_NULL;
    if (misaligned(X) || misaligned(W) || misaligned(b) || misaligned(gamma) || misaligned(beta) ||
        misaligned(Y) || misaligned(Z))
        return FF_ERR_ALIGN;

    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState *st = current_device_state();
    if (!st)
        return FF_ERR_LAUNCH;
    Plan pl;
    rc = make_plan(M, K, N, dtype, st->num_cus, st, g_forced_variant, linear_only, pl);
    if (rc != FF_OK)
        return rc;
    char *ws = nullptr;
    if (no_alloc) {
        // the static array is the workspace; what the kernels expect to find zero (error word, the
        // arrival counters this plan uses) is cleared by a kernel on the caller's stream first
        if (pl.total_bytes > kNoAllocBytes)
            return FF_ERR_WORKSPACE;
        ws = static_cast<char *>(no_alloc_scratch(*st));
        if (ws == nullptr)
            return FF_ERR_LAUNCH;
        // the error word (offset 0) is cleared by the first call on a device only: later calls leave a
        // failure flagged by an earlier one for ff_check_device to report
        const size_t first = st->no_alloc_used ? kCounterOffset : 0;
        const size_t ctrl = pl.variant == FF_VARIANT_SMALL_M
                                ? kCounterOffset + (size_t)kSyncWays * kSyncStride * sizeof(unsigned)
                                : kCounterOffset + (size_t)pl.RB * 2 * sizeof(unsigned);
        const size_t words = (ctrl - first + 3) / 4;
        hipLaunchKernelGGL(fill_words_kernel, dim3((unsigned)((words + 255) / 256 < 64 ? (words + 255) / 256 : 64)),
                           dim3(256), 0, stream, reinterpret_cast<unsigned *>(ws + first), words, 0u);
        if (hipGetLastError() != hipSuccess)
            return FF_ERR_LAUNCH;
        st->no_alloc_used = true;
    } else {
        rc = prepare_workspace(*st, pl.total_bytes, stream);
        if (rc != FF_OK)
            return rc;
        ws = static_cast<char *>(st->ws);
    }
    unsigned *err = reinterpret_cast<unsigned *>(ws);
    unsigned *counters = reinterpret_cast<unsigned *>(ws + kCounterOffset);
    const long long wait_ticks = g_wait_limit_us * st->ticks_per_us;
    const bool bf16 = dtype == FF_BF16;

    if (pl.variant == FF_VARIANT_SMALL_M) {
        SmallMParams p{};
        p.X = X; p.W = W; p.b = b; p.gamma = gamma; p.beta = beta; p.Y = Y;
        p.partials = reinterpret_cast<floatx2 *>(ws + pl.partial_off);
        p.counters = counters;
        p.err = err;
        p.eps = eps;
        p.M = (int)M; p.K = (int)K; p.N = (int)N;
        p.strips = pl.strips;
        p.extra_arrivals = g_extra_arrivals;
        p.wait_ticks = wait_ticks;
        p.timeline = (st->timeline != nullptr &&
                      st->timeline_bytes >= (size_t)pl.grid * kTimelineSlots * sizeof(unsigned long long))
                         ? st->timeline
                         : nullptr;
        if (launch_smallm_kernel(pl.mt, p, pl.grid, stream) != hipSuccess)
            return FF_ERR_LAUNCH;
        t_last_variant = pl.variant;
        return FF_OK;
    }

    TileParams p{};
    p.X = X; p.W = W; p.b = b; p.gamma = gamma; p.beta = beta; p.Y = Y;
    p.F = linear_only ? Z : reinterpret_cast<float *>(ws + pl.g_off);
    p.partials = reinterpret_cast<floatx2 *>(ws + pl.partial_off);
    p.counters = counters;
    p.err = err;
    p.eps = eps;
    p.M = (int)M; p.K = (int)K; p.N = (int)N;
    p.NT = pl.NT; p.RB = pl.RB; p.rounds = pl.rounds; p.swz_sc_log2 = pl.swz_sc_log2; p.nt_log2 = pl.nt_log2;
    p.grid_log2 = pl.grid_log2;
    p.stagger_ticks = (long long)pl.stagger_us * st->ticks_per_us;
    p.extra_arrivals = g_extra_arrivals;
    p.wait_ticks = wait_ticks;
    p.timeline = nullptr;
    p.timeline_rounds = 0;
    if (st->timeline != nullptr) {
        const size_t per_round = (size_t)pl.grid * kTimelineSlots * sizeof(unsigned long long);
        const size_t rounds = st->timeline_bytes / per_round;
        p.timeline = rounds > 0 ? st->timeline : nullptr;
        p.timeline_rounds = (int)(rounds < (size_t)pl.rounds ? rounds : (size_t)pl.rounds);
    }
    const int mode = linear_only ? kLinearOnly
                                 : (pl.variant == FF_VARIANT_TILED_FUSED ? kFused : kTwoPass);
    if (launch_tile_kernel(bf16, pl.shape, mode, p, pl.grid, stream) != hipSuccess)
        return FF_ERR_LAUNCH;
    if (mode == kTwoPass) {
        FinalizeParams f{};
        f.G = p.F; f.partials = p.partials; f.gamma = gamma; f.beta = beta; f.Y = Y;
        f.eps = eps; f.M = (int)M; f.N = (int)N; f.NT = pl.NT; f.BM = pl.tile_m; f.BN = pl.tile_n;
        if (launch_finalize_kernel(bf16, f, stream) != hipSuccess)
            return FF_ERR_LAUNCH;
    }
    if (!linear_only)
        t_last_variant = pl.variant;
    return FF_OK;
}

}  // namespace

extern "C" {

int ff_fused_linear_gelu_ln(const void *X, const void *W, const void *b, const void *gamma,
                            const void *beta, float eps, int64_t M, int64_t K, int64_t N, int dtype,
                            void *Y, void *stream)
{
    return run(X, W, b, gamma, beta, eps, M, K, N, dtype, Y, nullptr, false,
               static_cast<hipStream_t>(stream));
}

int ff_fused_linear_gelu_ln_noalloc(const void *X, const void *W, const void *b, const void *gamma,
                                    const void *beta, float eps, int64_t M, int64_t K, int64_t N, int dtype,
                                    void *Y, void *stream)
{
    return run(X, W, b, gamma, beta, eps, M, K, N, dtype, Y, nullptr, false,
               static_cast<hipStream_t>(stream), true);
}

size_t ff_noalloc_max_bytes(void) { return kNoAllocBytes; }

int ff_debug_linear(const void *X, const void *W, const void *b, int64_t M, int64_t K, int64_t N,
                    int dtype, float *Z_f32, void *stream)
{
    return run(X, W, b, nullptr, nullptr, 0.0f, M, K, N, dtype, nullptr, Z_f32, true,
               static_cast<hipStream_t>(stream));
}

}  // extern "C"

namespace {

// Column strips and row chunks of the second chain's first phase: 128-byte strips, and as many row
// chunks as give about one (strip, chunk) item per compute unit of the part this was tuned on (the
// kernel loops when there are more items than workgroups).  Few chunks keep the second phase's sum short.
struct RowMeanPlan {
    int strips, k_pad, chunks, rows_per_chunk;
    size_t partial_bytes, cpart_bytes;
};

RowMeanPlan rowmean_plan(int64_t K, int64_t N, int dtype, int num_cus)
{
    RowMeanPlan r{};
    const int64_t strip_elems = 128 / (dtype == FF_BF16 ? 2 : 4);
    r.strips = (int)((K + strip_elems - 1) / strip_elems);
    r.k_pad = (int)(r.strips * strip_elems);
    int64_t want = 256 / r.strips;
    if (want < 1)
        want = 1;
    const int64_t q = kRowMeanRowsPerStep;
    r.rows_per_chunk = (int)(((N + want - 1) / want + q - 1) / q * q);
    r.chunks = (int)((N + r.rows_per_chunk - 1) / r.rows_per_chunk);
    r.partial_bytes = round_up((size_t)r.chunks * (size_t)r.k_pad * sizeof(float), 256);
    r.cpart_bytes = round_up((size_t)num_cus * sizeof(float), 256);
    return r;
}

}  // namespace

extern "C" {

int ff_fused_linear_sub_rowmean_gelu_residual(const void *X, const void *W, const void *b, const void *s,
                                              int64_t M, int64_t K, int64_t N, int dtype, void *Out,
                                              void *stream)
{
    int rc = validate_shape(M, K, N, dtype);
    if (rc != FF_OK)
        return rc;
    if (!X || !W || !Out)
        return FF_ERR_NULL;
    if (misaligned(X) || misaligned(W) || misaligned(b) || misaligned(s) || misaligned(Out))
        return FF_ERR_ALIGN;
    // rowdot keeps K floats of the column means in LDS
    if (K > 32768)
        return FF_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState *st = current_device_state();
    if (!st)
        return FF_ERR_LAUNCH;
    RowMeanParams p{};
    const RowMeanPlan pl = rowmean_plan(K, N, dtype, st->num_cus);
    rc = prepare_workspace(*st, kCtrlBytes + pl.partial_bytes + pl.cpart_bytes, static_cast<hipStream_t>(stream));
    if (rc != FF_OK)
        return rc;
    char *ws = static_cast<char *>(st->ws);
    p.X = X; p.W = W; p.b = b; p.s = s; p.Out = Out;
    p.partial = reinterpret_cast<float *>(ws + kCtrlBytes);
    p.cpart = reinterpret_cast<float *>(ws + kCtrlBytes + pl.partial_bytes);
    p.counters = reinterpret_cast<unsigned *>(ws + kCounterOffset);
    p.err = reinterpret_cast<unsigned *>(ws);
    p.M = (int)M; p.K = (int)K; p.N = (int)N;
    p.strips = pl.strips; p.k_pad = pl.k_pad; p.chunks = pl.chunks; p.rows_per_chunk = pl.rows_per_chunk;
    p.grid = st->num_cus;  // one workgroup per compute unit, all resident: the phases meet inside the launch
    p.extra_arrivals = g_extra_arrivals;
    p.wait_ticks = g_wait_limit_us * st->ticks_per_us;
    if (launch_rowmean_chain(dtype == FF_BF16, p, static_cast<hipStream_t>(stream)) != hipSuccess)
        return FF_ERR_LAUNCH;
    return FF_OK;
}

}  // extern "C"

namespace {

size_t rowmean_workspace_bytes(int64_t K, int64_t N, int dtype)
{
    // sized for any device: the per-workgroup slices take at most 1024 compute units' worth
    const RowMeanPlan pl = rowmean_plan(K, N, dtype, 1024);
    return kCtrlBytes + pl.partial_bytes + pl.cpart_bytes;
}

}  // namespace

extern "C" {

size_t ff_rowmean_workspace_bytes(int64_t M, int64_t K, int64_t N, int dtype)
{
    if (validate_shape(M, K, N, dtype) != FF_OK)
        return 0;
    return rowmean_workspace_bytes(K, N, dtype);
}

int ff_cross_entropy_mean(const void *logits, const int64_t *targets, int64_t B, int64_t C, int dtype,
                          float *row_loss, float *mean_loss, void *stream)
{
    if (dtype != FF_F32 && dtype != FF_BF16)
        return FF_ERR_DTYPE;
    if (B <= 0 || C <= 0 || B > (int64_t)1 << 30 || C > (int64_t)1 << 30)
        return FF_ERR_SHAPE;
    if (!logits || !targets || !mean_loss)
        return FF_ERR_NULL;
    if (misaligned(logits) || (reinterpret_cast<uintptr_t>(targets) & 7u) ||
        (reinterpret_cast<uintptr_t>(row_loss) & 3u) || (reinterpret_cast<uintptr_t>(mean_loss) & 3u))
        return FF_ERR_ALIGN;
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState *st = current_device_state();
    if (!st)
        return FF_ERR_LAUNCH;
    XentParams p{};
    const int64_t row_bytes = C * (dtype == FF_BF16 ? 2 : 4);
    // a wavefront per row while there are rows enough to fill the chip and a row is short;
    // otherwise the whole workgroup shares a row
    p.wg_per_row = (row_bytes >= 64 * 1024 || B < (int64_t)st->num_cus * 16) ? 1 : 0;
    const int64_t groups = p.wg_per_row ? B : (B + 3) / 4;
    // Workgroups per compute unit (measured): fp32 rows stream fastest from few (2: 6.4 against
    // 5.7 TB/s with 8); bf16 rows carry twice the exponentials per byte and need more wavefronts to
    // keep the vector ALUs fed (8), unless that leaves a wavefront fewer than four rows, whose
    // load / reduce phases then stop overlapping across the chip.
    int64_t per_cu = dtype == FF_BF16 ? 8 : 2;
    const int64_t fill = groups / ((int64_t)st->num_cus * 4);
    if (per_cu > fill)
        per_cu = fill < 2 ? 2 : fill;
    const int64_t cap = (int64_t)st->num_cus * per_cu;
    p.grid = (int)(groups < cap ? groups : cap);
    const int rc = prepare_workspace(*st, kCtrlBytes + round_up((size_t)p.grid * sizeof(floatx2), 256),
                                     static_cast<hipStream_t>(stream));
    if (rc != FF_OK)
        return rc;
    char *ws = static_cast<char *>(st->ws);
    p.logits = logits;
    p.targets = reinterpret_cast<const long long *>(targets);
    p.row_loss = row_loss;
    p.mean_loss = mean_loss;
    p.partials = reinterpret_cast<floatx2 *>(ws + kCtrlBytes);
    // the last counter pair of the control region; the tiled kernels never reach it
    p.counter = reinterpret_cast<unsigned *>(ws + kCounterOffset) + 2 * (kMaxRowBlocks - 1);
    p.B = (int)B;
    p.C = (int)C;
    if (launch_xent_kernel(dtype == FF_BF16, p, static_cast<hipStream_t>(stream)) != hipSuccess)
        return FF_ERR_LAUNCH;
    return FF_OK;
}

size_t ff_cross_entropy_workspace_bytes(int64_t B, int64_t C, int dtype)
{
    if ((dtype != FF_F32 && dtype != FF_BF16) || B <= 0 || C <= 0)
        return 0;
    // sized for the largest grid any device uses here (8 workgroups per compute unit, 1024 units)
    return kCtrlBytes + 8192 * sizeof(floatx2);
}

int ff_metric_select_host(const double *r, const uint8_t *keep, int64_t n_tasks, int64_t n_metrics,
                          int top_k, double percentile, int min_tasks, int32_t *top, double *score,
                          uint8_t *selected, double *threshold)
{
    if (!r)
        return FF_ERR_NULL;
    if (n_tasks <= 0 || n_metrics <= 0 || top_k <= 0 || n_tasks > 1 << 20 || n_metrics > 1 << 24 ||
        !(percentile >= 0.0 && percentile <= 100.0) || min_tasks < 1)
        return FF_ERR_SHAPE;
    try {
        metric_select_host(r, keep, (int)n_tasks, (int)n_metrics, top_k, percentile, min_tasks, top, score,
                           selected, threshold);
    } catch (...) {  // host allocation failed: nothing may leave through the C boundary
        return FF_ERR_WORKSPACE;
    }
    return FF_OK;
}

int ff_metric_selection(const double *values, const double *runtime, int64_t n_tasks, int64_t n_kernels,
                        int64_t n_metrics, int top_k, double percentile, double collinear_tau,
                        int min_tasks, double *r_host, double *score_host, int32_t *top_host,
                        uint8_t *selected_host, double *threshold_host, void *stream)
{
    if (!values || !runtime)
        return FF_ERR_NULL;
    if (n_tasks <= 0 || n_kernels <= 0 || n_metrics <= 0 || top_k <= 0 || n_tasks > 1 << 16 ||
        n_kernels > 1 << 20 || n_metrics > 1 << 24 || !(percentile >= 0.0 && percentile <= 100.0) ||
        min_tasks < 1)
        return FF_ERR_SHAPE;
    const bool filter = collinear_tau > 0.0 && collinear_tau <= 1.0;
    if (filter && n_metrics > 8192)
        return FF_ERR_UNSUPPORTED;  // the J x J correlation matrix of a task is held in the workspace
    if ((reinterpret_cast<uintptr_t>(values) & 7u) || (reinterpret_cast<uintptr_t>(runtime) & 7u))
        return FF_ERR_ALIGN;
    const int n = (int)n_tasks, V = (int)n_kernels, J = (int)n_metrics;
    hipStream_t st_stream = static_cast<hipStream_t>(stream);
    try {
    std::vector<double> r((size_t)n * J);
    std::vector<uint8_t> keep;
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        DeviceState *st = current_device_state();
        if (!st)
            return FF_ERR_LAUNCH;
        const size_t r_bytes = round_up((size_t)n * J * sizeof(double), 256);
        const size_t z_bytes = filter ? round_up((size_t)V * J * sizeof(double), 256) : 0;
        const size_t c_bytes = filter ? round_up((size_t)J * J * sizeof(double), 256) : 0;
        const int rc = prepare_workspace(*st, kCtrlBytes + r_bytes + z_bytes + c_bytes, st_stream);
        if (rc != FF_OK)
            return rc;
        char *ws = static_cast<char *>(st->ws);
        double *r_dev = reinterpret_cast<double *>(ws + kCtrlBytes);
        double *z_dev = reinterpret_cast<double *>(ws + kCtrlBytes + r_bytes);
        double *c_dev = reinterpret_cast<double *>(ws + kCtrlBytes + r_bytes + z_bytes);
        if (launch_pearson(values, runtime, r_dev, n, V, J, st_stream) != hipSuccess)
            return FF_ERR_LAUNCH;
        if (hipMemcpyAsync(r.data(), r_dev, (size_t)n * J * sizeof(double), hipMemcpyDeviceToHost, st_stream) !=
            hipSuccess)
            return FF_ERR_LAUNCH;
        if (filter) {
            keep.resize((size_t)n * J);
            std::vector<double> C((size_t)J * J);
            for (int i = 0; i < n; ++i) {
                if (launch_corr_matrix(values + (size_t)i * V * J, z_dev, c_dev, V, J, st_stream) != hipSuccess)
                    return FF_ERR_LAUNCH;
                if (hipMemcpyAsync(C.data(), c_dev, (size_t)J * J * sizeof(double), hipMemcpyDeviceToHost,
                                   st_stream) != hipSuccess ||
                    hipStreamSynchronize(st_stream) != hipSuccess)
                    return FF_ERR_LAUNCH;
                metric_greedy_keep(C.data(), J, collinear_tau, keep.data() + (size_t)i * J);
            }
        }
        if (hipStreamSynchronize(st_stream) != hipSuccess)
            return FF_ERR_LAUNCH;
    }
    metric_select_host(r.data(), filter ? keep.data() : nullptr, n, J, top_k, percentile, min_tasks, top_host,
                       score_host, selected_host, threshold_host);
    if (r_host)
        std::copy(r.begin(), r.end(), r_host);
    } catch (...) {  // host allocation failed: nothing may leave through the C boundary
        return FF_ERR_WORKSPACE;
    }
    return FF_OK;
}

size_t ff_workspace_bytes(int64_t M, int64_t K, int64_t N, int dtype)
{
    if (validate_shape(M, K, N, dtype) != FF_OK)
        return 0;
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState *st = current_device_state();
    const int num_cus = st ? st->num_cus : 256;
    Plan pl;
    if (make_plan(M, K, N, dtype, num_cus, st, g_forced_variant, false, pl) != FF_OK)
        return 0;
    return pl.total_bytes;
}

int ff_plan_query(int64_t M, int64_t K, int64_t N, int dtype, int out[8])
{
    if (out == nullptr)
        return FF_ERR_NULL;
    const int rc = validate_shape(M, K, N, dtype);
    if (rc != FF_OK)
        return rc;
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState *st = current_device_state();
    const int num_cus = st ? st->num_cus : 256;
    Plan pl;
    const int prc = make_plan(M, K, N, dtype, num_cus, st, g_forced_variant, false, pl);
    if (prc != FF_OK)
        return prc;
    const bool small = pl.variant == FF_VARIANT_SMALL_M;
    out[0] = pl.variant;
    out[1] = small ? (int)M : pl.tile_m;
    out[2] = small ? kSmallMStripCols : pl.tile_n;
    out[3] = small ? 8 : tile_shape_waves(pl.shape);
    out[4] = pl.grid;
    out[5] = small ? 1 : pl.rounds;
    out[6] = (pl.grid + num_cus - 1) / num_cus;
    out[7] = (!small && pl.swz_sc_log2 >= 0) ? 1 : 0;
    return FF_OK;
}

int ff_set_workspace(void *dev_ptr, size_t bytes)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState *st = current_device_state();
    if (!st)
        return FF_ERR_LAUNCH;
    if (dev_ptr != nullptr && ((reinterpret_cast<uintptr_t>(dev_ptr) & 255u) != 0))
        return FF_ERR_ALIGN;
    if (dev_ptr != nullptr && bytes < kCtrlBytes)
        return FF_ERR_WORKSPACE;
    if (dev_ptr != nullptr && init_control_region(dev_ptr) != hipSuccess) {
        (void)hipGetLastError();
        return FF_ERR_LAUNCH;  // the old binding stays
    }
    if (st->ws != nullptr && st->ws_owned) {
        if (hipDeviceSynchronize() != hipSuccess || hipFree(st->ws) != hipSuccess) {
            (void)hipGetLastError();
            return FF_ERR_LAUNCH;
        }
    }
    st->ws = dev_ptr;
    st->ws_bytes = dev_ptr ? bytes : 0;
    st->ws_owned = false;
    return FF_OK;
}

int ff_check_device(void *stream)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState *st = current_device_state();
    if (!st)
        return FF_ERR_LAUNCH;
    if (hipStreamSynchronize(static_cast<hipStream_t>(stream)) != hipSuccess) {
        (void)hipGetLastError();
        return FF_ERR_LAUNCH;
    }
    bool failed = false;
    void *regions[2] = {st->ws, st->no_alloc_used ? st->no_alloc_ptr : nullptr};
    for (void *region : regions) {
        if (region == nullptr)
            continue;
        unsigned flag = 0;
        if (hipMemcpy(&flag, region, sizeof(flag), hipMemcpyDeviceToHost) != hipSuccess) {
            (void)hipGetLastError();
            return FF_ERR_LAUNCH;
        }
        if (flag != 0) {
            // a wait gave up: counters may be half-way; start from a clean control region
            (void)init_control_region(region);
            failed = true;
        }
    }
    return failed ? FF_ERR_DEVICE : FF_OK;
}

const char *ff_status_string(int status)
{
    switch (status) {
    case FF_OK: return "FF_OK";
    case FF_ERR_NULL: return "FF_ERR_NULL: a required pointer is NULL";
    case FF_ERR_SHAPE: return "FF_ERR_SHAPE: M, K and N must be positive, M and N at most 2^30, K at most 2^21";
    case FF_ERR_DTYPE: return "FF_ERR_DTYPE: dtype must be FF_F32 or FF_BF16";
    case FF_ERR_ALIGN: return "FF_ERR_ALIGN: pointers must be 16-byte aligned";
    case FF_ERR_UNSUPPORTED: return "FF_ERR_UNSUPPORTED: K and N must be multiples of 8 (bf16) or 4 (fp32), or the forced variant cannot run this shape";
    case FF_ERR_WORKSPACE: return "FF_ERR_WORKSPACE: workspace too small or allocation failed";
    case FF_ERR_LAUNCH: return "FF_ERR_LAUNCH: the HIP runtime refused the request";
    case FF_ERR_DEVICE: return "FF_ERR_DEVICE: a workgroup gave up waiting for the other tiles of its rows";
    default: return "unknown ff_status";
    }
}

int ff_version(void) { return 100; }

int ff_last_variant(void) { return t_last_variant; }

int ff_debug_force_variant(int variant)
{
    if (variant < FF_VARIANT_AUTO || variant > FF_VARIANT_SMALL_M)
        return FF_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_mutex);
    g_forced_variant = variant;
    return FF_OK;
}

int ff_debug_force_tile(int tile, int wg_per_cu)
{
    if ((tile != 0 && tile != 64 && tile != 128 && tile != 256) || wg_per_cu < 0 || wg_per_cu > 2)
        return FF_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_mutex);
    g_forced_tile = tile;
    g_forced_wg_per_cu = wg_per_cu;
    return FF_OK;
}

int ff_debug_force_waves(int waves)
{
    if (waves != 0 && waves != 4 && waves != 8)
        return FF_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_mutex);
    g_forced_waves = waves;
    return FF_OK;
}

int ff_debug_set_stagger_us(int microseconds)
{
    if (microseconds < 0 || microseconds > 1000)
        return FF_ERR_SHAPE;
    std::lock_guard<std::mutex> lock(g_mutex);
    g_stagger_us = microseconds;
    return FF_OK;
}

int ff_debug_set_timeline(void *dev_ptr, size_t bytes)
{
    if (dev_ptr != nullptr && (reinterpret_cast<uintptr_t>(dev_ptr) & 7u) != 0)
        return FF_ERR_ALIGN;
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState *st = current_device_state();
    if (!st)
        return FF_ERR_LAUNCH;
    st->timeline = static_cast<unsigned long long *>(dev_ptr);
    st->timeline_bytes = dev_ptr ? bytes : 0;
    return FF_OK;
}

int ff_debug_copy(const void *src, void *dst, size_t bytes, void *stream)
{
    if (!src || !dst)
        return FF_ERR_NULL;
    if (misaligned(src) || misaligned(dst))
        return FF_ERR_ALIGN;
    if (bytes % 16 != 0)
        return FF_ERR_UNSUPPORTED;
    DeviceState *st = current_device_state();
    if (!st)
        return FF_ERR_LAUNCH;
    if (launch_copy_kernel(src, dst, bytes, st->num_cus, static_cast<hipStream_t>(stream)) != hipSuccess)
        return FF_ERR_LAUNCH;
    return FF_OK;
}

int ff_debug_mfma_loop(int64_t iters, double *flops)
{
    if (!flops)
        return FF_ERR_NULL;
    if (iters <= 0 || iters > (int64_t)1 << 32)
        return FF_ERR_SHAPE;
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState *st = current_device_state();
    if (!st)
        return FF_ERR_LAUNCH;
    // the kernel's per-thread results go to the workspace (they only keep the loop alive)
    const int rc = prepare_workspace(*st, kCtrlBytes + (size_t)st->num_cus * 256 * sizeof(float), nullptr);
    if (rc != FF_OK)
        return rc;
    float *sink = reinterpret_cast<float *>(static_cast<char *>(st->ws) + kCtrlBytes);
    if (launch_mfma_loop(iters, sink, st->num_cus, nullptr, flops) != hipSuccess)
        return FF_ERR_LAUNCH;
    return FF_OK;
}

int ff_debug_stream_read(const void *src, size_t bytes)
{
    if (!src)
        return FF_ERR_NULL;
    if (misaligned(src))
        return FF_ERR_ALIGN;
    if (bytes % 16 != 0)
        return FF_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState *st = current_device_state();
    if (!st)
        return FF_ERR_LAUNCH;
    const int rc = prepare_workspace(*st, kCtrlBytes + (size_t)st->num_cus * 2 * 256 * sizeof(unsigned), nullptr);
    if (rc != FF_OK)
        return rc;
    unsigned *sink = reinterpret_cast<unsigned *>(static_cast<char *>(st->ws) + kCtrlBytes);
    if (launch_stream_read(src, bytes, sink, st->num_cus, nullptr) != hipSuccess)
        return FF_ERR_LAUNCH;
    return FF_OK;
}

int ff_debug_expect_extra_arrivals(int count)
{
    if (count < 0 || count > 1024)
        return FF_ERR_SHAPE;
    std::lock_guard<std::mutex> lock(g_mutex);
    g_extra_arrivals = count;
    return FF_OK;
}

int ff_debug_set_wait_limit_us(int64_t microseconds)
{
    if (microseconds <= 0)
        return FF_ERR_SHAPE;
    std::lock_guard<std::mutex> lock(g_mutex);
    g_wait_limit_us = microseconds;
    return FF_OK;
}

}  // extern "C"
