// Host/device interface of the kernels: parameter blocks and launch functions.
#pragma once
#include <type_traits>

#include "ff_device.hpp"

namespace ff {

enum { kFused = 0, kTwoPass = 1, kLinearOnly = 2 };
enum { kPipeDma = 0, kPipeXReg = 1 };

struct TileParams {
    const void *X;       // [M,K]
    const void *W;       // [N,K]
    const void *b;       // [N] or null
    const void *gamma;   // [N] or null
    const void *beta;    // [N] or null
    void *Y;             // kFused: [M,N] in the tensor dtype
    float *F;            // kTwoPass: fp32 G scratch [M,N]; kLinearOnly: fp32 Z out
    floatx2 *partials;   // [RB][NT][BM] (mean, M2) per tile row
    unsigned *counters;  // [RB][2] arrival, departure
    unsigned *err;       // error word
    float eps;
    int M, K, N;
    int NT;              // tiles along N
    int RB;              // row-blocks
    int rounds;          // ceil(RB * NT / grid)
    int swz_sc_log2;     // XCD-aware order: log2 of the super-block width in tiles, -1 = plain order
    int nt_log2;         // log2(NT) when the XCD-aware order is on
    int grid_log2;       // log2(grid) when the XCD-aware order is on
    long long stagger_ticks;  // start delay (wall-clock ticks) of the second half of the grid, 0 = none
    int extra_arrivals;  // test hook: added to the arrival target (non-zero makes waits expire)
    long long wait_ticks;
    unsigned long long *timeline;  // test hook: phase timestamps, or null
    int timeline_rounds;           // rounds of tiles the timeline buffer has room for
};

// Timeline record of one tile: slots 0..6 wall-clock stamps (tile start, first slab landed, main
// loop done, statistics published, other tiles arrived, statistics merged, stores issued); slots
// kTimelineCycleSlot, +1 the shader clock at the start and end of the main loop.
constexpr int kTimelineSlots = 16;
constexpr int kTimelineCycleSlot = 8;

struct FinalizeParams {
    const float *G;
    const floatx2 *partials;
    const void *gamma;
    const void *beta;
    void *Y;
    float eps;
    int M, N, NT, BM, BN;
};

struct SmallMParams {
    const void *X, *W, *b, *gamma, *beta;
    void *Y;
    floatx2 *partials;   // [strips][16 * MT] (mean, M2)
    unsigned *counters;  // [2]
    unsigned *err;
    float eps;
    int M, K, N;
    int strips;          // N / 32 rounded up
    int extra_arrivals;  // test hook: added to the arrival target (non-zero makes waits expire)
    long long wait_ticks;
    unsigned long long *timeline;  // test hook: phase timestamps, or null
};

// second chain: 512 threads; phase 1 covers 64 rows x 128 bytes of W per load instruction
constexpr int kRowMeanThreads = 512;
constexpr int kRowMeanRowsPerStep = 64;

struct RowMeanParams {
    const void *X, *W, *b, *s;
    void *Out;
    float *partial;      // [chunks][k_pad] partial column sums of W
    float *cpart;        // [grid] slices of sum(b - s)
    unsigned *counters;  // control-region counter array (zero before and after a launch)
    unsigned *err;
    int M, K, N;
    int strips;          // 128-byte column strips; k_pad = strips * (128 / sizeof T)
    int k_pad;
    int chunks, rows_per_chunk;  // row chunks of W; rows_per_chunk is a multiple of kRowMeanRowsPerStep
    int grid;            // one workgroup per compute unit: all co-resident
    int extra_arrivals;  // test hook
    long long wait_ticks;
};

struct XentParams {
    const void *logits;        // [B][C]
    const long long *targets;  // [B]
    float *row_loss;           // [B] or null
    float *mean_loss;          // [1]
    floatx2 *partials;         // [grid]: one number per workgroup (second component unused)
    unsigned *counter;         // arrivals of this launch; zero before and after
    int B, C;
    int grid;
    int wg_per_row;            // 1: a workgroup per row (long rows, few rows); 0: a wavefront per row
};

hipError_t launch_copy_kernel(const void *src, void *dst, size_t bytes, int num_cus, hipStream_t stream);
hipError_t launch_mfma_loop(long long iters, float *sink, int num_cus, hipStream_t stream, double *flops);
hipError_t launch_stream_read(const void *src, size_t bytes, unsigned *sink, int num_cus, hipStream_t stream);

// profiling-metric selection: device correlations, host selection
hipError_t launch_pearson(const double *values, const double *runtime, double *r, int n, int V, int J,
                          hipStream_t stream);
hipError_t launch_corr_matrix(const double *task_values, double *Z, double *C, int V, int J, hipStream_t stream);
void metric_greedy_keep(const double *C, int J, double tau, unsigned char *keep);
void metric_select_host(const double *r, const unsigned char *keep, int n, int J, int k, double q,
                        int min_tasks, int *top, double *score, unsigned char *selected, double *threshold);

hipError_t launch_xent_kernel(bool bf16, const XentParams &p, hipStream_t stream);
hipError_t launch_rowmean_chain(bool bf16, const RowMeanParams &p, hipStream_t stream);
// Tile shapes of the tiled kernels (columns x rows of the output a workgroup owns).
enum TileShape {
    kTile64 = 0,       // 64 x 64, four wavefronts, up to four workgroups per compute unit
    kTile128 = 1,      // 128 x 128, four wavefronts, two workgroups per compute unit
    kTile256 = 2,      // 256 x 256, four wavefronts of 4 x 4 MFMA blocks, one workgroup per compute unit
    kTile256W8 = 3,    // 256 x 256, eight wavefronts of 4 x 2 blocks, one workgroup per compute unit
    kTile256x128 = 4,  // 256 columns x 128 rows, four wavefronts of 4 x 2 blocks, two workgroups per compute unit
    kNumTileShapes = 5
};
inline int tile_shape_cols(int shape) { return shape == kTile64 ? 64 : (shape == kTile128 ? 128 : 256); }
inline int tile_shape_rows(int shape)
{
    return shape == kTile64 ? 64 : ((shape == kTile128 || shape == kTile256x128) ? 128 : 256);
}
inline int tile_shape_waves(int shape) { return shape == kTile256W8 ? 8 : 4; }
hipError_t launch_tile_kernel(bool bf16, int shape, int mode, const TileParams &p, int grid, hipStream_t stream);
int tile_kernel_blocks_per_cu(bool bf16, int shape, int mode);
hipError_t launch_finalize_kernel(bool bf16, const FinalizeParams &p, hipStream_t stream);
hipError_t launch_smallm_kernel(int mt, const SmallMParams &p, int grid, hipStream_t stream);

constexpr int kSmallMStripCols = 32;
constexpr int kSmallMMaxStripsPerGroup = 8;

}  // namespace ff
