// Host/device interface of the kernels: parameter blocks and launch functions.
#pragma once
#include <type_traits>

#include "ff_device.hpp"

namespace ff {

enum { kFused = 0, kTwoPass = 1, kLinearOnly = 2 };

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
    int swz_sc;          // XCD-aware order: super-block width in tiles, 0 = plain order
    int extra_arrivals;  // test hook: added to the arrival target (non-zero makes waits expire)
    long long wait_ticks;
};

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
hipError_t launch_tile_kernel(bool bf16, int tile, int mode, const TileParams &p, int grid,
                              hipStream_t stream);
hipError_t launch_finalize_kernel(bool bf16, const FinalizeParams &p, hipStream_t stream);
hipError_t launch_smallm_kernel(int mt, const SmallMParams &p, int grid, hipStream_t stream);

constexpr int kSmallMStripCols = 32;
constexpr int kSmallMMaxStripsPerGroup = 8;

}  // namespace ff
