// Profiling-metric selection (the paper's Sec. 2.3, Steps 2 and 3; Alg. 2).
//
// Input: n tasks, V kernels per task, J metrics per kernel, one runtime per kernel.
//   Step 2, per task: r[i][m] = Pearson correlation over the task's kernels between metric m and
//   the runtime; optionally drop metrics that duplicate an earlier kept one (|correlation| >= tau);
//   Top-k = the k kept metrics with the largest |r|.
//   Step 3: candidates = union of the Top-k lists; score S[m] = mean over all tasks of |r[i][m]|;
//   selected = candidates that are in the Top-k of at least `min_tasks` tasks, whose r has one sign
//   over those tasks, and whose score exceeds the given percentile of the candidates' scores.
// The correlations (one thread per task and metric, and one per pair of metrics for the duplicate
// filter) are computed on the GPU in fp64; the selection itself is a few hundred numbers and runs
// on the host.  An undefined correlation (constant column or constant runtime) is NaN: it never
// enters a Top-k and counts as 0 in the score.  Ties in |r| go to the lower metric index.  The
// percentile interpolates linearly between order statistics.
#include "ff_tile.hpp"

#include <algorithm>
#include <cmath>
#include <vector>

namespace ff {

namespace {

// r[i][m]: two passes over the V values of the column (mean, then centred sums), all in fp64.
__global__ __launch_bounds__(256) void pearson_kernel(const double *values, const double *runtime, double *r,
                                                      int V, int J)
{
    const int m = blockIdx.x * 256 + threadIdx.x;
    const int i = blockIdx.y;
    if (m >= J)
        return;
    const double *col = values + (size_t)i * V * J + m;
    const double *rt = runtime + (size_t)i * V;
    // a sample is constant when all its values are equal (compared as values: the mean of equal
    // values need not round back to that value, so the variance is no test)
    double mx = 0.0, my = 0.0;
    bool x_const = true, y_const = true;
    for (int v = 0; v < V; ++v) {
        const double x = col[(size_t)v * J];
        mx += x;
        my += rt[v];
        x_const = x_const && x == col[0];
        y_const = y_const && rt[v] == rt[0];
    }
    if (x_const || y_const) {
        r[(size_t)i * J + m] = __builtin_nan("");
        return;
    }
    mx /= (double)V;
    my /= (double)V;
    double sxy = 0.0, sxx = 0.0, syy = 0.0;
    for (int v = 0; v < V; ++v) {
        const double dx = col[(size_t)v * J] - mx;
        const double dy = rt[v] - my;
        sxy += dx * dy;
        sxx += dx * dx;
        syy += dy * dy;
    }
    r[(size_t)i * J + m] = (sxx > 0.0 && syy > 0.0) ? sxy / sqrt(sxx * syy) : __builtin_nan("");
}

// Z[v][m] = (x - mean) / sqrt(sum (x - mean)^2) for one task; a constant column becomes NaN.
__global__ __launch_bounds__(256) void standardise_kernel(const double *task_values, double *Z, int V, int J)
{
    const int m = blockIdx.x * 256 + threadIdx.x;
    if (m >= J)
        return;
    double mx = 0.0;
    bool x_const = true;
    for (int v = 0; v < V; ++v) {
        mx += task_values[(size_t)v * J + m];
        x_const = x_const && task_values[(size_t)v * J + m] == task_values[m];
    }
    mx /= (double)V;
    double sxx = 0.0;
    for (int v = 0; v < V; ++v) {
        const double d = task_values[(size_t)v * J + m] - mx;
        sxx += d * d;
    }
    const double inv = (!x_const && sxx > 0.0) ? 1.0 / sqrt(sxx) : __builtin_nan("");
    for (int v = 0; v < V; ++v)
        Z[(size_t)v * J + m] = (task_values[(size_t)v * J + m] - mx) * inv;
}

// C[a][b] = sum_v Z[v][a] Z[v][b]: the correlation of metrics a and b (NaN if either is constant)
__global__ __launch_bounds__(256) void corr_matrix_kernel(const double *Z, double *C, int V, int J)
{
    const int b = blockIdx.x * 16 + (threadIdx.x & 15);
    const int a = blockIdx.y * 16 + (threadIdx.x >> 4);
    if (a >= J || b >= J)
        return;
    double acc = 0.0;
    for (int v = 0; v < V; ++v)
        acc += Z[(size_t)v * J + a] * Z[(size_t)v * J + b];
    C[(size_t)a * J + b] = acc;
}

}  // namespace

hipError_t launch_pearson(const double *values, const double *runtime, double *r, int n, int V, int J,
                          hipStream_t stream)
{
    hipLaunchKernelGGL(pearson_kernel, dim3((J + 255) / 256, n), dim3(256), 0, stream, values, runtime, r, V, J);
    return hipGetLastError();
}

hipError_t launch_corr_matrix(const double *task_values, double *Z, double *C, int V, int J, hipStream_t stream)
{
    hipLaunchKernelGGL(standardise_kernel, dim3((J + 255) / 256), dim3(256), 0, stream, task_values, Z, V, J);
    hipLaunchKernelGGL(corr_matrix_kernel, dim3((J + 15) / 16, (J + 15) / 16), dim3(256), 0, stream, Z, C, V, J);
    return hipGetLastError();
}

// keep[m] for one task from its J x J correlation matrix: metrics in index order, a metric goes when
// it correlates at |c| >= tau with one already kept.
void metric_greedy_keep(const double *C, int J, double tau, unsigned char *keep)
{
    std::vector<int> kept;
    kept.reserve(J);
    for (int m = 0; m < J; ++m) {
        bool ok = true;
        for (int m2 : kept) {
            const double c = C[(size_t)m * J + m2];
            if (!std::isnan(c) && std::fabs(c) >= tau) {
                ok = false;
                break;
            }
        }
        keep[m] = ok ? 1 : 0;
        if (ok)
            kept.push_back(m);
    }
}

// Steps after the correlations, on the host.  r [n][J]; keep [n][J] or null (all kept).
// top [n][k] (-1 padded), score [J], selected [J] (0/1), *threshold; each output optional.
void metric_select_host(const double *r, const unsigned char *keep, int n, int J, int k, double q,
                        int min_tasks, int *top, double *score, unsigned char *selected, double *threshold)
{
    std::vector<int> tops((size_t)n * k, -1);
    std::vector<int> in_top((size_t)n * J, 0);
    std::vector<int> cand;
    for (int i = 0; i < n; ++i) {
        const double *ri = r + (size_t)i * J;
        cand.clear();
        for (int m = 0; m < J; ++m)
            if ((!keep || keep[(size_t)i * J + m]) && !std::isnan(ri[m]))
                cand.push_back(m);
        std::sort(cand.begin(), cand.end(), [ri](int a, int b) {
            const double fa = std::fabs(ri[a]), fb = std::fabs(ri[b]);
            return fa > fb || (fa == fb && a < b);
        });
        for (int j = 0; j < k && j < (int)cand.size(); ++j) {
            tops[(size_t)i * k + j] = cand[j];
            in_top[(size_t)i * J + cand[j]] = 1;
        }
    }
    std::vector<double> S(J, 0.0);
    for (int m = 0; m < J; ++m) {
        double acc = 0.0;
        for (int i = 0; i < n; ++i) {
            const double v = r[(size_t)i * J + m];
            acc += std::isnan(v) ? 0.0 : std::fabs(v);
        }
        S[m] = acc / (double)n;
    }
    std::vector<double> cs;
    for (int m = 0; m < J; ++m) {
        bool c = false;
        for (int i = 0; i < n && !c; ++i)
            c = in_top[(size_t)i * J + m] != 0;
        if (c)
            cs.push_back(S[m]);
    }
    double cut = std::nan("");
    if (!cs.empty()) {
        std::sort(cs.begin(), cs.end());
        const double pos = (double)(cs.size() - 1) * q / 100.0;
        const size_t lo = (size_t)std::floor(pos);
        const size_t hi = lo + 1 < cs.size() ? lo + 1 : cs.size() - 1;
        cut = cs[lo] + (pos - (double)lo) * (cs[hi] - cs[lo]);
    }
    if (selected) {
        for (int m = 0; m < J; ++m) {
            int count = 0;
            bool pos_seen = false, neg_seen = false, zero_seen = false;
            for (int i = 0; i < n; ++i) {
                if (!in_top[(size_t)i * J + m])
                    continue;
                ++count;
                const double v = r[(size_t)i * J + m];
                if (v > 0.0)
                    pos_seen = true;
                else if (v < 0.0)
                    neg_seen = true;
                else
                    zero_seen = true;
            }
            const int kinds = (pos_seen ? 1 : 0) + (neg_seen ? 1 : 0) + (zero_seen ? 1 : 0);
            selected[m] = (count >= min_tasks && count > 0 && kinds == 1 && S[m] > cut) ? 1 : 0;
        }
    }
    if (top)
        std::copy(tops.begin(), tops.end(), top);
    if (score)
        std::copy(S.begin(), S.end(), score);
    if (threshold)
        *threshold = cut;
}

}  // namespace ff
