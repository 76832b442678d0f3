// Steps on either side of the layer path:
//   * column statistics of an fp32 matrix, turned into the frozen standardisation parameters
//     (shift = mean, mul = 1/sqrt(var + eps)) that the binarise+pack step takes as inputs
//     (Sec. 4.4, first step of the general binarisation recipe; Sec. 7.2 Setups);
//   * prediction from the last layer's output: softmax over the classes and the index of the
//     largest entry (Sec. 3.2).
// Both are streaming passes bound by reading their input once.
#include "bigcn_internal.h"

namespace bigcn {

constexpr int kStatsTile = kWave;       // columns per lane slot: one per lane
constexpr int kStatsMaxTiles = 4;       // a workgroup covers up to 4 tiles = 256 columns of its rows
constexpr int kStatsLoads = 8;          // loads in flight per wavefront

static int stats_tiles_per_group(int64_t cols)
{
    const int64_t tiles = (cols + kStatsTile - 1) / kStatsTile;
    return tiles >= kStatsMaxTiles ? kStatsMaxTiles : static_cast<int>(tiles);
}

static int64_t stats_groups(int64_t cols)
{
    const int64_t span = static_cast<int64_t>(stats_tiles_per_group(cols)) * kStatsTile;
    return (cols + span - 1) / span;
}

static int64_t stats_chunks(int64_t rows, int64_t cols)
{
    const int64_t groups = stats_groups(cols);
    int64_t chunks = (2048 + groups - 1) / groups;               // about 2048 workgroups in all
    const int64_t max_chunks = (rows + kWavesPerBlock * kStatsLoads - 1) / (kWavesPerBlock * kStatsLoads);
    if (chunks > max_chunks) chunks = max_chunks;
    return chunks < 1 ? 1 : chunks;
}

// Workgroup (column group, chunk): sums of (x - pivot) and (x - pivot)^2 over the chunk's rows
// for NT * 64 columns, in fp64; lane l owns columns base + l, base + 64 + l, ...  so a wavefront
// reads NT * 256 contiguous bytes of each row (a narrow matrix is read by one workgroup per row
// chunk, never by two that would fetch the same cache lines into different L2s).
// pivot = the column's value in row 0: it keeps the later subtraction E[y^2] - E[y]^2 well
// conditioned when a column's mean is large against its spread.
template <int NT>
__global__ __launch_bounds__(kBlock) void column_partial_kernel(const float *__restrict__ x, int64_t rows,
                                                                int cols, int64_t ld, int64_t rows_per_chunk,
                                                                double *__restrict__ partial)
{
    constexpr int RU = kStatsLoads / NT;      // rows in flight per wavefront
    __shared__ double red[kWavesPerBlock - 1][2 * NT][kWave];
    const int lane = lane_id();
    const int wave = wave_in_block();
    const int c0 = blockIdx.x * (NT * kStatsTile) + lane;
    const int64_t r0 = static_cast<int64_t>(blockIdx.y) * rows_per_chunk;
    const int64_t r1 = r0 + rows_per_chunk < rows ? r0 + rows_per_chunk : rows;
    bool in[NT];
    float pivot[NT];
    double s[NT], ss[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        in[t] = c0 + t * kStatsTile < cols;
        pivot[t] = in[t] ? x[c0 + t * kStatsTile] : 0.0f;
        s[t] = 0.0;
        ss[t] = 0.0;
    }
    for (int64_t r = r0 + wave * RU; r < r1; r += kWavesPerBlock * RU) {
        float v[RU][NT];
#pragma unroll
        for (int u = 0; u < RU; ++u)
#pragma unroll
            for (int t = 0; t < NT; ++t)
                v[u][t] = (in[t] && r + u < r1) ? x[(r + u) * ld + c0 + t * kStatsTile] : pivot[t];
#pragma unroll
        for (int u = 0; u < RU; ++u)
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const double y = static_cast<double>(v[u][t]) - static_cast<double>(pivot[t]);
                s[t] += y;
                ss[t] = fma(y, y, ss[t]);
            }
    }
    if (wave > 0) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            red[wave - 1][2 * t][lane] = s[t];
            red[wave - 1][2 * t + 1][lane] = ss[t];
        }
    }
    __syncthreads();
    if (wave == 0) {
        double *dst = partial + static_cast<int64_t>(blockIdx.y) * 2 * cols;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            if (!in[t]) continue;
#pragma unroll
            for (int w = 0; w < kWavesPerBlock - 1; ++w) {
                s[t] += red[w][2 * t][lane];
                ss[t] += red[w][2 * t + 1][lane];
            }
            dst[c0 + t * kStatsTile] = s[t];
            dst[cols + c0 + t * kStatsTile] = ss[t];
        }
    }
}

// Workgroup per 64 columns: wavefront w sums the partials of chunks w, w + 4, ... (eight loads
// in flight), the four wavefront sums are combined in order, then mean and biased variance.
__global__ __launch_bounds__(kBlock) void column_finish_kernel(const float *__restrict__ x, int64_t rows, int cols,
                                                               const double *__restrict__ partial, int64_t chunks,
                                                               double eps, float *__restrict__ shift,
                                                               float *__restrict__ mul)
{
    constexpr int U = 8;
    __shared__ double red[kWavesPerBlock - 1][2][kWave];
    const int lane = lane_id();
    const int wave = wave_in_block();
    const int c = blockIdx.x * kStatsTile + lane;
    const bool in = c < cols;
    double s = 0.0, ss = 0.0;
    for (int64_t k0 = wave; k0 < chunks; k0 += kWavesPerBlock * U) {
        double a[U], b[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t k = k0 + static_cast<int64_t>(u) * kWavesPerBlock;
            const bool have = in && k < chunks;
            a[u] = have ? partial[k * 2 * cols + c] : 0.0;
            b[u] = have ? partial[k * 2 * cols + cols + c] : 0.0;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            s += a[u];
            ss += b[u];
        }
    }
    if (wave > 0) {
        red[wave - 1][0][lane] = s;
        red[wave - 1][1][lane] = ss;
    }
    __syncthreads();
    if (wave != 0 || !in) return;
#pragma unroll
    for (int w = 0; w < kWavesPerBlock - 1; ++w) {
        s += red[w][0][lane];
        ss += red[w][1][lane];
    }
    const double inv_n = 1.0 / static_cast<double>(rows);
    const double mean_y = s * inv_n;
    double var = ss * inv_n - mean_y * mean_y;
    if (var < 0.0) var = 0.0;
    shift[c] = static_cast<float>(static_cast<double>(x[c]) + mean_y);
    mul[c] = static_cast<float>(1.0 / sqrt(var + eps));
}

// Prediction, 64 classes or more: G lanes share one row (lane g takes classes g, g + G, ...).
// Among equal maxima the lowest class index wins.
// kOneLoad: d <= G, every lane holds at most one class; R such loads are issued back to back.
template <int G, int R, bool kOneLoad>
__global__ __launch_bounds__(kBlock) void predict_kernel(const float *__restrict__ logits, int64_t n, int d,
                                                         int64_t ld, int32_t *__restrict__ labels,
                                                         float *__restrict__ probs, int64_t ld_probs)
{
    constexpr int S = kWave / G;
    const int lane = lane_id();
    const int g = lane & (G - 1);
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * kWavesPerBlock + wave_in_block();
    const int64_t n_waves = static_cast<int64_t>(gridDim.x) * kWavesPerBlock;
    for (int64_t row0 = wave * (S * R); row0 < n; row0 += n_waves * (S * R)) {
        float first[R];
        if (kOneLoad) {
#pragma unroll
            for (int u = 0; u < R; ++u) {
                const int64_t row = row0 + u * S + lane / G;
                first[u] = (row < n && g < d) ? logits[row * ld + g] : -INFINITY;
            }
        }
#pragma unroll
        for (int u = 0; u < R; ++u) {
            const int64_t row = row0 + u * S + lane / G;
            const bool live = row < n;
            const float *src = logits + (live ? row : 0) * ld;
            float best = -INFINITY;
            int arg = d;                         // past the end: loses every tie
            if (kOneLoad) {
                if (g < d) { best = first[u]; arg = g; }
            } else {
                for (int c = g; c < d; c += G) {
                    const float v = src[c];
                    if (v > best || arg == d) { best = v; arg = c; }
                }
            }
#pragma unroll
            for (int off = 1; off < G; off <<= 1) {
                const float ob = __shfl_xor(best, off, kWave);
                const int oa = __shfl_xor(arg, off, kWave);
                if (oa < d && (arg == d || ob > best || (ob == best && oa < arg))) { best = ob; arg = oa; }
            }
            if (live && g == 0 && labels != nullptr) labels[row] = arg;
            if (probs == nullptr) continue;      // uniform over the grid
            float e = 0.0f, sum = 0.0f;
            if (kOneLoad) {
                e = (live && g < d) ? expf(first[u] - best) : 0.0f;
                sum = e;
            } else {
                for (int c = g; c < d; c += G) sum += expf(src[c] - best);
            }
#pragma unroll
            for (int off = 1; off < G; off <<= 1) sum += __shfl_xor(sum, off, kWave);
            const float inv = 1.0f / sum;
            if (!live) continue;
            if (kOneLoad) {
                if (g < d) probs[row * ld_probs + g] = e * inv;
            } else {
                for (int c = g; c < d; c += G) probs[row * ld_probs + c] = expf(src[c] - best) * inv;
            }
        }
    }
}

// Fewer than 64 classes: a workgroup stages 256 rows in LDS (one row per load instruction of a
// wavefront, eight in flight), then every thread scans its own row.  The LDS row stride is odd,
// so the 64 lanes of a wavefront hit distinct banks.  Per row this costs a few instructions per
// class on ONE lane, where the lanes-per-row form spends a butterfly of shuffles per row.
constexpr int kPredictRows = kBlock;

__global__ __launch_bounds__(kBlock) void predict_small_kernel(const float *__restrict__ logits, int64_t n, int d,
                                                               int64_t ld, int32_t *__restrict__ labels,
                                                               float *__restrict__ probs, int64_t ld_probs)
{
    extern __shared__ float tile[];                 // kPredictRows * stride floats
    const int stride = d | 1;
    const int lane = lane_id();
    const int wave = wave_in_block();
    const int64_t row0 = static_cast<int64_t>(blockIdx.x) * kPredictRows;
    const int64_t left = n - row0;
    const int rows_here = left < kPredictRows ? static_cast<int>(left) : kPredictRows;
    constexpr int U = 8;
    const bool col_in = lane < d;
    // stage: wavefront w takes rows 64 w .. 64 w + 63 of the tile
    for (int r0 = wave * kWave; r0 < wave * kWave + kWave; r0 += U) {
        float v[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
            v[u] = (col_in && r0 + u < rows_here) ? logits[(row0 + r0 + u) * ld + lane] : 0.0f;
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (col_in) tile[(r0 + u) * stride + lane] = v[u];
    }
    __syncthreads();
    // scan: thread t owns row t of the tile
    const int t = static_cast<int>(threadIdx.x);
    float *mine = tile + t * stride;
    float best = mine[0];
    int arg = 0;
    for (int c = 1; c < d; ++c) {
        const float v = mine[c];
        if (v > best) { best = v; arg = c; }
    }
    if (t < rows_here && labels != nullptr) labels[row0 + t] = arg;
    if (probs == nullptr) return;                   // uniform over the grid
    float sum = 0.0f;
    for (int c = 0; c < d; ++c) {
        const float e = expf(mine[c] - best);
        mine[c] = e;
        sum += e;
    }
    const float inv = 1.0f / sum;
    for (int c = 0; c < d; ++c) mine[c] *= inv;
    __syncthreads();
    for (int r0 = wave * kWave; r0 < wave * kWave + kWave; r0 += U) {
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (col_in && r0 + u < rows_here) probs[(row0 + r0 + u) * ld_probs + lane] = tile[(r0 + u) * stride + lane];
    }
}

}  // namespace bigcn

using namespace bigcn;

extern "C" size_t bigcn_column_stats_workspace_bytes(int64_t rows, int64_t cols)
{
    if (rows <= 0 || cols <= 0 || cols > (static_cast<int64_t>(1) << 24)) return 0;
    return static_cast<size_t>(stats_chunks(rows, cols)) * 2 * static_cast<size_t>(cols) * sizeof(double);
}

extern "C" int bigcn_column_stats(const float *x, int64_t rows, int64_t cols, int64_t ld, double eps,
                                  float *shift, float *mul, void *workspace, size_t workspace_bytes,
                                  void *stream)
{
    if (x == nullptr || shift == nullptr || mul == nullptr) return BIGCN_ENULL;
    if (rows <= 0 || cols <= 0 || ld < cols || !(eps >= 0.0)) return BIGCN_EINVAL;
    if (cols > (static_cast<int64_t>(1) << 24)) return BIGCN_ESHAPE;
    const size_t need = bigcn_column_stats_workspace_bytes(rows, cols);
    if (workspace == nullptr || workspace_bytes < need || reinterpret_cast<uintptr_t>(workspace) % 8 != 0)
        return BIGCN_EWORKSPACE;
    hipStream_t s = as_stream(stream);
    const int64_t chunks = stats_chunks(rows, cols);
    const int64_t rows_per_chunk = (rows + chunks - 1) / chunks;
    const dim3 grid(static_cast<unsigned>(stats_groups(cols)), static_cast<unsigned>(chunks));
    double *partial = static_cast<double *>(workspace);
#define BIGCN_STATS_CASE(NT)                                                                            \
    case NT:                                                                                            \
        hipLaunchKernelGGL(column_partial_kernel<NT>, grid, dim3(kBlock), 0, s, x, rows,               \
                           static_cast<int>(cols), ld, rows_per_chunk, partial);                        \
        break
    switch (stats_tiles_per_group(cols)) {
        BIGCN_STATS_CASE(1);
        BIGCN_STATS_CASE(2);
        BIGCN_STATS_CASE(3);
        BIGCN_STATS_CASE(4);
    default:
        return BIGCN_EINVAL;
    }
#undef BIGCN_STATS_CASE
    if (hipGetLastError() != hipSuccess) return BIGCN_EHIP;
    hipLaunchKernelGGL(column_finish_kernel, dim3(static_cast<unsigned>((cols + kStatsTile - 1) / kStatsTile)),
                       dim3(kBlock), 0, s, x, rows, static_cast<int>(cols), partial, chunks, eps, shift, mul);
    return check_launch();
}

extern "C" int bigcn_predict(const float *logits, int64_t n, int64_t d, int64_t ld, int32_t *labels,
                             float *probs, int64_t ld_probs, void *stream)
{
    if (logits == nullptr || (labels == nullptr && probs == nullptr)) return BIGCN_ENULL;
    if (n < 0 || d <= 0 || ld < d || (probs != nullptr && ld_probs < d)) return BIGCN_EINVAL;
    if (d > (1 << 20) || n > (static_cast<int64_t>(1) << 38)) return BIGCN_ESHAPE;
    if (n == 0) return BIGCN_OK;
    if (d < kWave) {
        const size_t lds = static_cast<size_t>(kPredictRows) * (d | 1) * sizeof(float);    // < 64 KB
        hipLaunchKernelGGL(predict_small_kernel, dim3(static_cast<unsigned>((n + kPredictRows - 1) / kPredictRows)),
                           dim3(kBlock), lds, as_stream(stream), logits, n, static_cast<int>(d), ld, labels, probs,
                           ld_probs);
        return check_launch();
    }
    // 64 classes or more: all 64 lanes share a row
    constexpr int kRowsInFlight = 8;
    const bool one_load = d == kWave;
    const int64_t rows_per_block = static_cast<int64_t>(kWavesPerBlock) * (one_load ? kRowsInFlight : 1);
    int64_t blocks = (n + rows_per_block - 1) / rows_per_block;
    if (blocks > 256 * 64) blocks = 256 * 64;
    hipStream_t s = as_stream(stream);
    if (one_load)
        hipLaunchKernelGGL((predict_kernel<kWave, kRowsInFlight, true>), dim3(static_cast<unsigned>(blocks)),
                           dim3(kBlock), 0, s, logits, n, static_cast<int>(d), ld, labels, probs, ld_probs);
    else
        hipLaunchKernelGGL((predict_kernel<kWave, 1, false>), dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0,
                           s, logits, n, static_cast<int>(d), ld, labels, probs, ld_probs);
    return check_launch();
}
