// Entropy estimate of a hidden layer by binning (Sec. 6.2): every neuron (column of an fp32
// activation matrix, one row per node) is discretised into `bins` equal-width intervals over
// its own [min, max]; H^(h_i) = - sum_m p_m log2 p_m with p_m = count_m / N, and the layer's
// estimate is the sum over its neurons.
//
// Three streaming steps: column minima / maxima (order-independent atomics on an order-preserving
// integer image of the floats), per-column histograms (workgroup-private counters in LDS, flushed
// with integer atomics: exact and order-independent), entropies in fp64.
#include "bigcn_internal.h"

namespace bigcn {

constexpr int kEntropyTile = 8;            // columns per histogram workgroup
constexpr int kEntropyMaxBins = 1024;

// Order-preserving map float -> uint32 (and back): a < b  <=>  key(a) < key(b).
__device__ __forceinline__ uint32_t float_key(float x)
{
    const uint32_t u = __float_as_uint(x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_float(uint32_t k)
{
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

__global__ __launch_bounds__(kBlock) void entropy_init_kernel(uint32_t *__restrict__ lo_key, uint32_t *__restrict__ hi_key,
                                                              int cols, uint32_t *__restrict__ counts, int64_t n_counts)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i < cols) {
        lo_key[i] = 0xffffffffu;
        hi_key[i] = 0u;
    }
    if (i < n_counts) counts[i] = 0u;
}

// Workgroup (64-column tile, row chunk): lane = column.
__global__ __launch_bounds__(kBlock) void entropy_range_kernel(const float *__restrict__ h, int64_t rows, int cols,
                                                               int64_t ld, int64_t rows_per_chunk,
                                                               uint32_t *__restrict__ lo_key,
                                                               uint32_t *__restrict__ hi_key)
{
    const int lane = lane_id();
    const int wave = wave_in_block();
    const int c = blockIdx.x * kWave + lane;
    if (c >= cols) return;
    const int64_t r0 = static_cast<int64_t>(blockIdx.y) * rows_per_chunk;
    const int64_t r1 = r0 + rows_per_chunk < rows ? r0 + rows_per_chunk : rows;
    float lo = INFINITY, hi = -INFINITY;
    constexpr int U = 8;                          // loads in flight per lane
    int64_t r = r0 + wave;
    for (; r + (U - 1) * kWavesPerBlock < r1; r += U * kWavesPerBlock) {
        float v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = h[(r + u * kWavesPerBlock) * ld + c];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            lo = fminf(lo, v[u]);
            hi = fmaxf(hi, v[u]);
        }
    }
    for (; r < r1; r += kWavesPerBlock) {
        const float v = h[r * ld + c];
        lo = fminf(lo, v);
        hi = fmaxf(hi, v);
    }
    if (lo <= hi) {
        atomicMin(&lo_key[c], float_key(lo));
        atomicMax(&hi_key[c], float_key(hi));
    }
}

// Workgroup (8-column tile, row chunk): 64 lanes = 8 rows x 8 columns per load; counters of the
// tile in LDS.  The bin of a value is decided in fp32: min(bins - 1, floor((x - lo) * scale)) with
// scale = bins / (hi - lo), every operation rounded (no contraction is possible in this form).
__global__ __launch_bounds__(kBlock) void entropy_histogram_kernel(const float *__restrict__ h, int64_t rows, int cols,
                                                                   int64_t ld, int64_t rows_per_chunk, int bins,
                                                                   const uint32_t *__restrict__ lo_key,
                                                                   const uint32_t *__restrict__ hi_key,
                                                                   uint32_t *__restrict__ counts)
{
    extern __shared__ uint32_t local[];           // [kEntropyTile][bins]
    for (int i = threadIdx.x; i < kEntropyTile * bins; i += kBlock) local[i] = 0u;
    __syncthreads();
    const int tc = threadIdx.x & (kEntropyTile - 1);
    const int tr = threadIdx.x / kEntropyTile;                  // 0..31
    const int c = blockIdx.x * kEntropyTile + tc;
    const int64_t r0 = static_cast<int64_t>(blockIdx.y) * rows_per_chunk;
    const int64_t r1 = r0 + rows_per_chunk < rows ? r0 + rows_per_chunk : rows;
    if (c < cols) {
        const float lo = key_float(lo_key[c]);
        const float width = key_float(hi_key[c]) - lo;
        const float scale = width > 0.0f ? static_cast<float>(bins) / width : 0.0f;
        uint32_t *mine = local + tc * bins;
        auto count = [&](float v) {
            const float pos = floorf((v - lo) * scale);
            int m = static_cast<int>(pos);
            m = m > bins - 1 ? bins - 1 : (m < 0 ? 0 : m);
            atomicAdd(&mine[m], 1u);
        };
        constexpr int U = 8;                      // loads in flight per lane
        constexpr int kStep = kBlock / kEntropyTile;
        int64_t r = r0 + tr;
        for (; r + (U - 1) * kStep < r1; r += U * kStep) {
            float v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) v[u] = h[(r + u * kStep) * ld + c];
#pragma unroll
            for (int u = 0; u < U; ++u) count(v[u]);
        }
        for (; r < r1; r += kStep) count(h[r * ld + c]);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kEntropyTile * bins; i += kBlock) {
        const int col = blockIdx.x * kEntropyTile + i / bins;
        const uint32_t v = local[i];
        if (v != 0u && col < cols) atomicAdd(&counts[static_cast<int64_t>(col) * bins + (i % bins)], v);
    }
}

// One wavefront per column: entropy in bits from the counts; per_neuron[c] (nullable).
__global__ __launch_bounds__(kWave) void entropy_column_kernel(const uint32_t *__restrict__ counts, int bins, int64_t rows,
                                                               double *__restrict__ per_neuron)
{
    const int c = blockIdx.x;
    const int lane = threadIdx.x;
    const double inv_n = 1.0 / static_cast<double>(rows);
    double s = 0.0;
    for (int m = lane; m < bins; m += kWave) {
        const uint32_t k = counts[static_cast<int64_t>(c) * bins + m];
        if (k != 0u) {
            const double p = static_cast<double>(k) * inv_n;
            s -= p * log2(p);
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, kWave);
    if (lane == 0) per_neuron[c] = s;
}

// Sum of the per-neuron entropies in column order (one thread: a few thousand terms at most).
__global__ void entropy_total_kernel(const double *__restrict__ per_neuron, int cols, double *__restrict__ total)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    double s = 0.0;
    for (int c = 0; c < cols; ++c) s += per_neuron[c];
    *total = s;
}

struct EntropyMap {
    size_t lo_off, hi_off, per_off, counts_off, total;
};

static EntropyMap map_entropy(int64_t cols, int bins)
{
    auto up = [](size_t v) { return (v + 255) & ~static_cast<size_t>(255); };
    EntropyMap m;
    size_t off = 0;
    m.lo_off = off;     off = up(off + static_cast<size_t>(cols) * 4);
    m.hi_off = off;     off = up(off + static_cast<size_t>(cols) * 4);
    m.per_off = off;    off = up(off + static_cast<size_t>(cols) * 8);
    m.counts_off = off; off = up(off + static_cast<size_t>(cols) * bins * 4);
    m.total = off;
    return m;
}

}  // namespace bigcn

using namespace bigcn;

extern "C" size_t bigcn_entropy_workspace_bytes(int64_t cols, int bins)
{
    if (cols <= 0 || cols > BIGCN_MAX_K_BITS || bins < 1 || bins > kEntropyMaxBins) return 0;
    return map_entropy(cols, bins).total;
}

extern "C" int bigcn_entropy(const float *h, int64_t rows, int64_t cols, int64_t ld, int bins,
                             double *per_neuron, double *total, uint32_t *counts_out, void *workspace,
                             size_t workspace_bytes, void *stream)
{
    if (h == nullptr || total == nullptr) return BIGCN_ENULL;
    if (rows <= 0 || cols <= 0 || ld < cols || bins < 1) return BIGCN_EINVAL;
    if (cols > BIGCN_MAX_K_BITS || bins > kEntropyMaxBins || rows >= (static_cast<int64_t>(1) << 32)) return BIGCN_ESHAPE;
    const EntropyMap map = map_entropy(cols, bins);
    if (workspace == nullptr || workspace_bytes < map.total || reinterpret_cast<uintptr_t>(workspace) % 256 != 0)
        return BIGCN_EWORKSPACE;
    hipStream_t s = as_stream(stream);
    char *ws = static_cast<char *>(workspace);
    uint32_t *lo_key = reinterpret_cast<uint32_t *>(ws + map.lo_off);
    uint32_t *hi_key = reinterpret_cast<uint32_t *>(ws + map.hi_off);
    double *per = per_neuron != nullptr ? per_neuron : reinterpret_cast<double *>(ws + map.per_off);
    uint32_t *counts = counts_out != nullptr ? counts_out : reinterpret_cast<uint32_t *>(ws + map.counts_off);
    const int64_t n_counts = cols * bins;
    const int icols = static_cast<int>(cols);

    hipLaunchKernelGGL(entropy_init_kernel, dim3(static_cast<unsigned>((n_counts + kBlock - 1) / kBlock)), dim3(kBlock), 0,
                       s, lo_key, hi_key, icols, counts, n_counts);
    if (hipGetLastError() != hipSuccess) return BIGCN_EHIP;
    {
        const int64_t tiles = (cols + kWave - 1) / kWave;
        int64_t chunks = (2048 + tiles - 1) / tiles;
        const int64_t max_chunks = (rows + 63) / 64;
        if (chunks > max_chunks) chunks = max_chunks;
        const int64_t rpc = (rows + chunks - 1) / chunks;
        hipLaunchKernelGGL(entropy_range_kernel, dim3(static_cast<unsigned>(tiles), static_cast<unsigned>(chunks)),
                           dim3(kBlock), 0, s, h, rows, icols, ld, rpc, lo_key, hi_key);
        if (hipGetLastError() != hipSuccess) return BIGCN_EHIP;
    }
    {
        const int64_t tiles = (cols + kEntropyTile - 1) / kEntropyTile;
        int64_t chunks = (4096 + tiles - 1) / tiles;
        const int64_t max_chunks = (rows + 255) / 256;
        if (chunks > max_chunks) chunks = max_chunks;
        if (chunks < 1) chunks = 1;
        const int64_t rpc = (rows + chunks - 1) / chunks;
        const size_t lds = static_cast<size_t>(kEntropyTile) * bins * sizeof(uint32_t);
        hipLaunchKernelGGL(entropy_histogram_kernel, dim3(static_cast<unsigned>(tiles), static_cast<unsigned>(chunks)),
                           dim3(kBlock), lds, s, h, rows, icols, ld, rpc, bins, lo_key, hi_key, counts);
        if (hipGetLastError() != hipSuccess) return BIGCN_EHIP;
    }
    hipLaunchKernelGGL(entropy_column_kernel, dim3(static_cast<unsigned>(cols)), dim3(kWave), 0, s, counts, bins, rows, per);
    if (hipGetLastError() != hipSuccess) return BIGCN_EHIP;
    hipLaunchKernelGGL(entropy_total_kernel, dim3(1), dim3(kWave), 0, s, per, icols, total);
    return check_launch();
}
