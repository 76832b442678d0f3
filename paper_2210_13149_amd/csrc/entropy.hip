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

constexpr int kEntropyTile = 32;           // columns per histogram workgroup (one 128-byte line per row)
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

// Workgroup (tile of NT x 64 columns, row chunk): lane l owns columns base + l, base + 64 + l, ...,
// so a matrix of up to 256 columns is read in whole rows by one workgroup per row chunk (two
// tiles of 64 columns each fetched the lines that straddle their border twice).
template <int NT>
__global__ __launch_bounds__(kBlock) void entropy_range_kernel(const float *__restrict__ h, int64_t rows, int cols,
                                                               int64_t ld, int64_t rows_per_chunk,
                                                               uint32_t *__restrict__ lo_key,
                                                               uint32_t *__restrict__ hi_key)
{
    const int lane = lane_id();
    const int wave = wave_in_block();
    const int c0 = blockIdx.x * (NT * kWave) + lane;
    const int64_t r0 = static_cast<int64_t>(blockIdx.y) * rows_per_chunk;
    const int64_t r1 = r0 + rows_per_chunk < rows ? r0 + rows_per_chunk : rows;
    bool in[NT];
    float lo[NT], hi[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        in[t] = c0 + t * kWave < cols;
        lo[t] = INFINITY;
        hi[t] = -INFINITY;
    }
    constexpr int U = 8 / NT;                     // rows in flight per wavefront (8 loads)
    for (int64_t r = r0 + wave * U; r < r1; r += kWavesPerBlock * U) {
        float v[U][NT];
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int t = 0; t < NT; ++t)
                v[u][t] = (in[t] && r + u < r1) ? h[(r + u) * ld + c0 + t * kWave] : NAN;
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                lo[t] = fminf(lo[t], v[u][t]);    // fminf / fmaxf return the other operand for a NaN
                hi[t] = fmaxf(hi[t], v[u][t]);
            }
    }
#pragma unroll
    for (int t = 0; t < NT; ++t)
        if (in[t] && lo[t] <= hi[t]) {
            atomicMin(&lo_key[c0 + t * kWave], float_key(lo[t]));
            atomicMax(&hi_key[c0 + t * kWave], float_key(hi[t]));
        }
}

// Workgroup (32-column tile, row chunk): 256 threads = 8 rows x 32 columns per load, so every
// row piece is a whole 128-byte line (with 8-column tiles each line crossed the L2 boundary 4.6
// times).  Counters of the tile in LDS, two columns to a 32-bit word (a chunk has at most 65535
// rows, so a column's count never carries into its neighbour's half): 16 x bins words, 64 KB at
// 1024 bins.  The bin of a value is decided in fp32: min(bins - 1, floor((x - lo) * scale)) with
// scale = bins / (hi - lo), every operation rounded (no contraction is possible in this form).
__global__ __launch_bounds__(kBlock) void entropy_histogram_kernel(const float *__restrict__ h, int64_t rows, int cols,
                                                                   int64_t ld, int64_t rows_per_chunk, int bins,
                                                                   const uint32_t *__restrict__ lo_key,
                                                                   const uint32_t *__restrict__ hi_key,
                                                                   uint32_t *__restrict__ counts)
{
    extern __shared__ uint32_t local[];           // [kEntropyTile / 2][bins]
    for (int i = threadIdx.x; i < (kEntropyTile / 2) * bins; i += kBlock) local[i] = 0u;
    __syncthreads();
    const int tc = threadIdx.x & (kEntropyTile - 1);
    const int tr = threadIdx.x / kEntropyTile;                  // 0..7
    const int c = blockIdx.x * kEntropyTile + tc;
    const int64_t r0 = static_cast<int64_t>(blockIdx.y) * rows_per_chunk;
    const int64_t r1 = r0 + rows_per_chunk < rows ? r0 + rows_per_chunk : rows;
    if (c < cols) {
        const float lo = key_float(lo_key[c]);
        const float width = key_float(hi_key[c]) - lo;
        const float scale = width > 0.0f ? static_cast<float>(bins) / width : 0.0f;
        uint32_t *mine = local + (tc >> 1) * bins;
        const uint32_t one = 1u << (16 * (tc & 1));
        auto count = [&](float v) {
            const float pos = floorf((v - lo) * scale);
            int m = static_cast<int>(pos);
            m = m > bins - 1 ? bins - 1 : (m < 0 ? 0 : m);
            atomicAdd(&mine[m], one);
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
    for (int i = threadIdx.x; i < (kEntropyTile / 2) * bins; i += kBlock) {
        const int col = blockIdx.x * kEntropyTile + 2 * (i / bins);
        const uint32_t v = local[i];
        const uint32_t even = v & 0xffffu, odd = v >> 16;
        if (even != 0u && col < cols) atomicAdd(&counts[static_cast<int64_t>(col) * bins + (i % bins)], even);
        if (odd != 0u && col + 1 < cols) atomicAdd(&counts[static_cast<int64_t>(col + 1) * bins + (i % bins)], odd);
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
        const int64_t words = (cols + kWave - 1) / kWave;
        const int nt = words >= 4 ? 4 : static_cast<int>(words);
        const int64_t tiles = (words + nt - 1) / nt;
        int64_t chunks = (2048 + tiles - 1) / tiles;
        const int64_t max_chunks = (rows + 63) / 64;
        if (chunks > max_chunks) chunks = max_chunks;
        const int64_t rpc = (rows + chunks - 1) / chunks;
        const dim3 grid(static_cast<unsigned>(tiles), static_cast<unsigned>(chunks));
        switch (nt) {
        case 1: hipLaunchKernelGGL(entropy_range_kernel<1>, grid, dim3(kBlock), 0, s, h, rows, icols, ld, rpc, lo_key, hi_key); break;
        case 2: hipLaunchKernelGGL(entropy_range_kernel<2>, grid, dim3(kBlock), 0, s, h, rows, icols, ld, rpc, lo_key, hi_key); break;
        case 3: hipLaunchKernelGGL(entropy_range_kernel<3>, grid, dim3(kBlock), 0, s, h, rows, icols, ld, rpc, lo_key, hi_key); break;
        default: hipLaunchKernelGGL(entropy_range_kernel<4>, grid, dim3(kBlock), 0, s, h, rows, icols, ld, rpc, lo_key, hi_key); break;
        }
        if (hipGetLastError() != hipSuccess) return BIGCN_EHIP;
    }
    {
        const int64_t tiles = (cols + kEntropyTile - 1) / kEntropyTile;
        int64_t chunks = (4096 + tiles - 1) / tiles;
        const int64_t max_chunks = (rows + 255) / 256;
        if (chunks > max_chunks) chunks = max_chunks;
        const int64_t min_chunks = (rows + 65534) / 65535;       // 16-bit counters per chunk
        if (chunks < min_chunks) chunks = min_chunks;
        if (chunks < 1) chunks = 1;
        if (chunks > 65535) return BIGCN_ESHAPE;                  // more rows than 65535 chunks of 65535
        const int64_t rpc = (rows + chunks - 1) / chunks;
        const size_t lds = static_cast<size_t>(kEntropyTile / 2) * bins * sizeof(uint32_t);
        hipLaunchKernelGGL(entropy_histogram_kernel, dim3(static_cast<unsigned>(tiles), static_cast<unsigned>(chunks)),
                           dim3(kBlock), lds, s, h, rows, icols, ld, rpc, bins, lo_key, hi_key, counts);
        if (hipGetLastError() != hipSuccess) return BIGCN_EHIP;
    }
    hipLaunchKernelGGL(entropy_column_kernel, dim3(static_cast<unsigned>(cols)), dim3(kWave), 0, s, counts, bins, rows, per);
    if (hipGetLastError() != hipSuccess) return BIGCN_EHIP;
    hipLaunchKernelGGL(entropy_total_kernel, dim3(1), dim3(kWave), 0, s, per, icols, total);
    return check_launch();
}
