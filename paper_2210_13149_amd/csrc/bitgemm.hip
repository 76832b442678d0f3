// Kernel 2: binary matrix product  c_ij = K - 2*popcount(a_i xor b_j)  with the fused
// rescale  zeta_ij = beta_i * alpha_j * c_ij  (Sec. 4.2.3: XNOR + bit count in place of the
// floating-point inner product of two +-1 vectors).
//
// Mapping (wave64, integer VALU path): lane l of a wavefront owns output columns
// l, l+64, ..., l+64(V-1); the packed rows of B for the workgroup's column block live in
// LDS as [word][column] so that a wavefront reads 512 contiguous bytes per access; the
// wavefront walks R rows of A at a time, and because all 64 lanes work on the same row of
// A its words are wave-uniform (scalar loads, XOR with a scalar operand).  Per 64 binary
// multiply-accumulates a lane issues two v_xor_b32 and two v_bcnt_u32_b32 (the bit count
// accumulates for free), which is the integer-VALU roofline of the operation.
#include "bigcn_internal.h"

namespace bigcn {

// ---- epilogues ---------------------------------------------------------------------------
// Public entry point: int32 accumulators and / or rescaled fp32, row-major.
struct EpilogueApi {
    const float *a_scale;
    const float *b_scale;
    int32_t *acc;
    int64_t ld_acc;
    float *out;
    int64_t ld_out;
    template <int V>
    __device__ __forceinline__ void store(int64_t row, int col0, int lane, int n, const int (&c)[V]) const
    {
        const float sa = out != nullptr ? a_scale[row] : 0.0f;
#pragma unroll
        for (int v = 0; v < V; ++v) {
            const int j = col0 + lane + 64 * v;
            if (j < n) {
                if (acc != nullptr) acc[row * ld_acc + j] = c[v];
                if (out != nullptr) out[row * ld_out + j] = sa * b_scale[j] * static_cast<float>(c[v]);
            }
        }
    }
};

// Fused forward: the integer products of a node in a RowLayout (fp16 or fp32 storage).
template <typename T>
struct EpilogueLayout {
    T *rows;
    int groups;      // RowLayout::groups
    int vec;         // RowLayout::vec
    template <int V>
    __device__ __forceinline__ void store(int64_t row, int col0, int lane, int n, const int (&c)[V]) const
    {
        const int positions = groups * vec;
        T *dst = rows + row * positions;
        if (groups == 64 && vec == V && col0 == 0) {
            // this lane's V columns l, l+64, ... are V consecutive stored values
            T tmp[V];
#pragma unroll
            for (int v = 0; v < V; ++v)
                tmp[v] = (lane + 64 * v < n) ? static_cast<T>(static_cast<float>(c[v])) : static_cast<T>(0.0f);
            T *p = dst + lane * V;
            if constexpr (sizeof(T) * V == 8) {
                *reinterpret_cast<uint2 *>(p) = *reinterpret_cast<const uint2 *>(tmp);
            } else if constexpr (sizeof(T) * V == 16) {
                *reinterpret_cast<uint4 *>(p) = *reinterpret_cast<const uint4 *>(tmp);
            } else {
#pragma unroll
                for (int v = 0; v < V; ++v) p[v] = tmp[v];
            }
        } else {
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const int j = col0 + lane + 64 * v;
                if (j < positions) {
                    const int pos = (j % groups) * vec + j / groups;
                    dst[pos] = j < n ? static_cast<T>(static_cast<float>(c[v])) : static_cast<T>(0.0f);
                }
            }
        }
    }
};

// ---- the kernel -----------------------------------------------------------------------------
// grid.x walks row blocks (grid-stride), grid.y is the column block of 64*V columns.
template <int V, int R, class Epilogue>
__global__ __launch_bounds__(kBlock) void bitgemm_kernel(
    const uint64_t *__restrict__ a, int64_t m, int64_t lda, const uint64_t *__restrict__ b, int n,
    int64_t ldb, int k_bits, Epilogue epi)
{
    extern __shared__ uint64_t lds_b[];          // [n_words][64*V]
    constexpr int CB = 64 * V;
    const int n_words = (k_bits + 63) >> 6;
    const int col0 = blockIdx.y * CB;

    for (int idx = threadIdx.x; idx < CB * n_words; idx += kBlock) {
        const int c = idx / n_words;
        const int w = idx - c * n_words;
        const int j = col0 + c;
        lds_b[w * CB + c] = j < n ? b[static_cast<int64_t>(j) * ldb + w] : 0ull;
    }
    __syncthreads();
    const uint2 *lds_b2 = reinterpret_cast<const uint2 *>(lds_b);

    const int lane = lane_id();
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * kWavesPerBlock + wave_in_block();
    const int64_t n_waves = static_cast<int64_t>(gridDim.x) * kWavesPerBlock;

    for (int64_t row0 = wave * R; row0 < m; row0 += n_waves * R) {
        int pop[R][V];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int v = 0; v < V; ++v) pop[r][v] = 0;

        const uint32_t *arow[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int64_t row = row0 + r < m ? row0 + r : m - 1;   // clamp: tail rows recompute the last row
            arow[r] = reinterpret_cast<const uint32_t *>(a + row * lda);
        }
        // WC words of every row of A are fetched together (wave-uniform: scalar loads), then
        // combined with the lane's columns of B; 32-bit halves so that each half costs exactly
        // one XOR and one accumulating bit count.
        constexpr int WC = 2;
        int w = 0;
        for (; w + WC <= n_words; w += WC) {
            uint32_t aw[R][2 * WC];
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int q = 0; q < 2 * WC; ++q) aw[r][q] = arow[r][2 * w + q];
#pragma unroll
            for (int u = 0; u < WC; ++u) {
                uint2 bw[V];
#pragma unroll
                for (int v = 0; v < V; ++v) bw[v] = lds_b2[(w + u) * CB + lane + 64 * v];
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int v = 0; v < V; ++v) {
                        pop[r][v] = __popc(aw[r][2 * u] ^ bw[v].x) + pop[r][v];
                        pop[r][v] = __popc(aw[r][2 * u + 1] ^ bw[v].y) + pop[r][v];
                    }
            }
        }
        for (; w < n_words; ++w) {
            uint2 bw[V];
#pragma unroll
            for (int v = 0; v < V; ++v) bw[v] = lds_b2[w * CB + lane + 64 * v];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const uint32_t lo = arow[r][2 * w], hi = arow[r][2 * w + 1];
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    pop[r][v] = __popc(lo ^ bw[v].x) + pop[r][v];
                    pop[r][v] = __popc(hi ^ bw[v].y) + pop[r][v];
                }
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (row0 + r >= m) break;                               // wave-uniform
            int c[V];
#pragma unroll
            for (int v = 0; v < V; ++v) c[v] = k_bits - 2 * pop[r][v];
            epi.template store<V>(row0 + r, col0, lane, n, c);
        }
    }
}

template <int V, int R, class Epilogue>
static int launch_bitgemm(const uint64_t *a, int64_t m, int64_t lda, const uint64_t *b, int64_t n,
                          int64_t ldb, int64_t k_bits, const Epilogue &epi, hipStream_t stream)
{
    const int n_words = static_cast<int>((k_bits + 63) / 64);
    const size_t lds = static_cast<size_t>(64) * V * n_words * sizeof(uint64_t);
    const int col_blocks = static_cast<int>((n + 64 * V - 1) / (64 * V));
    // every workgroup stages its B block once: give each at least 16 row blocks per wave
    int64_t row_blocks = (m + R - 1) / R;
    int64_t blocks = (row_blocks + kWavesPerBlock * 16 - 1) / (kWavesPerBlock * 16);
    const int64_t cap = 256 * 8;
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL((bitgemm_kernel<V, R, Epilogue>), dim3(static_cast<unsigned>(blocks), col_blocks),
                       dim3(kBlock), lds, stream, a, m, lda, b, static_cast<int>(n), ldb,
                       static_cast<int>(k_bits), epi);
    return check_launch();
}

// Columns per workgroup are limited by the 64 KB of LDS a workgroup may use:
// 64 * V * n_words * 8 bytes <= 65536  <=>  V * n_words <= 128.
template <class Epilogue>
static int dispatch_bitgemm(int v_wanted, const uint64_t *a, int64_t m, int64_t lda, const uint64_t *b,
                            int64_t n, int64_t ldb, int64_t k_bits, const Epilogue &epi,
                            hipStream_t stream)
{
    const int n_words = static_cast<int>((k_bits + 63) / 64);
    int v = v_wanted;
    while (v > 1 && v * n_words > 128) v >>= 1;
    if (v >= 8) return launch_bitgemm<8, 2>(a, m, lda, b, n, ldb, k_bits, epi, stream);
    if (v >= 4) return launch_bitgemm<4, 4>(a, m, lda, b, n, ldb, k_bits, epi, stream);
    if (v >= 2) return launch_bitgemm<2, 4>(a, m, lda, b, n, ldb, k_bits, epi, stream);
    return launch_bitgemm<1, 4>(a, m, lda, b, n, ldb, k_bits, epi, stream);
}

static int columns_per_lane(int64_t n)
{
    const int64_t v = (n + 63) / 64;
    return v >= 8 ? 8 : (v >= 3 ? 4 : (v == 2 ? 2 : 1));
}

int launch_bitgemm_layout(const uint64_t *a_bits, int64_t m, int64_t lda, const uint64_t *b_bits,
                          int64_t n, int64_t ldb, int64_t k_bits, void *c_rows, RowLayout layout,
                          hipStream_t stream)
{
    if (m == 0 || n == 0) return BIGCN_OK;
    // with 64 groups the kernel's lane -> column map equals the layout's: use its vec
    const int v = layout.groups == 64 ? layout.vec : columns_per_lane(layout.positions());
    if (layout.half) {
        EpilogueLayout<__half> epi{static_cast<__half *>(c_rows), layout.groups, layout.vec};
        return dispatch_bitgemm(v, a_bits, m, lda, b_bits, n, ldb, k_bits, epi, stream);
    }
    EpilogueLayout<float> epi{static_cast<float *>(c_rows), layout.groups, layout.vec};
    return dispatch_bitgemm(v, a_bits, m, lda, b_bits, n, ldb, k_bits, epi, stream);
}

}  // namespace bigcn

extern "C" int bigcn_binary_gemm(const uint64_t *a_bits, const float *a_scale, int64_t m,
                                 int64_t lda_words, const uint64_t *b_bits, const float *b_scale,
                                 int64_t n, int64_t ldb_words, int64_t k_bits, int32_t *acc,
                                 int64_t ld_acc, float *out, int64_t ld_out, void *stream)
{
    if (a_bits == nullptr || b_bits == nullptr) return BIGCN_ENULL;
    if (acc == nullptr && out == nullptr) return BIGCN_ENULL;
    if (out != nullptr && (a_scale == nullptr || b_scale == nullptr)) return BIGCN_ENULL;
    if (m < 0 || n < 0 || k_bits <= 0) return BIGCN_EINVAL;
    const int64_t n_words = (k_bits + 63) / 64;
    if (lda_words < n_words || ldb_words < n_words) return BIGCN_EINVAL;
    if (acc != nullptr && ld_acc < n) return BIGCN_EINVAL;
    if (out != nullptr && ld_out < n) return BIGCN_EINVAL;
    if (n > INT32_MAX) return BIGCN_EINVAL;
    if (k_bits > BIGCN_MAX_K_BITS) return BIGCN_ESHAPE;
    if (m == 0 || n == 0) return BIGCN_OK;
    bigcn::EpilogueApi epi{a_scale, b_scale, acc, ld_acc, out, ld_out};
    return bigcn::dispatch_bitgemm(bigcn::columns_per_lane(n), a_bits, m, lda_words, b_bits, n,
                                   ldb_words, k_bits, epi, bigcn::as_stream(stream));
}
