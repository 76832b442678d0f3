// Back propagation through one binarised graph-convolution layer (Sec. 4.3, Algorithm 1):
//
//   g_zeta = A~^T g_out                          (aggregation kernel; A~ is symmetric)
//   g_wt   = H~^T g_zeta,   H~ = beta_i F_i      (d_in x d_out, a reduction over the nodes)
//   g_ht   = g_zeta W~^T,   W~ = alpha_j B_j     (n x d_in)
//   g_in   = g_ht 1[|g_ht| < 1] (* mul)          (clipped straight-through rule)
//   g_w    = B_tj (sum_k g_wt[k,j] B_kj) / d_in + alpha_j g_wt[t,j] 1[|W_tj| < 1]
//
// The two dense products have one +-1 operand each.  They run on the fp32 matrix cores
// (v_mfma_f32_32x32x2_f32): the +-1 operand is expanded from packed bits in registers (three
// vector operations per value, hidden behind the 64-cycle multiply), the scales beta / alpha are
// folded into the fp32 operand while it is staged through LDS.
//
// First layer (no input gradient wanted, d_in <= d_out): g_wt = H~^T (A~ g_out) = (A~ H~)^T g_out,
// because A~ is symmetric.  U = A~ H~ gathers packed sign rows (d_in / 8 bytes + one scale per
// neighbour) instead of fp32 gradient rows (4 d_out bytes): the packed word of a neighbour is used
// directly as the lane mask of a conditional add (lane l owns column 64 w + l).
//
// Operand layout of the 32x32x2 multiply, lane l:  A[i = l % 32][k = l / 32],
// B[k = l / 32][j = l % 32]; accumulator register r holds row 8 (r / 4) + 4 (l / 32) + r % 4 and
// column l % 32.
#include "bigcn_internal.h"

namespace bigcn {

typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kStageRows = 64;      // rows (of g_zeta, of the fp32 operand) staged per step

// +1.0f where bit `pos` of `word` is set, else -1.0f.
__device__ __forceinline__ float sign_from_bit(uint32_t word, int pos)
{
    return __uint_as_float(0xbf800000u ^ (((word >> pos) & 1u) << 31));
}

// ---- g_ht = (g_zeta alpha) B^T, clipped, times mul ---------------------------------------------
// Workgroup: 128 rows (four wavefronts x 32) x 128 columns t of the layer input; wavefront: 32
// rows x 4 column tiles.  K runs over the layer's output columns j in steps of 64 (one packed
// word of the weights packed along j): the 128 x 64 slab of g_zeta * alpha_j goes through LDS, the
// +-1 operand B[j][t] is bit j of the lane's own packed weight row t.
__global__ __launch_bounds__(kBlock, 4) void backward_input_kernel(
    const float *__restrict__ g_zeta, int64_t n, int d_out, int64_t ld_gz, const float *__restrict__ alpha,
    const uint64_t *__restrict__ wt_bits, int64_t ld_wt, int d_in, const float *__restrict__ mul,
    float *__restrict__ g_in, int64_t ld_gin)
{
    constexpr int KC = 64;
    __shared__ float slab[128][KC + 1];
    const int lane = lane_id();
    const int wave = wave_in_block();
    const int i32 = lane & 31, half = lane >> 5;
    const int64_t row0 = static_cast<int64_t>(blockIdx.x) * 128;
    const int col0 = blockIdx.y * 128;

    v16f acc[4];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[q][r] = 0.0f;

    int t[4];
    bool t_in[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        t[q] = col0 + 32 * q + i32;
        t_in[q] = t[q] < d_in;
    }

    for (int j0 = 0; j0 < d_out; j0 += KC) {
        // stage g_zeta[row0 .. +128][j0 .. +64] * alpha_j: thread (r = tid / 64 + 4 it, c = tid % 64)
        __syncthreads();
        {
            const int c = threadIdx.x & 63;
            const int j = j0 + c;
            const float a = j < d_out ? alpha[j] : 0.0f;
#pragma unroll 8
            for (int it = 0; it < 32; ++it) {
                const int r = (threadIdx.x >> 6) + 4 * it;
                const int64_t row = row0 + r;
                slab[r][c] = (row < n && j < d_out) ? g_zeta[row * ld_gz + j] * a : 0.0f;
            }
        }
        __syncthreads();
        // this lane's packed weight words for the chunk: bit (j - j0) of word j0 / 64 of row t;
        // pre-shifted by the lane's k offset (l / 32)
        uint32_t lo[4], hi[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint64_t w = t_in[q] ? wt_bits[static_cast<int64_t>(t[q]) * ld_wt + (j0 >> 6)] : 0ull;
            const uint64_t shifted = w >> half;
            lo[q] = static_cast<uint32_t>(shifted);
            hi[q] = static_cast<uint32_t>(shifted >> 32);
        }
        const float *arow = &slab[wave * 32 + i32][half];
#pragma unroll
        for (int s = 0; s < KC / 2; ++s) {
            const float a = arow[2 * s];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                // k = 2 s + half; after the pre-shift it is bit 2 s of the 64-bit word (bit 31 of
                // the low half has moved down from the high half's bit 0 only for half = 1, which
                // the 64-bit shift above already did)
                const float b = s < 16 ? sign_from_bit(lo[q], 2 * s) : sign_from_bit(hi[q], 2 * s - 32);
                acc[q] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[q], 0, 0, 0);
            }
        }
    }
    // epilogue: clipped straight-through rule, optional per-column factor
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if (!t_in[q]) continue;
        const float m = mul != nullptr ? mul[t[q]] : 1.0f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t row = row0 + wave * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
            if (row < n) {
                const float g = acc[q][r];
                g_in[row * ld_gin + t[q]] = (fabsf(g) < 1.0f ? g : 0.0f) * m;
            }
        }
    }
}

// ---- partial g_wt = H~^T g_zeta over a chunk of nodes -------------------------------------------
// Workgroup (chunk, j block of 64, t block of 256): wavefront w owns t = 64 w .. 64 w + 63 (two
// tiles) x two j tiles.  Per step 64 nodes are staged: g_zeta[i][j] * beta_i (fp32, LDS) and the
// packed signs of the nodes' 256 input columns (LDS); operand A[t][i] is bit t of node i.
__global__ __launch_bounds__(kBlock) void backward_weight_partial_kernel(
    const float *__restrict__ g_zeta, int64_t n, int d_out, int64_t ld_gz, const float *__restrict__ beta,
    const uint64_t *__restrict__ f_bits, int64_t ld_f, int d_in, int64_t rows_per_chunk,
    float *__restrict__ partial)
{
    __shared__ float slab[kStageRows][64 + 1];          // [node][j]
    __shared__ uint64_t signs[kStageRows][4 + 1];        // [node][word of the 256-column t block]
    const int lane = lane_id();
    const int wave = wave_in_block();
    const int i32 = lane & 31, half = lane >> 5;
    const int j0 = blockIdx.y * 64;
    const int t0 = blockIdx.z * 256;
    const int64_t i_begin = static_cast<int64_t>(blockIdx.x) * rows_per_chunk;
    const int64_t i_end = i_begin + rows_per_chunk < n ? i_begin + rows_per_chunk : n;

    v16f acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.0f;

    // the lane's two t values, their word inside the 256-column block and bit inside the word
    const int tw = wave;                              // 64 consecutive t per wavefront = one word
    const int bit[2] = {i32, 32 + i32};

    for (int64_t i0 = i_begin; i0 < i_end; i0 += kStageRows) {
        __syncthreads();
        {
            const int c = threadIdx.x & 63;
            const int j = j0 + c;
#pragma unroll 4
            for (int it = 0; it < kStageRows / 4; ++it) {
                const int r = (threadIdx.x >> 6) + 4 * it;
                const int64_t row = i0 + r;
                const bool live = row < i_end && j < d_out;
                slab[r][c] = live ? g_zeta[row * ld_gz + j] * beta[row] : 0.0f;
            }
            // 64 nodes x 4 words: one word per thread
            const int r = threadIdx.x >> 2, w = threadIdx.x & 3;
            const int64_t row = i0 + r;
            const int word = (t0 >> 6) + w;
            signs[r][w] = (row < i_end && word < (d_in + 63) / 64) ? f_bits[row * ld_f + word] : 0ull;
        }
        __syncthreads();
#pragma unroll 4
        for (int s = 0; s < kStageRows / 2; ++s) {
            const int node = 2 * s + half;
            const uint64_t w = signs[node][tw];
            const float b0 = slab[node][i32];
            const float b1 = slab[node][32 + i32];
            const uint32_t wlo = static_cast<uint32_t>(w), whi = static_cast<uint32_t>(w >> 32);
            const float a0 = sign_from_bit(wlo, bit[0]);
            const float a1 = sign_from_bit(whi, bit[1] - 32);
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
        }
    }
    // partial[chunk][t][j]; rows of nodes past i_end contributed zeros (slab = 0)
    float *dst = partial + static_cast<int64_t>(blockIdx.x) * d_in * d_out;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int j = j0 + 32 * b + i32;
            if (j >= d_out) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int t = t0 + 64 * wave + 32 * a + 8 * (r >> 2) + 4 * half + (r & 3);
                if (t < d_in) dst[static_cast<int64_t>(t) * d_out + j] = acc[a][b][r];
            }
        }
}

// ---- U = A~ H~ from packed signs ---------------------------------------------------------------
// U[i][c] = sum_p vals[p] beta_k (2 bit_kc - 1) = 2 P[i][c] - W_i over the neighbours k of node i,
// P = sum over the neighbours whose bit is set, W = sum of all weights.  One wavefront per node
// (plan order); 64 neighbours are fetched at a time, lane j holding neighbour j's weight and its
// NW packed words of this pass (both from the neighbour's record, see sign_records_kernel); the words are broadcast one neighbour at a time and act as the
// lane mask of the add.  Neighbours are added in list order (run-to-run identical).
// records[k] = {packed words of node k (n_words of them), beta_k in the low half of one more word}:
// bits and scale of a neighbour arrive with one gather instead of two.
__global__ __launch_bounds__(kBlock) void sign_records_kernel(const uint64_t *__restrict__ f_bits, int64_t ld_f,
                                                              const float *__restrict__ beta, int64_t n, int n_words,
                                                              uint64_t *__restrict__ records)
{
    const int64_t total = n * (n_words + 1);
    for (int64_t e = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; e < total;
         e += static_cast<int64_t>(gridDim.x) * kBlock) {
        const int64_t row = e / (n_words + 1);
        const int w = static_cast<int>(e - row * (n_words + 1));
        records[e] = w < n_words ? f_bits[row * ld_f + w] : static_cast<uint64_t>(__float_as_uint(beta[row]));
    }
}

template <int NW>
__global__ __launch_bounds__(kBlock) void aggregate_signs_kernel(
    const int32_t *__restrict__ row_order, int64_t n, const int64_t *__restrict__ row_ptr,
    const int32_t *__restrict__ col_idx, const float *__restrict__ vals, const uint64_t *__restrict__ records,
    int d_in, int word0, float *__restrict__ u, int64_t ld_u)
{
    const int lane = lane_id();
    const int64_t entry = static_cast<int64_t>(blockIdx.x) * kWavesPerBlock + wave_in_block();
    if (entry >= n) return;                                    // wave-uniform
    const int64_t row = row_order[entry];
    const int64_t p0 = row_ptr[row], p1 = row_ptr[row + 1];
    const int n_words = (d_in + 63) >> 6;

    float set_sum[NW];
#pragma unroll
    for (int q = 0; q < NW; ++q) set_sum[q] = 0.0f;
    float all_sum = 0.0f;                                      // per-lane partial of W
    for (int64_t pb = p0; pb < p1; pb += kWave) {
        const int cnt = static_cast<int>(p1 - pb < kWave ? p1 - pb : kWave);
        float wk = 0.0f;
        uint32_t lo[NW], hi[NW];
#pragma unroll
        for (int q = 0; q < NW; ++q) { lo[q] = 0u; hi[q] = 0u; }
        if (lane < cnt) {
            const uint64_t *rec = records + static_cast<int64_t>(col_idx[pb + lane]) * (n_words + 1);
            wk = (vals != nullptr ? vals[pb + lane] : 1.0f) * __uint_as_float(static_cast<uint32_t>(rec[n_words]));
#pragma unroll
            for (int q = 0; q < NW; ++q) {
                if (word0 + q < n_words) {
                    const uint64_t word = rec[word0 + q];
                    lo[q] = static_cast<uint32_t>(word);
                    hi[q] = static_cast<uint32_t>(word >> 32);
                }
            }
        }
        all_sum += wk;
        for (int t = 0; t < cnt; ++t) {
            const float wt = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wk), t));
#pragma unroll
            for (int q = 0; q < NW; ++q) {
                const uint64_t mask = static_cast<uint64_t>(static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(lo[q]), t))) |
                                      (static_cast<uint64_t>(static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(hi[q]), t))) << 32);
                set_sum[q] += __builtin_amdgcn_inverse_ballot_w64(mask) ? wt : 0.0f;
            }
        }
    }
    const float total = wave_sum(all_sum);
#pragma unroll
    for (int q = 0; q < NW; ++q) {
        const int c = 64 * (word0 + q) + lane;
        if (c < d_in) u[row * ld_u + c] = fmaf(2.0f, set_sum[q], -total);
    }
}

// ---- partial g_wt = U^T g_out over a chunk of nodes (both operands fp32) --------------------------
// Workgroup (chunk, j block of 64, t block of 128): wavefront w owns t = 32 w .. 32 w + 31 x two
// j tiles.  Per step 32 nodes go through LDS: g_out[i][j] and U[i][t]; the next step's values are
// fetched into registers while the current step is multiplied.
constexpr int kDenseStage = 32;

__global__ __launch_bounds__(kBlock) void backward_weight_dense_partial_kernel(
    const float *__restrict__ g_out, int64_t n, int d_out, int64_t ld_g, const float *__restrict__ u, int64_t ld_u,
    int d_in, int64_t rows_per_chunk, float *__restrict__ partial)
{
    __shared__ float slab[kDenseStage][64 + 1];           // [node][j]
    __shared__ float utile[kDenseStage][128 + 1];         // [node][t]
    const int lane = lane_id();
    const int wave = wave_in_block();
    const int i32 = lane & 31, half = lane >> 5;
    const int j0 = blockIdx.y * 64;
    const int t0 = blockIdx.z * 128;
    const int64_t i_begin = static_cast<int64_t>(blockIdx.x) * rows_per_chunk;
    const int64_t i_end = i_begin + rows_per_chunk < n ? i_begin + rows_per_chunk : n;

    v16f acc[2];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[b][r] = 0.0f;

    // this thread's share of a step: 8 values of g_out (rows gr + 4 it) and 16 of U (rows ur + 2 it)
    const int gc = threadIdx.x & 63, gr = threadIdx.x >> 6;
    const int uc = threadIdx.x & 127, ur = threadIdx.x >> 7;
    const bool g_col_in = j0 + gc < d_out, u_col_in = t0 + uc < d_in;
    float g_next[kDenseStage / 4], u_next[kDenseStage / 2];
    auto fetch = [&](int64_t i0) {
#pragma unroll
        for (int it = 0; it < kDenseStage / 4; ++it) {
            const int64_t row = i0 + gr + 4 * it;
            g_next[it] = (row < i_end && g_col_in) ? g_out[row * ld_g + j0 + gc] : 0.0f;
        }
#pragma unroll
        for (int it = 0; it < kDenseStage / 2; ++it) {
            const int64_t row = i0 + ur + 2 * it;
            u_next[it] = (row < i_end && u_col_in) ? u[row * ld_u + t0 + uc] : 0.0f;
        }
    };
    if (i_begin < i_end) fetch(i_begin);
    for (int64_t i0 = i_begin; i0 < i_end; i0 += kDenseStage) {
        __syncthreads();                                  // every wavefront has left the previous step
#pragma unroll
        for (int it = 0; it < kDenseStage / 4; ++it) slab[gr + 4 * it][gc] = g_next[it];
#pragma unroll
        for (int it = 0; it < kDenseStage / 2; ++it) utile[ur + 2 * it][uc] = u_next[it];
        __syncthreads();
        if (i0 + kDenseStage < i_end) fetch(i0 + kDenseStage);       // in flight during the multiplies
#pragma unroll 4
        for (int s = 0; s < kDenseStage / 2; ++s) {
            const int node = 2 * s + half;
            const float a = utile[node][32 * wave + i32];
            const float b0 = slab[node][i32];
            const float b1 = slab[node][32 + i32];
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b0, acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b1, acc[1], 0, 0, 0);
        }
    }
    float *dst = partial + static_cast<int64_t>(blockIdx.x) * d_in * d_out;
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int j = j0 + 32 * b + i32;
        if (j >= d_out) continue;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int t = t0 + 32 * wave + 8 * (r >> 2) + 4 * half + (r & 3);
            if (t < d_in) dst[static_cast<int64_t>(t) * d_out + j] = acc[b][r];
        }
    }
}

// Rows of d floats copied into rows of dp >= d floats (dp a multiple of 4), the tail zeroed: the
// aggregation reads 16 bytes per lane only from rows that are 16-byte aligned.
__global__ __launch_bounds__(kBlock) void pad_rows_kernel(const float *__restrict__ src, int64_t ld_src, int64_t n,
                                                          int d, int dp, float *__restrict__ dst)
{
    const int64_t total = n * dp;
    for (int64_t e = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; e < total;
         e += static_cast<int64_t>(gridDim.x) * kBlock) {
        const int64_t row = e / dp;
        const int c = static_cast<int>(e - row * dp);
        dst[e] = c < d ? src[row * ld_src + c] : 0.0f;
    }
}

// g_wt[t][j] = sum over chunks (in chunk order, fp64), written as fp32.
__global__ __launch_bounds__(kBlock) void backward_weight_reduce_kernel(const float *__restrict__ partial,
                                                                        int64_t chunks, int64_t elems,
                                                                        float *__restrict__ g_wt)
{
    const int64_t e = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (e >= elems) return;
    double s = 0.0;
    for (int64_t c = 0; c < chunks; ++c) s += static_cast<double>(partial[c * elems + e]);
    g_wt[e] = static_cast<float>(s);
}

// Sec. 4.3, gradient of the full-precision weights: workgroup per column j (64 lanes stride
// over t): column sum of g_wt[t][j] B_tj, then both terms.
__global__ __launch_bounds__(kWave) void backward_weight_finish_kernel(
    const float *__restrict__ g_wt, const float *__restrict__ w, int64_t ld_w, const float *__restrict__ alpha,
    int d_in, int d_out, float *__restrict__ g_w, int64_t ld_gw)
{
    const int j = blockIdx.x;
    const int lane = threadIdx.x;
    double s = 0.0;
    for (int t = lane; t < d_in; t += kWave) {
        const float b = w[static_cast<int64_t>(t) * ld_w + j] >= 0.0f ? 1.0f : -1.0f;
        s += static_cast<double>(g_wt[static_cast<int64_t>(t) * d_out + j]) * b;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, kWave);
    const float column = static_cast<float>(s / static_cast<double>(d_in));
    const float a = alpha[j];
    for (int t = lane; t < d_in; t += kWave) {
        const float wv = w[static_cast<int64_t>(t) * ld_w + j];
        const float b = wv >= 0.0f ? 1.0f : -1.0f;
        const float g = g_wt[static_cast<int64_t>(t) * d_out + j];
        g_w[static_cast<int64_t>(t) * ld_gw + j] = b * column + (fabsf(wv) < 1.0f ? a * g : 0.0f);
    }
}

struct BackwardMap {
    size_t g_zeta_off, g_pad_off, records_off, wt_bits_off, scratch_scale_off, w_bits_off, alpha_off, g_wt_off, partial_off, total;
    int64_t d_pad;        // row stride of g_zeta: d_out rounded up to a multiple of 4
    int64_t chunks, rows_per_chunk;
};

static size_t align256(size_t v) { return (v + 255) & ~static_cast<size_t>(255); }

static BackwardMap map_backward(int64_t n, int64_t d_in, int64_t d_out)
{
    BackwardMap m;
    // enough workgroups to fill the chip a few times; whole staging steps per chunk
    const int64_t blocks_per_chunk = ((d_out + 63) / 64) * ((d_in + 255) / 256);
    int64_t chunks = (1024 + blocks_per_chunk - 1) / blocks_per_chunk;
    const int64_t max_chunks = (n + kStageRows - 1) / kStageRows;
    if (chunks > max_chunks) chunks = max_chunks;
    if (chunks < 1) chunks = 1;
    int64_t rpc = (n + chunks - 1) / chunks;
    rpc = (rpc + kStageRows - 1) / kStageRows * kStageRows;
    m.chunks = (n + rpc - 1) / rpc;
    if (m.chunks < 1) m.chunks = 1;
    m.rows_per_chunk = rpc;
    size_t off = 0;
    m.d_pad = (d_out + 3) / 4 * 4;
    m.g_zeta_off = off;        off = align256(off + static_cast<size_t>(n) * m.d_pad * sizeof(float));
    m.g_pad_off = off;         // padded copy of g_out, only when d_out is not a multiple of 4
    if (m.d_pad != d_out) off = align256(off + static_cast<size_t>(n) * m.d_pad * sizeof(float));
    m.records_off = off;       // {packed signs, scale} per node, only for the first-layer order (d_in <= d_out)
    if (d_in <= d_out) off = align256(off + static_cast<size_t>(n) * ((d_in + 63) / 64 + 1) * sizeof(uint64_t));
    m.wt_bits_off = off;       off = align256(off + static_cast<size_t>(d_in) * ((d_out + 63) / 64) * sizeof(uint64_t));
    m.scratch_scale_off = off; off = align256(off + static_cast<size_t>(d_in) * sizeof(float));
    m.w_bits_off = off;        off = align256(off + static_cast<size_t>(d_out) * ((d_in + 63) / 64) * sizeof(uint64_t));
    m.alpha_off = off;         off = align256(off + static_cast<size_t>(d_out) * sizeof(float));
    m.g_wt_off = off;          off = align256(off + static_cast<size_t>(d_in) * d_out * sizeof(float));
    m.partial_off = off;       off = align256(off + static_cast<size_t>(m.chunks) * d_in * d_out * sizeof(float));
    m.total = off;
    return m;
}

}  // namespace bigcn

using namespace bigcn;

extern "C" size_t bigcn_layer_backward_workspace_bytes(int64_t n, int64_t d_in, int64_t d_out)
{
    if (n <= 0 || d_in <= 0 || d_out <= 0 || d_in > BIGCN_MAX_K_BITS || d_out > BIGCN_MAX_K_BITS) return 0;
    return map_backward(n, d_in, d_out).total;
}

extern "C" int bigcn_layer_backward(const bigcn_plan *plan, const int64_t *row_ptr, const int32_t *col_idx,
                                    const float *vals, int64_t n, const float *g_out, int64_t ld_g,
                                    const uint64_t *f_bits, int64_t ld_f_words, const float *beta,
                                    const float *w, int64_t ld_w, int64_t d_in, int64_t d_out,
                                    const float *bn_mul, float *g_w, int64_t ld_gw, float *g_in,
                                    int64_t ld_gin, void *workspace, size_t workspace_bytes, void *stream)
{
    if (plan == nullptr || row_ptr == nullptr || col_idx == nullptr || vals == nullptr || g_out == nullptr ||
        f_bits == nullptr || beta == nullptr || w == nullptr || g_w == nullptr)
        return BIGCN_ENULL;
    if (n != plan->n || d_in <= 0 || d_out <= 0 || ld_g < d_out || ld_w < d_out || ld_gw < d_out ||
        ld_f_words < (d_in + 63) / 64 || (g_in != nullptr && ld_gin < d_in))
        return BIGCN_EINVAL;
    if (d_in > BIGCN_MAX_K_BITS || d_out > BIGCN_MAX_K_BITS) return BIGCN_ESHAPE;
    if (n == 0) return BIGCN_OK;
    const BackwardMap map = map_backward(n, d_in, d_out);
    if (workspace == nullptr || workspace_bytes < map.total || reinterpret_cast<uintptr_t>(workspace) % 256 != 0)
        return BIGCN_EWORKSPACE;
    hipStream_t s = as_stream(stream);
    char *ws = static_cast<char *>(workspace);
    float *g_zeta = reinterpret_cast<float *>(ws + map.g_zeta_off);
    uint64_t *wt_bits = reinterpret_cast<uint64_t *>(ws + map.wt_bits_off);
    float *row_scale = reinterpret_cast<float *>(ws + map.scratch_scale_off);
    uint64_t *w_bits = reinterpret_cast<uint64_t *>(ws + map.w_bits_off);
    float *alpha = reinterpret_cast<float *>(ws + map.alpha_off);
    float *g_wt = reinterpret_cast<float *>(ws + map.g_wt_off);
    float *partial = reinterpret_cast<float *>(ws + map.partial_off);
    const int64_t wt_ld = (d_out + 63) / 64, wb_ld = (d_in + 63) / 64;

    // weights packed both ways: along j for the input gradient (row t of W), and the column
    // scales alpha_j from the transposed view (Sec. 4.2.1)
    int rc = launch_pack(w, d_in, d_out, ld_w, 1, nullptr, nullptr, nullptr, 0, wt_bits, wt_ld, row_scale, s);
    if (rc != BIGCN_OK) return rc;
    rc = launch_pack(w, d_out, d_in, 1, ld_w, nullptr, nullptr, nullptr, 0, w_bits, wb_ld, alpha, s);
    if (rc != BIGCN_OK) return rc;

    if (g_in == nullptr && d_in <= d_out) {
        // first layer: g_wt = (A~ H~)^T g_out; U = A~ H~ (n x d_in) takes the place of g_zeta
        float *u = g_zeta;
        const int64_t node_blocks = (n + kWavesPerBlock - 1) / kWavesPerBlock;
        const int n_words = static_cast<int>((d_in + 63) / 64);
        uint64_t *records = reinterpret_cast<uint64_t *>(ws + map.records_off);
        {
            const int64_t total = n * (n_words + 1);
            int64_t blocks = (total + kBlock - 1) / kBlock;
            if (blocks > compute_units() * 32) blocks = compute_units() * 32;
            hipLaunchKernelGGL(sign_records_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0, s, f_bits,
                               ld_f_words, beta, n, n_words, records);
            if (hipGetLastError() != hipSuccess) return BIGCN_EHIP;
        }
        for (int word0 = 0; word0 < n_words; word0 += 4) {
#define BIGCN_SIGNS_CASE(NW)                                                                                        \
    hipLaunchKernelGGL(aggregate_signs_kernel<NW>, dim3(static_cast<unsigned>(node_blocks)), dim3(kBlock), 0, s,   \
                       plan->row_order, n, row_ptr, col_idx, vals, records, static_cast<int>(d_in), word0, u,      \
                       d_in)
            const int left = n_words - word0;
            if (left >= 4) BIGCN_SIGNS_CASE(4);
            else if (left == 3) BIGCN_SIGNS_CASE(3);
            else if (left == 2) BIGCN_SIGNS_CASE(2);
            else BIGCN_SIGNS_CASE(1);
#undef BIGCN_SIGNS_CASE
            if (hipGetLastError() != hipSuccess) return BIGCN_EHIP;
        }
        const dim3 grid_d(static_cast<unsigned>(map.chunks), static_cast<unsigned>((d_out + 63) / 64),
                          static_cast<unsigned>((d_in + 127) / 128));
        hipLaunchKernelGGL(backward_weight_dense_partial_kernel, grid_d, dim3(kBlock), 0, s, g_out, n,
                           static_cast<int>(d_out), ld_g, u, d_in, static_cast<int>(d_in), map.rows_per_chunk, partial);
        if (hipGetLastError() != hipSuccess) return BIGCN_EHIP;
    } else {
        // Algorithm 1, first line: A~ is symmetric (the plan's pattern check guarantees the pattern,
        // the coefficients D^-1/2 (A+I) D^-1/2 are symmetric by construction), so A~^T g = A~ g
        if (map.d_pad != d_out) {
            // rows of a width that is not a multiple of 4 floats (class counts such as 47) would take
            // the one-float-per-lane path of the aggregation: aggregate a zero-padded copy instead
            float *g_pad = reinterpret_cast<float *>(ws + map.g_pad_off);
            const int64_t total = n * map.d_pad;
            int64_t blocks = (total + kBlock - 1) / kBlock;
            if (blocks > compute_units() * 32) blocks = compute_units() * 32;
            hipLaunchKernelGGL(pad_rows_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0, s, g_out, ld_g, n,
                               static_cast<int>(d_out), static_cast<int>(map.d_pad), g_pad);
            if (hipGetLastError() != hipSuccess) return BIGCN_EHIP;
            rc = bigcn_spmm(plan, row_ptr, col_idx, vals, n, g_pad, map.d_pad, map.d_pad, g_zeta, map.d_pad, stream);
        } else {
            rc = bigcn_spmm(plan, row_ptr, col_idx, vals, n, g_out, d_out, ld_g, g_zeta, map.d_pad, stream);
        }
        if (rc != BIGCN_OK) return rc;

        const dim3 grid_w(static_cast<unsigned>(map.chunks), static_cast<unsigned>((d_out + 63) / 64),
                          static_cast<unsigned>((d_in + 255) / 256));
        hipLaunchKernelGGL(backward_weight_partial_kernel, grid_w, dim3(kBlock), 0, s, g_zeta, n,
                           static_cast<int>(d_out), map.d_pad, beta, f_bits, ld_f_words, static_cast<int>(d_in),
                           map.rows_per_chunk, partial);
        if (hipGetLastError() != hipSuccess) return BIGCN_EHIP;
    }
    const int64_t elems = d_in * d_out;
    hipLaunchKernelGGL(backward_weight_reduce_kernel, dim3(static_cast<unsigned>((elems + kBlock - 1) / kBlock)),
                       dim3(kBlock), 0, s, partial, map.chunks, elems, g_wt);
    if (hipGetLastError() != hipSuccess) return BIGCN_EHIP;
    hipLaunchKernelGGL(backward_weight_finish_kernel, dim3(static_cast<unsigned>(d_out)), dim3(kWave), 0, s, g_wt, w,
                       ld_w, alpha, static_cast<int>(d_in), static_cast<int>(d_out), g_w, ld_gw);
    if (hipGetLastError() != hipSuccess) return BIGCN_EHIP;

    if (g_in != nullptr) {
        const dim3 grid_i(static_cast<unsigned>((n + 127) / 128), static_cast<unsigned>((d_in + 127) / 128));
        hipLaunchKernelGGL(backward_input_kernel, grid_i, dim3(kBlock), 0, s, g_zeta, n, static_cast<int>(d_out),
                           map.d_pad, alpha, wt_bits, wt_ld, static_cast<int>(d_in), bn_mul, g_in, ld_gin);
        if (hipGetLastError() != hipSuccess) return BIGCN_EHIP;
    }
    return BIGCN_OK;
}
