// Kernel 1: sign-binarise and bit-pack matrix rows, with the L1 scale of each row
// (vector binarisation, Sec. 4.1; node features Sec. 4.2.2; weights Sec. 4.2.1 through a
// transposed view; optional per-column standardisation, Sec. 4.4 step 1).
//
// One wavefront owns a row: lane l reads column 64*w + l, so every load instruction of the
// wavefront covers 256 contiguous bytes, and the 64-bit ballot of the comparison *is* the
// packed word w (bit l <-> column 64*w + l).  The kernel is bound by reading x from HBM.
#include "bigcn_internal.h"

namespace bigcn {

// Rows of at most NW words, unit column stride: a wavefront keeps RB rows (8 loads) in
// flight to cover HBM latency with short rows.
template <int NW>
__global__ __launch_bounds__(kBlock) void pack_short_kernel(
    const float *__restrict__ x, int64_t rows, int cols, int64_t row_stride,
    const float *__restrict__ shift, const float *__restrict__ mul,
    const float *__restrict__ row_mul, int fold_last_sign, uint64_t *__restrict__ bits,
    int64_t ld_words, float *__restrict__ scale, int *__restrict__ clear_flag)
{
    if (clear_flag != nullptr && blockIdx.x == 0 && threadIdx.x == 0) *clear_flag = 0;
    constexpr int RB = 8 / NW;
    const int lane = lane_id();
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * kWavesPerBlock + wave_in_block();
    const int64_t n_waves = static_cast<int64_t>(gridDim.x) * kWavesPerBlock;

    float th[NW], ml[NW];
    bool in[NW];
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        const int c = 64 * w + lane;
        in[w] = c < cols;
        th[w] = (shift != nullptr && in[w]) ? shift[c] : 0.0f;
        ml[w] = (mul != nullptr && in[w]) ? mul[c] : 1.0f;
    }
    const float inv_cols = 1.0f / static_cast<float>(cols);

    for (int64_t row0 = wave * RB; row0 < rows; row0 += n_waves * RB) {
        float v[RB][NW];
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            const int64_t row = row0 + r;
#pragma unroll
            for (int w = 0; w < NW; ++w)
                v[r][w] = (row < rows && in[w]) ? x[row * row_stride + 64 * w + lane] : 0.0f;
        }
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            const int64_t row = row0 + r;
            if (row >= rows) break;             // wave-uniform
            float sum = 0.0f;
            uint64_t mine = 0, last_word = 0;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                const bool bit = in[w] && (v[r][w] >= th[w]);
                const uint64_t word = __ballot(bit);
                if (lane == w) mine = word;
                last_word = word;
                sum += in[w] ? fabsf((v[r][w] - th[w]) * ml[w]) : 0.0f;
            }
            sum = wave_sum(sum);
            if (lane < NW && 64 * lane < cols) bits[row * ld_words + lane] = mine;
            if (lane == 0) {
                float s = sum * inv_cols;
                if (row_mul != nullptr) s *= row_mul[row];
                if (fold_last_sign && ((last_word >> ((cols - 1) & 63)) & 1ull) == 0) s = -s;
                scale[row] = s;
            }
        }
    }
}

// Any row length and any strides: a wavefront walks its row four words at a time.
__global__ __launch_bounds__(kBlock) void pack_generic_kernel(
    const float *__restrict__ x, int64_t rows, int64_t cols, int64_t row_stride,
    int64_t col_stride, const float *__restrict__ shift, const float *__restrict__ mul,
    const float *__restrict__ row_mul, int fold_last_sign, uint64_t *__restrict__ bits,
    int64_t ld_words, float *__restrict__ scale, int *__restrict__ clear_flag)
{
    if (clear_flag != nullptr && blockIdx.x == 0 && threadIdx.x == 0) *clear_flag = 0;
    constexpr int U = 4;
    const int lane = lane_id();
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * kWavesPerBlock + wave_in_block();
    const int64_t n_waves = static_cast<int64_t>(gridDim.x) * kWavesPerBlock;
    const int64_t n_words = (cols + 63) / 64;
    const float inv_cols = 1.0f / static_cast<float>(cols);

    for (int64_t row = wave; row < rows; row += n_waves) {
        const float *xr = x + row * row_stride;
        float sum = 0.0f;
        uint64_t mine = 0, last_word = 0;
        for (int64_t w0 = 0; w0 < n_words; w0 += U) {
            float v[U], th[U], ml[U];
            bool in[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t c = 64 * (w0 + u) + lane;
                in[u] = c < cols;
                v[u] = in[u] ? xr[c * col_stride] : 0.0f;
                th[u] = (shift != nullptr && in[u]) ? shift[c] : 0.0f;
                ml[u] = (mul != nullptr && in[u]) ? mul[c] : 1.0f;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t w = w0 + u;
                if (w >= n_words) break;        // wave-uniform
                const bool bit = in[u] && (v[u] >= th[u]);
                const uint64_t word = __ballot(bit);
                if (lane == static_cast<int>(w & 63)) mine = word;
                last_word = word;
                sum += in[u] ? fabsf((v[u] - th[u]) * ml[u]) : 0.0f;
                if ((w & 63) == 63 || w == n_words - 1) {
                    // lanes 0..(w & 63) hold words (w & ~63) .. w: one coalesced store
                    const int64_t base = w & ~static_cast<int64_t>(63);
                    if (lane <= static_cast<int>(w & 63)) bits[row * ld_words + base + lane] = mine;
                }
            }
        }
        sum = wave_sum(sum);
        if (lane == 0) {
            float s = sum * inv_cols;
            if (row_mul != nullptr) s *= row_mul[row];
            if (fold_last_sign && ((last_word >> ((cols - 1) & 63)) & 1ull) == 0) s = -s;
            scale[row] = s;
        }
    }
}

// Source scale of an input that arrives already binarised: beta_i times the optional per-row
// factor, negated when the layout folds the last input bit and that bit is -1.
__global__ __launch_bounds__(kBlock) void source_scale_kernel(const float *__restrict__ beta,
                                                              const float *__restrict__ row_mul,
                                                              const uint64_t *__restrict__ bits,
                                                              int64_t ld_words, int64_t cols,
                                                              int fold_last_sign, float *__restrict__ scale,
                                                              int64_t rows, int *__restrict__ clear_flag)
{
    if (clear_flag != nullptr && blockIdx.x == 0 && threadIdx.x == 0) *clear_flag = 0;
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i >= rows) return;
    float s = beta[i];
    if (row_mul != nullptr) s *= row_mul[i];
    if (fold_last_sign && ((bits[i * ld_words + ((cols - 1) >> 6)] >> ((cols - 1) & 63)) & 1ull) == 0) s = -s;
    scale[i] = s;
}

int launch_source_scale(const float *beta, const float *row_mul, const uint64_t *bits, int64_t ld_words,
                        int64_t cols, int fold_last_sign, float *scale, int64_t rows, hipStream_t stream,
                        int *clear_flag)
{
    if (rows == 0) return BIGCN_OK;
    hipLaunchKernelGGL(source_scale_kernel, dim3(static_cast<unsigned>((rows + kBlock - 1) / kBlock)), dim3(kBlock),
                       0, stream, beta, row_mul, bits, ld_words, cols, fold_last_sign, scale, rows, clear_flag);
    return check_launch();
}

static int grid_for_waves(int64_t waves_needed)
{
    // enough workgroups to fill 256 CUs several times over; grid-stride loops take the rest
    const int64_t blocks = (waves_needed + kWavesPerBlock - 1) / kWavesPerBlock;
    const int64_t cap = static_cast<int64_t>(compute_units()) * 16;
    return static_cast<int>(blocks < 1 ? 1 : (blocks > cap ? cap : blocks));
}

int launch_pack(const float *x, int64_t rows, int64_t cols, int64_t row_stride,
                int64_t col_stride, const float *shift, const float *mul, const float *row_mul,
                int fold_last_sign, uint64_t *bits, int64_t ld_words, float *scale,
                hipStream_t stream, int *clear_flag)
{
    if (rows == 0) return BIGCN_OK;
    const int64_t n_words = (cols + 63) / 64;
    if (col_stride == 1 && n_words <= 4) {
        const int icols = static_cast<int>(cols);
#define BIGCN_PACK_SHORT(NW)                                                                  \
    hipLaunchKernelGGL(pack_short_kernel<NW>, dim3(grid_for_waves((rows + 8 / NW - 1) / (8 / NW))), \
                       dim3(kBlock), 0, stream, x, rows, icols, row_stride, shift, mul, row_mul, \
                       fold_last_sign, bits, ld_words, scale, clear_flag)
        switch (n_words) {
        case 1: BIGCN_PACK_SHORT(1); break;
        case 2: BIGCN_PACK_SHORT(2); break;
        case 3: BIGCN_PACK_SHORT(3); break;
        default: BIGCN_PACK_SHORT(4); break;
        }
#undef BIGCN_PACK_SHORT
    } else {
        hipLaunchKernelGGL(pack_generic_kernel, dim3(grid_for_waves(rows)), dim3(kBlock), 0, stream,
                           x, rows, cols, row_stride, col_stride, shift, mul, row_mul, fold_last_sign,
                           bits, ld_words, scale, clear_flag);
    }
    return check_launch();
}

}  // namespace bigcn

extern "C" int bigcn_pack(const float *x, int64_t rows, int64_t cols, int64_t row_stride,
                          int64_t col_stride, const float *shift, const float *mul,
                          uint64_t *bits, int64_t ld_words, float *scale, void *stream)
{
    if (x == nullptr || bits == nullptr || scale == nullptr) return BIGCN_ENULL;
    if (rows < 0 || cols <= 0 || row_stride <= 0 || col_stride <= 0) return BIGCN_EINVAL;
    if (ld_words < (cols + 63) / 64) return BIGCN_EINVAL;
    return bigcn::launch_pack(x, rows, cols, row_stride, col_stride, shift, mul, nullptr, 0, bits,
                              ld_words, scale, bigcn::as_stream(stream));
}
