// Kernel 1: sign-binarise and bit-pack matrix rows, with the L1 scale of each row
// (vector binarisation, Sec. 4.1; node features Sec. 4.2.2; weights Sec. 4.2.1 through a
// transposed view; optional per-column standardisation, Sec. 4.4 step 1).
//
// One wavefront owns a row: lane l reads column 64*w + l, so every load instruction of the
// wavefront covers 256 contiguous bytes, and the 64-bit ballot of the comparison *is* the
// packed word w (bit l <-> column 64*w + l).  The kernel is bound by reading x from HBM.
#include "bigcn_internal.h"

namespace bigcn {

// rows a wavefront of pack_short_kernel<NW> fetches together
constexpr int pack_rows_in_flight(int nw) { return nw >= 8 ? 1 : 8 / nw; }

// Rows of NW words (at most 1024 columns), unit column stride.  A lane keeps the thresholds and
// multipliers of its NW columns in registers.  A wavefront owns `chunk_rows` (at most 64)
// consecutive rows, fetches RB of them together (about 8 loads, at least one whole row) to cover
// HBM latency, and holds the results back: lane r keeps the packed words and the scale of the
// chunk's row r, so that the chunk is written with NW + 1 coalesced stores at its end.  Storing
// 16 + 4 bytes after every row costs a third of the kernel (0.245 against 0.17 ms on 2.4 M rows
// of 100 columns).
template <int NW>
__global__ __launch_bounds__(kBlock) void pack_short_kernel(
    const float *__restrict__ x, int64_t rows, int cols, int64_t row_stride,
    const float *__restrict__ shift, const float *__restrict__ mul,
    const float *__restrict__ row_mul, int fold_last_sign, uint64_t *__restrict__ bits,
    int64_t ld_words, float *__restrict__ scale, int chunk_rows, int *__restrict__ clear_flag)
{
    if (clear_flag != nullptr && blockIdx.x == 0 && threadIdx.x == 0) *clear_flag = 0;
    constexpr int RB = pack_rows_in_flight(NW);
    const int lane = lane_id();
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * kWavesPerBlock + wave_in_block();
    const int64_t row_begin = wave * chunk_rows;
    if (row_begin >= rows) return;                                   // wave-uniform
    const int64_t row_end = rows - row_begin < chunk_rows ? rows : row_begin + chunk_rows;

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
    uint64_t keep[NW];
#pragma unroll
    for (int w = 0; w < NW; ++w) keep[w] = 0;
    float keep_scale = 0.0f;

    for (int64_t row0 = row_begin; row0 < row_end; row0 += RB) {
        float v[RB][NW];
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            const int64_t row = row0 + r;
#pragma unroll
            for (int w = 0; w < NW; ++w)
                v[r][w] = (row < row_end && in[w]) ? x[row * row_stride + 64 * w + lane] : 0.0f;
        }
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            const int64_t row = row0 + r;
            if (row >= row_end) break;          // wave-uniform
            const bool me = lane == static_cast<int>(row - row_begin);
            float sum = 0.0f;
            uint64_t last_word = 0;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                const bool bit = in[w] && (v[r][w] >= th[w]);
                const uint64_t word = __ballot(bit);
                if (me) keep[w] = word;
                last_word = word;
                sum += in[w] ? fabsf((v[r][w] - th[w]) * ml[w]) : 0.0f;
            }
            sum = wave_sum_dpp(sum);
            float s = sum * inv_cols;
            if (row_mul != nullptr) s *= row_mul[row];
            if (fold_last_sign && ((last_word >> ((cols - 1) & 63)) & 1ull) == 0) s = -s;
            if (me) keep_scale = s;
        }
    }
    const int64_t my_row = row_begin + lane;
    if (my_row < row_end) {
#pragma unroll
        for (int w = 0; w < NW; ++w)
            if (64 * w < cols) bits[my_row * ld_words + w] = keep[w];
        scale[my_row] = keep_scale;
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
        sum = wave_sum_dpp(sum);
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

static int grid_for_waves(int64_t waves_needed)
{
    // enough workgroups to fill 256 CUs several times over; grid-stride loops take the rest
    const int64_t blocks = (waves_needed + kWavesPerBlock - 1) / kWavesPerBlock;
    const int64_t cap = static_cast<int64_t>(compute_units()) * 16;
    return static_cast<int>(blocks < 1 ? 1 : (blocks > cap ? cap : blocks));
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

int launch_pack(const float *x, int64_t rows, int64_t cols, int64_t row_stride,
                int64_t col_stride, const float *shift, const float *mul, const float *row_mul,
                int fold_last_sign, uint64_t *bits, int64_t ld_words, float *scale,
                hipStream_t stream, int *clear_flag)
{
    if (rows == 0) return BIGCN_OK;
    const int64_t n_words = (cols + 63) / 64;
    if (col_stride == 1 && n_words <= 16) {
        const int icols = static_cast<int>(cols);
        // 64 rows per wavefront once that still gives every SIMD several wavefronts, else 16
        const int chunk = rows >= static_cast<int64_t>(compute_units()) * 4 * 4 * 64 ? 64 : 16;
        const int64_t waves = (rows + chunk - 1) / chunk;
        const dim3 grid(static_cast<unsigned>((waves + kWavesPerBlock - 1) / kWavesPerBlock));
#define BIGCN_PACK_SHORT(NW)                                                                                       \
    case NW:                                                                                                       \
        hipLaunchKernelGGL(pack_short_kernel<NW>, grid, dim3(kBlock), 0, stream, x, rows, icols, row_stride,      \
                           shift, mul, row_mul, fold_last_sign, bits, ld_words, scale, chunk, clear_flag);         \
        break
        switch (n_words) {
            BIGCN_PACK_SHORT(1); BIGCN_PACK_SHORT(2); BIGCN_PACK_SHORT(3); BIGCN_PACK_SHORT(4);
            BIGCN_PACK_SHORT(5); BIGCN_PACK_SHORT(6); BIGCN_PACK_SHORT(7); BIGCN_PACK_SHORT(8);
            BIGCN_PACK_SHORT(9); BIGCN_PACK_SHORT(10); BIGCN_PACK_SHORT(11); BIGCN_PACK_SHORT(12);
            BIGCN_PACK_SHORT(13); BIGCN_PACK_SHORT(14); BIGCN_PACK_SHORT(15);
        default:
            BIGCN_PACK_SHORT(16);
        }
#undef BIGCN_PACK_SHORT
    } else {
        hipLaunchKernelGGL(pack_generic_kernel, dim3(grid_for_waves(rows)), dim3(kBlock), 0, stream,
                           x, rows, cols, row_stride, col_stride, shift, mul, row_mul, fold_last_sign,
                           bits, ld_words, scale, clear_flag);
    }
    return check_launch();
}

// Nothing but a read: every workgroup takes one contiguous piece of the array, a thread eight
// 16-byte loads at a time.  The rate a kernel bound by reading its input once can reach here.
__global__ __launch_bounds__(kBlock) void stream_read_kernel(const uint4 *__restrict__ src, int64_t n_vec,
                                                             float *__restrict__ sink)
{
    constexpr int U = 8;
    const int64_t per_block = (n_vec + gridDim.x - 1) / gridDim.x;
    const int64_t b0 = per_block * blockIdx.x;
    const int64_t b1 = b0 + per_block < n_vec ? b0 + per_block : n_vec;
    uint32_t acc = 0;
    int64_t i = b0 + threadIdx.x;
    for (; i + (U - 1) * kBlock < b1; i += U * kBlock) {
        uint4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = src[i + u * kBlock];
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < b1; i += kBlock) {
        const uint4 v = src[i];
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    // one word per thread, so that the loads cannot be dropped
    sink[static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x] = __uint_as_float(acc & 0x007fffffu);
}

}  // namespace bigcn

extern "C" int bigcn_probe_stream_read(const void *src, int64_t bytes, float *sink, int64_t sink_floats, void *stream)
{
    if (src == nullptr || sink == nullptr) return BIGCN_ENULL;
    if (bytes < 16 || reinterpret_cast<uintptr_t>(src) % 16 != 0) return BIGCN_EINVAL;
    const int blocks = bigcn::compute_units() * 32;
    if (sink_floats < static_cast<int64_t>(blocks) * bigcn::kBlock) return BIGCN_EWORKSPACE;
    hipLaunchKernelGGL(bigcn::stream_read_kernel, dim3(blocks), dim3(bigcn::kBlock), 0, bigcn::as_stream(stream),
                       static_cast<const uint4 *>(src), bytes / 16, sink);
    return bigcn::check_launch();
}

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
