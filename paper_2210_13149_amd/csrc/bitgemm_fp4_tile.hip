// Kernel 2 on the FP4 matrix cores, large-tile form: the +-1 inner products of Sec. 4.2.3,
// c_ij = sum_k F_ik B_kj, for shapes that are bound by the multiplies (many rows, at least 65
// columns, K of 512 bits or more).
//
// One wavefront owns a tile of 128 rows x 128 columns (4 x 4 multiplies of 32 x 32 x 64 per 64
// bits of K, v_mfma_scale_f32_32x32x64_f8f6f4 with both operands FP4 E2M1 and unit scales) and
// runs alone on its SIMD: 256 accumulator registers, every expanded operand feeds four
// multiplies.  There is no LDS stage and no barrier.  K is walked in chunks of 256 bits; lane
// (i, h) (i = lane % 32, h = lane / 32) loads, for each of its four rows 32 rt + i and its four
// columns 32 ct + i, the 16 bytes [32 chunk + 16 h, +16) of the packed row straight from global
// memory (the two lanes of a row read 32 consecutive bytes; a 128-byte line serves four chunks
// and stays in L2 meanwhile), two chunks ahead of the one being multiplied.  The order of the k
// values inside a multiply is free as long as both operands agree, so multiply t of a chunk
// simply takes dword t of every lane's 16 bytes.
//
// Codes: the 32 bits x of a dword become four operand dwords, operand dword d taking the bits
// d, d + 4, ..., d + 28 of x where they stand.
//   rows    (values {0, +1}):  x & (0x11111111 << d)  -> codes 0x1 / 0x2 / 0x4 = 0.5 / 1 / 2;
//                              d = 3 is shifted down to 0x2 (0x8 would be -0)
//   columns (values -b, b = +-1): sign bit of the code = the bit itself, magnitude 2 / 1 / 0.5 / 1
// so that every product is exactly 0 or -b_k: the fp32 accumulators hold -S, S = sum_k a_k b_k
// (integers below 2^24: exact), and with f = 2a - 1
//   c_ij = 2 S - sum_{k<K} b_kj = K - 2 (ones_j - S),  ones_j = set bits of column j below K.
// Bits at and beyond K are cleared in both operands when the last, partial chunk is loaded, so
// they contribute neither to S nor to ones_j.
#include "bigcn_internal.h"

namespace bigcn {

namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kTileRows = 128, kTileCols = 128;
constexpr int kChunkBits = 256;

// 16 bytes of a packed row; rows are only 8-byte aligned
struct __attribute__((aligned(8))) Bits128 {
    uint32_t d[4];
};

__device__ __forceinline__ v8i codes_row(uint32_t x)
{
    v8i op;
    op[0] = static_cast<int>(x & 0x11111111u);
    op[1] = static_cast<int>(x & 0x22222222u);
    op[2] = static_cast<int>(x & 0x44444444u);
    op[3] = static_cast<int>((x & 0x88888888u) >> 2);
    op[4] = op[5] = op[6] = op[7] = 0;
    return op;
}

// (x << shift) | c and (x & mask) | c as one instruction each: the compiler's own selection
// spends three (shift, and, or) because a literal cannot be an operand of these encodings; here
// the constants are register operands.
__device__ __forceinline__ uint32_t lshl_or(uint32_t x, uint32_t shift, uint32_t c)
{
    uint32_t r;
    asm("v_lshl_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "s"(shift), "v"(c));
    return r;
}
__device__ __forceinline__ uint32_t and_or(uint32_t x, uint32_t mask, uint32_t c)
{
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "s"(mask), "v"(c));
    return r;
}

// mag[d]: the magnitude codes of operand dword d in every nibble (registers, see lshl_or)
__device__ __forceinline__ v8i codes_col(uint32_t x, const uint32_t (&mag)[3])
{
    v8i op;
    op[0] = static_cast<int>(lshl_or(x & 0x11111111u, 3, mag[0]));     // 2.0
    op[1] = static_cast<int>(lshl_or(x & 0x22222222u, 2, mag[1]));     // 1.0
    op[2] = static_cast<int>(lshl_or(x & 0x44444444u, 1, mag[2]));     // 0.5
    op[3] = static_cast<int>(and_or(x, 0x88888888u, mag[1]));          // 1.0
    op[4] = op[5] = op[6] = op[7] = 0;
    return op;
}

struct Chunk {
    Bits128 a[4];
    Bits128 b[4];
};

}  // namespace

// grid.x: groups of row tiles, grid.y: groups of column tiles; wavefront w of a workgroup takes
// row tile row_tiles_per_block * blockIdx.x + w / col_tiles_per_block and column tile
// col_tiles_per_block * blockIdx.y + w % col_tiles_per_block (the wavefronts that share rows sit
// in one workgroup, so that the rows come from HBM once).
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(1, 1))) void bitgemm_fp4_tile_kernel(
    const uint64_t *__restrict__ a, int64_t m, int64_t lda, const uint64_t *__restrict__ b, int n,
    int64_t ldb, int k_bits, int col_tiles_per_block, const float *__restrict__ a_scale,
    const float *__restrict__ b_scale, int32_t *__restrict__ acc_out, int64_t ld_acc, float *__restrict__ out,
    int64_t ld_out)
{
    const int lane = lane_id();
    const int wave = wave_in_block();
    const int i32 = lane & 31;
    const int half = lane >> 5;
    const int row_tiles_per_block = kWavesPerBlock / col_tiles_per_block;
    const int64_t row0 = (static_cast<int64_t>(blockIdx.x) * row_tiles_per_block + wave / col_tiles_per_block) * kTileRows;
    const int col0 = (static_cast<int>(blockIdx.y) * col_tiles_per_block + wave % col_tiles_per_block) * kTileCols;
    if (row0 >= m || col0 >= n) return;                       // wave-uniform; the kernel has no barrier

    // this lane's four rows and four columns (clamped: results of clamped rows / columns are not stored)
    const unsigned char *a_ptr[4], *b_ptr[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        int64_t row = row0 + 32 * t + i32;
        if (row >= m) row = m - 1;
        int col = col0 + 32 * t + i32;
        if (col >= n) col = n - 1;
        a_ptr[t] = reinterpret_cast<const unsigned char *>(a + row * lda) + 16 * half;
        b_ptr[t] = reinterpret_cast<const unsigned char *>(b + static_cast<int64_t>(col) * ldb) + 16 * half;
    }

    const int n_full = k_bits / kChunkBits;                   // chunks that lie wholly below K

    // a chunk that lies wholly below K: 16 bytes per row / column and lane
    auto load = [&](int c, Chunk &s) {
        if (c >= n_full) return;                              // uniform
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            s.a[t] = *reinterpret_cast<const Bits128 *>(a_ptr[t] + 32 * c);
            s.b[t] = *reinterpret_cast<const Bits128 *>(b_ptr[t] + 32 * c);
        }
    };
    // the partial chunk at the end of K: dword by dword, nothing is read at or beyond bit K and
    // the bits beyond K inside the last dword are cleared
    auto load_partial = [&](Chunk &s) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int left = k_bits - (kChunkBits * n_full + 128 * half + 32 * u);
            const uint32_t keep = left >= 32 ? 0xffffffffu : (left <= 0 ? 0u : ((1u << left) - 1u));
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                s.a[t].d[u] = 0u;
                s.b[t].d[u] = 0u;
            }
            if (left > 0) {
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    s.a[t].d[u] = *reinterpret_cast<const uint32_t *>(a_ptr[t] + 32 * n_full + 4 * u) & keep;
                    s.b[t].d[u] = *reinterpret_cast<const uint32_t *>(b_ptr[t] + 32 * n_full + 4 * u) & keep;
                }
            }
        }
    };

    v16f acc[4][4];
#pragma unroll
    for (int rt = 0; rt < 4; ++rt)
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rt][ct][r] = 0.0f;
    int ones[4] = {0, 0, 0, 0};                               // set bits of this lane's half of its columns
    // magnitude codes 2.0 / 1.0 / 0.5 in every nibble, kept in vector registers (opaque to the
    // compiler so that they are not folded back into literals)
    uint32_t mag[3] = {0x44444444u, 0x22222222u, 0x11111111u};
#pragma unroll
    for (int d = 0; d < 3; ++d) asm volatile("" : "+v"(mag[d]));

    auto multiply = [&](const Chunk &s) {
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
            for (int u = 0; u < 4; ++u) ones[ct] += __popc(s.b[ct].d[u]);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            v8i aop[4], bop[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                aop[t] = codes_row(s.a[t].d[u]);
                bop[t] = codes_col(s.b[t].d[u], mag);
            }
#pragma unroll
            for (int rt = 0; rt < 4; ++rt)
#pragma unroll
                for (int ct = 0; ct < 4; ++ct)
                    acc[rt][ct] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                        aop[rt], bop[ct], acc[rt][ct], 4, 4, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
        }
    };

    // Three register sets in rotation, chunk c + 2 requested before chunk c is multiplied; the
    // loop body is three whole chunks so that the sets keep their names (no copies) and the loop
    // has one exit (the 256 accumulators must not meet at a join of several paths); the one or
    // two chunks left over are already in s0 / s1 when the loop ends.
    {
        Chunk s0, s1, s2;
        load(0, s0);
        load(1, s1);
        int c = 0;
        for (; c + 3 <= n_full; c += 3) {
            load(c + 2, s2);
            multiply(s0);
            load(c + 3, s0);
            multiply(s1);
            load(c + 4, s1);
            multiply(s2);
        }
        const bool partial = n_full * kChunkBits < k_bits;
        if (partial) load_partial(s2);
        if (c < n_full) multiply(s0);
        if (c + 1 < n_full) multiply(s1);
        if (partial) multiply(s2);
    }

    // epilogue: accumulator register r of lane (i, h) holds row 8 (r / 4) + 4 h + r % 4, column i
#pragma unroll
    for (int ct = 0; ct < 4; ++ct) {
        const int col_ones = ones[ct] + __shfl_xor(ones[ct], 32, kWave);
        const int j = col0 + 32 * ct + i32;
        const bool col_ok = j < n;
        const int base = k_bits - 2 * col_ones;               // c = base - 2 * acc  (acc = -S)
        const float sb = (out != nullptr && col_ok) ? b_scale[j] : 0.0f;
#pragma unroll
        for (int rt = 0; rt < 4; ++rt) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = row0 + 32 * rt + 8 * (r >> 2) + 4 * half + (r & 3);
                if (col_ok && row < m) {
                    const int c = base - 2 * static_cast<int>(acc[rt][ct][r]);
                    if (acc_out != nullptr) acc_out[row * ld_acc + j] = c;
                    if (out != nullptr) out[row * ld_out + j] = a_scale[row] * sb * static_cast<float>(c);
                }
            }
        }
    }
}

// Shapes the tile kernel takes: enough columns to fill most of a 128-column tile and enough K
// for the multiplies to dominate.
bool fp4_tile_covers(int64_t m, int64_t n, int64_t k_bits)
{
    return n > 64 && k_bits >= 512 && m >= 4096;
}

int launch_bitgemm_fp4_tile(const uint64_t *a_bits, const float *a_scale, int64_t m, int64_t lda,
                            const uint64_t *b_bits, const float *b_scale, int64_t n, int64_t ldb,
                            int64_t k_bits, int32_t *acc, int64_t ld_acc, float *out, int64_t ld_out,
                            hipStream_t stream)
{
    const int64_t row_tiles = (m + kTileRows - 1) / kTileRows;
    const int64_t col_tiles = (n + kTileCols - 1) / kTileCols;
    const int col_tiles_per_block = col_tiles >= 2 ? 2 : 1;
    const int row_tiles_per_block = kWavesPerBlock / col_tiles_per_block;
    const int64_t grid_x = (row_tiles + row_tiles_per_block - 1) / row_tiles_per_block;
    const int64_t grid_y = (col_tiles + col_tiles_per_block - 1) / col_tiles_per_block;
    if (grid_x > 0x7fffffff || grid_y > 65535) return BIGCN_ESHAPE;
    hipLaunchKernelGGL(bitgemm_fp4_tile_kernel, dim3(static_cast<unsigned>(grid_x), static_cast<unsigned>(grid_y)),
                       dim3(kBlock), 0, stream, a_bits, m, lda, b_bits, static_cast<int>(n), ldb,
                       static_cast<int>(k_bits), col_tiles_per_block, a_scale, b_scale, acc, ld_acc, out, ld_out);
    return check_launch();
}

}  // namespace bigcn
