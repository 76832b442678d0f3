// Kernel 2, matrix-core variant: the +-1 inner products of Sec. 4.2.3 evaluated with the
// int8 MFMA of gfx950 (v_mfma_i32_32x32x32_i8) instead of XOR + bit count.
//
// The packed operands are expanded on the fly.  A (node rows) is expanded to bytes in {0, 1}
// (three VALU operations per four elements), B (weight columns) to bytes in {-1, +1}, once per
// workgroup and K chunk, into LDS.  With a in {0,1} and f = 2a - 1:
//     sum_k f_k b_k = 2 * sum_k a_k b_k - sum_k b_k ,
// so the matrix core accumulates sum_k a_k b_k exactly in int32 and the epilogue subtracts the
// column sum of B (2 popcount(B_j) - K).  Pad bits of A are 0 and therefore contribute nothing.
//
// Tiling for wave64: a workgroup of four wavefronts owns 256 rows x 64 columns; each wavefront
// owns 64 rows x 64 columns as 2 x 2 MFMA tiles of 32 x 32 (64 accumulator registers), so every
// expanded A operand and every B operand read from LDS feeds two MFMAs.  K advances in chunks
// of 512 bits: the chunk of B is staged as [column][k] bytes with a 16-byte pad per column
// (conflict-free 16-byte reads); the chunk of A (256 rows x 64 bytes of packed bits) is staged as
// is, through coalesced loads.  The packed words of the next chunk (A and B) are fetched into
// registers while the current chunk is multiplied and written to LDS between two barriers.
#include "bigcn_internal.h"

namespace bigcn {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kMfmaChunkWords = 8;                       // 512 bits of K per stage
constexpr int kMfmaChunkBytes = kMfmaChunkWords * 64;    // expanded bytes per column and chunk
constexpr int kMfmaColStride = kMfmaChunkBytes + 16;     // LDS bytes per column
constexpr int kMfmaCols = 64;                            // columns per workgroup
constexpr int kMfmaRows = 256;                           // rows per workgroup

// four packed bits -> four bytes in {0, 1}
__device__ __forceinline__ uint32_t spread4(uint32_t nibble)
{
    return (nibble * 0x00204081u) & 0x01010101u;
}
// four packed bits -> four bytes in {-1, +1}
__device__ __forceinline__ uint32_t spread4_pm1(uint32_t nibble)
{
    return ~(spread4(nibble) * 0xFEu);      // 1 -> 0x01, 0 -> 0xFF, no borrow between bytes
}

// Expand two packed words of B (this thread's share of a chunk) into +-1 bytes in LDS.
__device__ __forceinline__ void stage_b_words(unsigned char *lds_b, const uint64_t (&word)[2],
                                              const bool (&live)[2])
{
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int item = static_cast<int>(threadIdx.x) + t * kBlock;
        const int c = item / kMfmaChunkWords;
        const int q = item - c * kMfmaChunkWords;
        uint4 *dst = reinterpret_cast<uint4 *>(lds_b + c * kMfmaColStride + q * 64);
#pragma unroll
        for (int part = 0; part < 4; ++part) {
            const uint32_t bits16 = static_cast<uint32_t>(word[t] >> (16 * part)) & 0xffffu;
            uint4 v;
            v.x = live[t] ? spread4_pm1(bits16 & 0xf) : 0u;
            v.y = live[t] ? spread4_pm1((bits16 >> 4) & 0xf) : 0u;
            v.z = live[t] ? spread4_pm1((bits16 >> 8) & 0xf) : 0u;
            v.w = live[t] ? spread4_pm1((bits16 >> 12) & 0xf) : 0u;
            dst[part] = v;
        }
    }
}

constexpr int kMfmaARowStride = kMfmaChunkWords * 8 + 8;   // LDS bytes per row of the A chunk

__global__ __launch_bounds__(kBlock) void bitgemm_mfma_kernel(
    const uint64_t *__restrict__ a, int64_t m, int64_t lda, const uint64_t *__restrict__ b, int n,
    int64_t ldb, int k_bits, const float *__restrict__ a_scale, const float *__restrict__ b_scale,
    int32_t *__restrict__ acc_out, int64_t ld_acc, float *__restrict__ out, int64_t ld_out)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds_b[kMfmaCols * kMfmaColStride];
    __shared__ __attribute__((aligned(16))) unsigned char lds_a[kMfmaRows * kMfmaARowStride];
    static_assert(kMfmaCols * kMfmaChunkWords == 2 * kBlock, "two words of B per thread and chunk");
    static_assert(kMfmaRows * kMfmaChunkWords == 8 * kBlock, "eight words of A per thread and chunk");
    const int n_words = (k_bits + 63) >> 6;
    const int lane = lane_id();
    const int wave = wave_in_block();
    const int i32 = lane & 31;          // row of an A tile / column of a B tile supplied by this lane
    const int half = lane >> 5;         // which 16 of the 32 k values of an MFMA this lane supplies
    const int64_t block_row0 = static_cast<int64_t>(blockIdx.x) * kMfmaRows;
    const int64_t row0 = block_row0 + wave * 64;
    const int col0 = blockIdx.y * kMfmaCols;

    v16i acc[2][2];
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
        for (int ct = 0; ct < 2; ++ct)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rt][ct][r] = 0;

    // Packed words of A reach the wavefronts through LDS: thread t fetches words (2 p + t % 4 * 2)
    // ... of row t / 4 + 64 p, i.e. four consecutive lanes read the 64 contiguous bytes a row
    // contributes to a chunk, so global loads are coalesced per row instead of one 8-byte
    // request per row and lane.
    const int a_thread_row = static_cast<int>(threadIdx.x) >> 2;      // 0..63, + 64 p
    const int a_thread_word = (static_cast<int>(threadIdx.x) & 3) * 2; // 0, 2, 4, 6
    const uint64_t *asrc[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        int64_t row = block_row0 + a_thread_row + 64 * p;
        if (row >= m) row = m - 1;                          // clamped rows are never stored
        asrc[p] = a + row * lda + a_thread_word;
    }
    // this thread's two words of every B chunk: (column, word) = item / 8, item % 8
    const uint64_t *bsrc[2];
    bool bcol_live[2];
    int bq[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int item = static_cast<int>(threadIdx.x) + t * kBlock;
        const int c = item / kMfmaChunkWords;
        bq[t] = item - c * kMfmaChunkWords;
        const int j = col0 + c;
        bcol_live[t] = j < n;
        bsrc[t] = b + static_cast<int64_t>(bcol_live[t] ? j : 0) * ldb;
    }

    uint64_t a_next[4][2];
    uint64_t b_next[2];
    bool b_live[2];
    auto fetch = [&](int w0) {
#pragma unroll
        for (int p = 0; p < 4; ++p)
#pragma unroll
            for (int e = 0; e < 2; ++e)                       // zero past the last word
                a_next[p][e] = (w0 + a_thread_word + e < n_words) ? asrc[p][w0 + e] : 0ull;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            b_live[t] = bcol_live[t] && w0 + bq[t] < n_words;
            b_next[t] = b_live[t] ? bsrc[t][w0 + bq[t]] : 0ull;
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            uint2 *dst = reinterpret_cast<uint2 *>(lds_a + (a_thread_row + 64 * p) * kMfmaARowStride + a_thread_word * 8);
            dst[0] = make_uint2(static_cast<uint32_t>(a_next[p][0]), static_cast<uint32_t>(a_next[p][0] >> 32));
            dst[1] = make_uint2(static_cast<uint32_t>(a_next[p][1]), static_cast<uint32_t>(a_next[p][1] >> 32));
        }
        stage_b_words(lds_b, b_next, b_live);
    };

    fetch(0);
    stage();
    __syncthreads();

    const unsigned char *a_lane[2];
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) a_lane[rt] = lds_a + (wave * 64 + 32 * rt + i32) * kMfmaARowStride;

    for (int w0 = 0; w0 < n_words; w0 += kMfmaChunkWords) {
        const bool more = w0 + kMfmaChunkWords < n_words;       // uniform
        if (more) fetch(w0 + kMfmaChunkWords);                  // in flight during the MFMAs below

#pragma unroll
        for (int q = 0; q < kMfmaChunkWords; ++q) {
            if (w0 + q >= n_words) break;                    // uniform
            uint2 aw[2];
#pragma unroll
            for (int rt = 0; rt < 2; ++rt) aw[rt] = *reinterpret_cast<const uint2 *>(a_lane[rt] + 8 * q);
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
                // 32 k values per step: bits [32 s, 32 s + 32) of the chunk, s = 2 q + sub;
                // this lane supplies 16 of them
                const int s = 2 * q + sub;
                v4i aop[2], bop[2];
#pragma unroll
                for (int rt = 0; rt < 2; ++rt) {
                    const uint32_t bits16 = ((sub ? aw[rt].y : aw[rt].x) >> (16 * half)) & 0xffffu;
                    aop[rt][0] = static_cast<int>(spread4(bits16 & 0xf));
                    aop[rt][1] = static_cast<int>(spread4((bits16 >> 4) & 0xf));
                    aop[rt][2] = static_cast<int>(spread4((bits16 >> 8) & 0xf));
                    aop[rt][3] = static_cast<int>(spread4((bits16 >> 12) & 0xf));
                }
#pragma unroll
                for (int ct = 0; ct < 2; ++ct)
                    bop[ct] = *reinterpret_cast<const v4i *>(lds_b + (32 * ct + i32) * kMfmaColStride + 32 * s + 16 * half);
#pragma unroll
                for (int rt = 0; rt < 2; ++rt)
#pragma unroll
                    for (int ct = 0; ct < 2; ++ct)
                        acc[rt][ct] = __builtin_amdgcn_mfma_i32_32x32x32_i8(aop[rt], bop[ct], acc[rt][ct], 0, 0, 0);
            }
        }
        __syncthreads();                                     // every wavefront has left this chunk
        if (more) stage();
        __syncthreads();
    }

    // epilogue: c = 2 * acc - (2 popcount(B_j) - K); accumulator register r of a 32x32 tile holds
    // row 8 (r / 4) + 4 half + r % 4 and column lane % 32
#pragma unroll
    for (int ct = 0; ct < 2; ++ct) {
        const int j = col0 + 32 * ct + i32;
        if (j >= n) continue;
        int ones = 0;
        for (int w = 0; w < n_words; ++w) ones += __popcll(b[static_cast<int64_t>(j) * ldb + w]);
        const int colsum = 2 * ones - k_bits;
        const float sb = out != nullptr ? b_scale[j] : 0.0f;
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = row0 + 32 * rt + 8 * (r >> 2) + 4 * half + (r & 3);
                if (row < m) {
                    const int c = 2 * acc[rt][ct][r] - colsum;
                    if (acc_out != nullptr) acc_out[row * ld_acc + j] = c;
                    if (out != nullptr) out[row * ld_out + j] = a_scale[row] * sb * static_cast<float>(c);
                }
            }
        }
    }
}

int launch_bitgemm_mfma(const uint64_t *a_bits, const float *a_scale, int64_t m, int64_t lda,
                        const uint64_t *b_bits, const float *b_scale, int64_t n, int64_t ldb,
                        int64_t k_bits, int32_t *acc, int64_t ld_acc, float *out, int64_t ld_out,
                        hipStream_t stream)
{
    const int64_t row_blocks = (m + kMfmaRows - 1) / kMfmaRows;
    const int64_t col_blocks = (n + kMfmaCols - 1) / kMfmaCols;
    if (row_blocks > 0x7fffffff || col_blocks > 65535) return BIGCN_ESHAPE;
    hipLaunchKernelGGL(bitgemm_mfma_kernel, dim3(static_cast<unsigned>(row_blocks), static_cast<unsigned>(col_blocks)),
                       dim3(kBlock), 0, stream, a_bits, m, lda, b_bits, static_cast<int>(n), ldb,
                       static_cast<int>(k_bits), a_scale, b_scale, acc, ld_acc, out, ld_out);
    return check_launch();
}

}  // namespace bigcn
