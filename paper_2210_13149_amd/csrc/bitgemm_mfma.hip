// Kernel 2, matrix-core variants: the +-1 inner products of Sec. 4.2.3 evaluated on the matrix
// cores of gfx950 instead of XOR + bit count.  Three kernels: int8 (v_mfma_i32_32x32x32_i8, described
// first), FP4 on the block-scaled path (bitgemm_fp4_kernel, same outputs as the int8 one) and the
// FP4 kernel that writes the one-byte product rows of the fused forward (bitgemm_fp4_rows_kernel).
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

#include <atomic>

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

// ---- FP4 matrix cores -------------------------------------------------------------------------
// The same product on the block-scaled multiply of gfx950 (v_mfma_scale_f32_32x32x64_f8f6f4 with
// both operands in FP4 E2M1 and unit scales): 64 values of K per instruction at twice the int8
// rate.  +1 is the FP4 code 0x2, -1 is 0xA, 0 is 0x0; a lane supplies 32 consecutive k values =
// 32 bits of a packed row = four dwords of eight codes.  A is expanded to {0, +1} (so pad bits
// contribute nothing), B to {-1, +1} with the bits past K set to 0, and, as above,
// sum_k f_k b_k = 2 sum_k a_k b_k - sum_k b_k.  The partial sums are integers below 2^24: the fp32
// accumulators are exact.
//
// Operand layout (checked on the device): A[i][k] is supplied by lane i + 32 (k / 32) as code
// number k % 32 of its 128 bits, B[k][j] by lane j + 32 (k / 32) likewise (the order inside the
// 32 is permuted on both sides, see fp4_codes_a); accumulator register r
// of lane l holds row 8 (r / 4) + 4 (l / 32) + r % 4 and column l % 32.
//
// Tiling: wavefront 32 RT rows x 32 CT columns (RT x CT tiles of 32 x 32), workgroup four
// wavefronts high; K in chunks of 256 bits in two LDS buffers (a chunk is staged while the one
// before it is multiplied; one barrier per chunk); the chunk of B is staged as [column][128 bytes
// of codes + 16 pad]; the number of set bits of every column is collected during the staging
// for the epilogue.
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

// The order of the k values inside a lane's operand is free as long as A and B agree, so the 32
// bits x of a packed half-word are not spread out bit by bit: dword d of the operand takes the
// bits d, d + 4, ..., d + 28 of x (code number i of dword d <-> bit 4 i + d), which is one mask
// and at most one shift per dword.
// {0, +1} codes (A): code = bit << 1.
__device__ __forceinline__ void fp4_codes_a(uint32_t x, int (&op)[4])
{
    op[0] = static_cast<int>((x & 0x11111111u) << 1);
    op[1] = static_cast<int>(x & 0x22222222u);
    op[2] = static_cast<int>((x & 0x44444444u) >> 1);
    op[3] = static_cast<int>((x & 0x88888888u) >> 2);
}
// {-1, +1} codes (B): code = 0x2 | (!bit << 3).
__device__ __forceinline__ uint4 fp4_codes_b(uint32_t x)
{
    const uint32_t n = ~x;
    return make_uint4(((n & 0x11111111u) << 3) | 0x22222222u, ((n & 0x22222222u) << 2) | 0x22222222u,
                      ((n & 0x44444444u) << 1) | 0x22222222u, (n & 0x88888888u) | 0x22222222u);
}
// 0xF for every code whose bit of `valid` is set, in the same order.
__device__ __forceinline__ uint4 fp4_code_mask(uint32_t valid)
{
    return make_uint4((valid & 0x11111111u) * 0xfu, ((valid >> 1) & 0x11111111u) * 0xfu,
                      ((valid >> 2) & 0x11111111u) * 0xfu, ((valid >> 3) & 0x11111111u) * 0xfu);
}

constexpr int kFp4ChunkWords = 4;                           // 256 bits of K per stage
constexpr int kFp4ColStride = kFp4ChunkWords * 32 + 16;     // LDS bytes per column of B codes
constexpr int kFp4ARowStride = kFp4ChunkWords * 8 + 8;      // LDS bytes per row of packed A

template <int RT, int CT>
__global__ __launch_bounds__(kBlock, 2) void bitgemm_fp4_kernel(
    const uint64_t *__restrict__ a, int64_t m, int64_t lda, const uint64_t *__restrict__ b, int n,
    int64_t ldb, int k_bits, const float *__restrict__ a_scale, const float *__restrict__ b_scale,
    int32_t *__restrict__ acc_out, int64_t ld_acc, float *__restrict__ out, int64_t ld_out)
{
    constexpr int kRows = kWavesPerBlock * 32 * RT;         // rows per workgroup
    constexpr int kCols = 32 * CT;                          // columns per workgroup
    constexpr int kAWords = kRows * kFp4ChunkWords / kBlock;    // words of A per thread and chunk (2 or 4)
    constexpr int kBWords = kCols * kFp4ChunkWords / kBlock;    // words of B per thread and chunk
    // two buffers: chunk c + 1 is staged while chunk c is multiplied
    __shared__ __attribute__((aligned(16))) unsigned char lds_b[2][kCols * kFp4ColStride];
    __shared__ __attribute__((aligned(16))) unsigned char lds_a[2][kRows * kFp4ARowStride];
    __shared__ int col_ones[kCols];
    const int n_words = (k_bits + 63) >> 6;
    const int lane = lane_id();
    const int wave = wave_in_block();
    const int i32 = lane & 31;
    const int half = lane >> 5;
    const int64_t block_row0 = static_cast<int64_t>(blockIdx.x) * kRows;
    const int64_t row0 = block_row0 + wave * 32 * RT;
    const int col0 = blockIdx.y * kCols;

    if (threadIdx.x < kCols) col_ones[threadIdx.x] = 0;

    v16f acc[RT][CT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rt][ct][r] = 0.0f;

    // staging shares of a thread: kAWords consecutive words of one row of A
    // (kFp4ChunkWords / kAWords threads share a row), kBWords words of B (column item / 4, word
    // item % 4, item = t + 256 u).  Addresses are recomputed at every fetch: the registers are
    // needed for the accumulators.
    static_assert(kFp4ChunkWords == 4, "item -> (column, word) below uses shifts");
    constexpr int kThreadsPerRow = kFp4ChunkWords / kAWords;
    const int a_thread_row = static_cast<int>(threadIdx.x) / kThreadsPerRow;
    const int a_thread_word = (static_cast<int>(threadIdx.x) % kThreadsPerRow) * kAWords;

    // two chunks are fetched ahead of the one being multiplied: two register sets, used alternately
    struct Fetched {
        uint64_t a[kAWords];
        uint64_t b[kBWords];
    };
    Fetched set0, set1;
    auto fetch = [&](int w0, Fetched &f) {
        int64_t row = block_row0 + a_thread_row;
        if (row >= m) row = m - 1;                              // clamped rows are never stored
        const uint64_t *src = a + row * lda + w0 + a_thread_word;
#pragma unroll
        for (int e = 0; e < kAWords; ++e) f.a[e] = (w0 + a_thread_word + e < n_words) ? src[e] : 0ull;
#pragma unroll
        for (int t = 0; t < kBWords; ++t) {
            const int item = static_cast<int>(threadIdx.x) + t * kBlock;
            const int j = col0 + (item >> 2);
            const int w = w0 + (item & 3);
            f.b[t] = (j < n && w < n_words) ? b[static_cast<int64_t>(j) * ldb + w] : 0ull;
        }
    };
    // w0: first word of the chunk that fetch() brought into f; buf: the LDS buffer to fill
    auto stage = [&](int w0, const Fetched &f, int buf) {
        uint2 *adst = reinterpret_cast<uint2 *>(lds_a[buf] + a_thread_row * kFp4ARowStride + a_thread_word * 8);
#pragma unroll
        for (int e = 0; e < kAWords; ++e)
            adst[e] = make_uint2(static_cast<uint32_t>(f.a[e]), static_cast<uint32_t>(f.a[e] >> 32));
        // 64 bits -> 64 codes (32 bytes): +1 -> 0x2, -1 -> 0xA, past K or past the last column -> 0x0
        const bool whole = (w0 + kFp4ChunkWords) * 64 <= k_bits && col0 + kCols <= n;   // uniform
        if (whole) {
            // every bit of the chunk counts: no masks
#pragma unroll
            for (int t = 0; t < kBWords; ++t) {
                const int item = static_cast<int>(threadIdx.x) + t * kBlock;
                const int c = item >> 2, q = item & 3;
                uint4 *dst = reinterpret_cast<uint4 *>(lds_b[buf] + c * kFp4ColStride + q * 32);
                atomicAdd(&col_ones[c], __popcll(f.b[t]));
#pragma unroll
                for (int part = 0; part < 2; ++part) dst[part] = fp4_codes_b(static_cast<uint32_t>(f.b[t] >> (32 * part)));
            }
            return;
        }
#pragma unroll
        for (int t = 0; t < kBWords; ++t) {
            const int item = static_cast<int>(threadIdx.x) + t * kBlock;
            const int c = item >> 2, q = item & 3;
            const int left = (col0 + c < n) ? k_bits - 64 * (w0 + q) : 0;        // bits of this word below K
            const uint64_t valid_bits = left >= 64 ? ~0ull : (left <= 0 ? 0ull : ((1ull << left) - 1ull));
            uint4 *dst = reinterpret_cast<uint4 *>(lds_b[buf] + c * kFp4ColStride + q * 32);
            const uint64_t word = f.b[t] & valid_bits;
            if (word != 0ull) atomicAdd(&col_ones[c], __popcll(word));
#pragma unroll
            for (int part = 0; part < 2; ++part) {
                const uint4 code = fp4_codes_b(static_cast<uint32_t>(f.b[t] >> (32 * part)));
                const uint4 keep = fp4_code_mask(static_cast<uint32_t>(valid_bits >> (32 * part)));
                dst[part] = make_uint4(code.x & keep.x, code.y & keep.y, code.z & keep.z, code.w & keep.w);
            }
        }
    };

    fetch(0, set0);
    if (kFp4ChunkWords < n_words) fetch(kFp4ChunkWords, set1);
    __syncthreads();                                      // col_ones cleared
    stage(0, set0, 0);
    __syncthreads();

    const int a_lane = (wave * 32 * RT + i32) * kFp4ARowStride + 4 * half;
    const int b_lane = i32 * kFp4ColStride + 16 * half;

    // multiply the chunk that starts at word w0 (it is in LDS buffer buf)
    auto multiply = [&](int w0, int buf) {
        auto step = [&](int q) {
            v8i aop[RT], bop[CT];
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                // this lane's 32 k of row 32 rt + i32
                const uint32_t bits = *reinterpret_cast<const uint32_t *>(lds_a[buf] + a_lane + 32 * rt * kFp4ARowStride + 8 * q);
                int codes[4];
                fp4_codes_a(bits, codes);
#pragma unroll
                for (int e = 0; e < 4; ++e) aop[rt][e] = codes[e];
                aop[rt][4] = aop[rt][5] = aop[rt][6] = aop[rt][7] = 0;
            }
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                const uint4 codes = *reinterpret_cast<const uint4 *>(lds_b[buf] + b_lane + 32 * ct * kFp4ColStride + 32 * q);
                bop[ct][0] = static_cast<int>(codes.x);
                bop[ct][1] = static_cast<int>(codes.y);
                bop[ct][2] = static_cast<int>(codes.z);
                bop[ct][3] = static_cast<int>(codes.w);
                bop[ct][4] = bop[ct][5] = bop[ct][6] = bop[ct][7] = 0;
            }
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int ct = 0; ct < CT; ++ct)
                    acc[rt][ct] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                        aop[rt], bop[ct], acc[rt][ct], 4, 4, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
        };
        if (w0 + kFp4ChunkWords <= n_words) {
            // a whole chunk: no exit between the steps, so their operands can be prepared ahead
#pragma unroll
            for (int q = 0; q < kFp4ChunkWords; ++q) step(q);
        } else {
            for (int q = 0; w0 + q < n_words; ++q) step(q);
        }
    };
    // Turn c: chunk c + 2 is fetched into the register set that chunk c was staged from, chunk c
    // (LDS buffer c % 2) is multiplied, chunk c + 1 is staged into the other buffer, one barrier.
    // That barrier publishes chunk c + 1 and tells that nobody reads buffer c % 2 any more, which
    // the next turn overwrites.  Two chunks per loop turn so that sets and buffers keep their names.
    for (int w0 = 0; w0 < n_words; w0 += 2 * kFp4ChunkWords) {
        const int w1 = w0 + kFp4ChunkWords, w2 = w0 + 2 * kFp4ChunkWords, w3 = w0 + 3 * kFp4ChunkWords;
        if (w2 < n_words) fetch(w2, set0);
        multiply(w0, 0);
        if (w1 >= n_words) break;                           // uniform
        stage(w1, set1, 1);
        __syncthreads();
        if (w3 < n_words) fetch(w3, set1);
        multiply(w1, 1);
        if (w2 < n_words) stage(w2, set0, 0);
        __syncthreads();
    }
    __syncthreads();                                        // col_ones complete for every wavefront

    // epilogue: c = 2 * acc - (2 popcount(B_j) - K)
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
        const int j = col0 + 32 * ct + i32;
        if (j >= n) continue;
        const int colsum = 2 * col_ones[32 * ct + i32] - k_bits;
        const float sb = out != nullptr ? b_scale[j] : 0.0f;
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = row0 + 32 * rt + 8 * (r >> 2) + 4 * half + (r & 3);
                if (row < m) {
                    const int c = 2 * static_cast<int>(acc[rt][ct][r]) - colsum;
                    if (acc_out != nullptr) acc_out[row * ld_acc + j] = c;
                    if (out != nullptr) out[row * ld_out + j] = a_scale[row] * sb * static_cast<float>(c);
                }
            }
        }
    }
}

template <int RT, int CT>
static int launch_bitgemm_fp4_t(const uint64_t *a_bits, const float *a_scale, int64_t m, int64_t lda,
                                const uint64_t *b_bits, const float *b_scale, int64_t n, int64_t ldb,
                                int64_t k_bits, int32_t *acc, int64_t ld_acc, float *out, int64_t ld_out,
                                hipStream_t stream)
{
    constexpr int kRows = kWavesPerBlock * 32 * RT, kCols = 32 * CT;
    const int64_t row_blocks = (m + kRows - 1) / kRows;
    const int64_t col_blocks = (n + kCols - 1) / kCols;
    if (row_blocks > 0x7fffffff || col_blocks > 65535) return BIGCN_ESHAPE;
    hipLaunchKernelGGL((bitgemm_fp4_kernel<RT, CT>), dim3(static_cast<unsigned>(row_blocks), static_cast<unsigned>(col_blocks)),
                       dim3(kBlock), 0, stream, a_bits, m, lda, b_bits, static_cast<int>(n), ldb,
                       static_cast<int>(k_bits), a_scale, b_scale, acc, ld_acc, out, ld_out);
    return check_launch();
}

// More than 64 columns: a wavefront owns 32 rows x 128 columns, so that an expanded A operand
// feeds four multiplies; otherwise 64 rows x 64 columns.  Either way 64 accumulator registers
// and three wavefronts per SIMD.
int launch_bitgemm_fp4(const uint64_t *a_bits, const float *a_scale, int64_t m, int64_t lda,
                       const uint64_t *b_bits, const float *b_scale, int64_t n, int64_t ldb,
                       int64_t k_bits, int32_t *acc, int64_t ld_acc, float *out, int64_t ld_out,
                       hipStream_t stream)
{
    if (fp4_tile_covers(m, n, k_bits, acc != nullptr ? ld_acc : 0, out != nullptr ? ld_out : 0, lda, ldb))
        return launch_bitgemm_fp4_tile(a_bits, a_scale, m, lda, b_bits, b_scale, n, ldb, k_bits, acc, ld_acc, out,
                                       ld_out, stream);
    if (n > 64)
        return launch_bitgemm_fp4_t<1, 4>(a_bits, a_scale, m, lda, b_bits, b_scale, n, ldb, k_bits, acc, ld_acc, out,
                                          ld_out, stream);
    return launch_bitgemm_fp4_t<2, 2>(a_bits, a_scale, m, lda, b_bits, b_scale, n, ldb, k_bits, acc, ld_acc, out,
                                      ld_out, stream);
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

// ---- product rows of the fused forward on the FP4 matrix cores (K <= 1024) ---------------------
// One-byte product rows of 64, 128, 256 or 512 stored positions (position p of a RowLayout holds
// column p / vec + groups (p % vec)).  Here the weights are the {0, +1} operand and the features
// the {-1, +1} one: with S = sum over the set weight bits of f_k and F = sum_k f_k, the product is
// 2 S - F and the stored value floor(K'/2) - popcount(f xor b) equals S - (F + K' mod 2) / 2, a
// constant per row, so the accumulators of a row start at 128 minus that constant and come out
// as value + 128.
// A block keeps the packed weights of all positions in LDS for its whole life, as
// [half-word of K][position] dwords (a lane's read is one dword, turned into codes by four
// masks and a shift, see fp4_rows_weight_codes); a wavefront owns 32 rows at a time.  Per tile of
// 128 positions (rows of 64 positions: one tile of 64): 4 (2) multiplies per 64 bits of K with
// the weights as first operand, so that the four registers of a group hold four consecutive
// positions of one row; the saturating byte conversion packs them, a flip of the top bits gives
// two's complement (values beyond a byte saturate and are caught by the 7-bit test), positions
// past the last column are zeroed, and the bytes go to the wavefront's LDS buffer
// [row][tile + 8].  Then 16 (8) lanes per row take 8 bytes each, test the 7-bit range where the
// layout asks for it (bit 7 differs from bit 6), stamp the scale (top bits of the carrier bytes,
// the last four bytes of the row, or the last byte of each of the last four lanes) and write
// the rows' pieces of the tile.  Rows with a value outside 7 bits are noted and, after the last
// tile, redone one at a time with XOR and bit counts from the same LDS weights: their values go
// to the alternate array (bytes or fp16) and the carrier bytes of the main row get a NaN scale,
// as in the vector-ALU kernels.  The bits and the scale of the next 32 rows are fetched while
// the current ones are multiplied.
struct Fp4RowsParams {
    int positions;        // 64, 128, 256 or 512
    int groups, vec;      // of the RowLayout
    int n;                // columns
    int k_bits;           // K' (without a folded last bit)
    int n_steps;          // ceil(K' / 64)
    int seven_bit;        // scale bits in the top bits of the carrier bytes
    int tail_scale;       // scale in the last four bytes
    int last_bytes;       // rows of 64 positions: scale byte i in the last byte of lane 4 + i
    int escape;           // rows outside the 7-bit range go to alt_rows
    int alt_half;         // ... as fp16 (else as bytes)
};

// A tile is 128 positions wide (64 for rows of 64 positions); bytes per row of a wavefront's LDS tile
__host__ __device__ constexpr int fp4_rows_tile(int positions) { return positions < 128 ? positions : 128; }
__host__ __device__ constexpr int fp4_rows_stride(int positions) { return fp4_rows_tile(positions) + 8; }

__host__ __device__ inline size_t fp4_rows_lds_bytes(int positions, int n_steps)
{
    return static_cast<size_t>(8) * n_steps * positions + positions +
           static_cast<size_t>(kWavesPerBlock) * 32 * fp4_rows_stride(positions);
}

// Codes of the rows kernel.  A set weight bit only has to multiply its feature by one, so the
// weight of dword d stays where its bit is inside the nibble (0x1 = 0.5, 0x2 = 1, 0x4 = 2; the
// fourth bit is moved to 0x2) and the feature codes of that dword carry the inverse magnitude
// (+-2, +-1, +-0.5, +-1): every product is exactly +-1 or 0, and a weight word costs four masks
// and one shift.  Same order of the k values as fp4_codes_a / fp4_codes_b.
__device__ __forceinline__ void fp4_rows_weight_codes(uint32_t x, int (&op)[4])
{
    op[0] = static_cast<int>(x & 0x11111111u);
    op[1] = static_cast<int>(x & 0x22222222u);
    op[2] = static_cast<int>(x & 0x44444444u);
    op[3] = static_cast<int>((x & 0x88888888u) >> 2);
}
__device__ __forceinline__ uint4 fp4_rows_feature_codes(uint32_t x)
{
    const uint32_t n = ~x;                                  // a clear bit is -1: sign bit of the code
    return make_uint4(((n & 0x11111111u) << 3) | 0x44444444u, ((n & 0x22222222u) << 2) | 0x22222222u,
                      ((n & 0x44444444u) << 1) | 0x11111111u, (n & 0x88888888u) | 0x22222222u);
}

// bits of the half-word (q, half) that lie below K'
__device__ __forceinline__ uint32_t fp4_rows_valid(int k_bits, int q, int half)
{
    const int left = k_bits - 64 * q - 32 * half;
    return left >= 32 ? ~0u : (left <= 0 ? 0u : ((1u << left) - 1u));
}

template <int P, int kMaxSteps>        // P stored positions; kMaxSteps 4: K' <= 256, 16: K' <= 1024
__global__ __launch_bounds__(kBlock, 3) void bitgemm_fp4_rows_kernel(
    const uint64_t *__restrict__ a, int64_t m, int64_t lda, const uint64_t *__restrict__ b, int64_t ldb,
    const float *__restrict__ src_scale, Fp4RowsParams p, unsigned char *__restrict__ rows,
    void *__restrict__ alt_rows, int *__restrict__ escape_flag)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char fp4_rows_lds[];
    constexpr int kTile = fp4_rows_tile(P);                  // positions per tile
    constexpr int kCt = kTile / 32;                          // 32 x 32 products per tile
    constexpr int kStride = fp4_rows_stride(P);
    constexpr int kSegs = kTile / 8;                         // lanes that write one row's piece of a tile
    constexpr int n_tiles = P / kTile;
    uint32_t *wbits = reinterpret_cast<uint32_t *>(fp4_rows_lds);               // [2 n_steps][P]
    unsigned char *live = fp4_rows_lds + static_cast<size_t>(8) * p.n_steps * P;   // [P]: 0xff below n columns
    const int lane = lane_id();
    const int wave = wave_in_block();
    const int i32 = lane & 31, half = lane >> 5;
    unsigned char *mine = live + P + wave * 32 * kStride;
    const uint32_t *wlane = wbits + half * P + i32;           // this lane's weight words: + 2 q P + position of tile
    const unsigned char *live_lane = live + 4 * half;
    unsigned char *mine_lane = mine + i32 * kStride + 4 * half;
    const int64_t wave_id = static_cast<int64_t>(blockIdx.x) * kWavesPerBlock + wave;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kWavesPerBlock * 32;

    for (int item = threadIdx.x; item < P * p.n_steps; item += kBlock) {
        const int q = item / P, pos = item - q * P;
        const int col = pos / p.vec + p.groups * (pos % p.vec);
        const uint64_t word = col < p.n ? b[static_cast<int64_t>(col) * ldb + q] : 0ull;
        wbits[(2 * q) * P + pos] = static_cast<uint32_t>(word);
        wbits[(2 * q + 1) * P + pos] = static_cast<uint32_t>(word >> 32);
        if (q == 0) live[pos] = col < p.n ? 0xffu : 0u;
    }
    __syncthreads();

    // half-words 2 q + half and scale of row r0 + i32 (clamped: such rows are never stored)
    uint32_t next[kMaxSteps], next_scale;
    auto fetch = [&](int64_t r0) {
        int64_t arow = r0 + i32;
        if (arow >= m) arow = m - 1;
        const uint32_t *src = reinterpret_cast<const uint32_t *>(a + arow * lda) + half;
#pragma unroll
        for (int q = 0; q < kMaxSteps; ++q) next[q] = q < p.n_steps ? src[2 * q] : 0u;
        next_scale = src_scale != nullptr ? __float_as_uint(src_scale[arow]) : 0u;
    };
    int64_t row0 = wave_id * 32;
    fetch(row0);
    for (; row0 < m; row0 += stride) {
        uint32_t cur[kMaxSteps];
        int ones = 0;
#pragma unroll
        for (int q = 0; q < kMaxSteps; ++q) {
            cur[q] = next[q] & fp4_rows_valid(p.k_bits, q, half);
            ones += __popc(cur[q]);
        }
        ones += __shfl_xor(ones, 32);
        // (F + K' mod 2) / 2 with F = 2 ones - K': an even number halved
        const float start = 128.0f - static_cast<float>((2 * ones - p.k_bits + (p.k_bits & 1)) / 2);
        if (half == 0) *reinterpret_cast<uint32_t *>(mine + i32 * kStride + kTile) = next_scale;
        fetch(row0 + stride);
        uint32_t escaped = 0;                                 // rows of this wavefront's 32 that need the alternate array
#pragma unroll 1
        for (int t = 0; t < n_tiles; ++t) {
            // register 4 g + e of tile ct: position 128 t + 32 ct + 8 g + 4 half + e, row i32
            v16f acc[kCt];
#pragma unroll
            for (int ct = 0; ct < kCt; ++ct)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[ct][r] = start;
#pragma unroll
            for (int q = 0; q < kMaxSteps; ++q) {
                if (q >= p.n_steps) break;                    // uniform
                uint4 code = fp4_rows_feature_codes(cur[q]);
                if (q == p.n_steps - 1) {
                    const uint4 keep = fp4_code_mask(fp4_rows_valid(p.k_bits, q, half));
                    code = make_uint4(code.x & keep.x, code.y & keep.y, code.z & keep.z, code.w & keep.w);
                }
                v8i fop;
                fop[0] = static_cast<int>(code.x);
                fop[1] = static_cast<int>(code.y);
                fop[2] = static_cast<int>(code.z);
                fop[3] = static_cast<int>(code.w);
                fop[4] = fop[5] = fop[6] = fop[7] = 0;
#pragma unroll
                for (int ct = 0; ct < kCt; ++ct) {
                    int wcodes[4];
                    fp4_rows_weight_codes(wlane[2 * q * P + kTile * t + 32 * ct], wcodes);
                    v8i wop;
#pragma unroll
                    for (int e = 0; e < 4; ++e) wop[e] = wcodes[e];
                    wop[4] = wop[5] = wop[6] = wop[7] = 0;
                    acc[ct] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(wop, fop, acc[ct], 4, 4, 0, 0x7f7f7f7f, 0,
                                                                             0x7f7f7f7f);
                }
            }
#pragma unroll
            for (int ct = 0; ct < kCt; ++ct)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    uint32_t packed = 0;
#pragma unroll
                    for (int e = 0; e < 4; ++e) packed = __builtin_amdgcn_cvt_pk_u8_f32(acc[ct][4 * g + e], e, packed);
                    const uint32_t keep = *reinterpret_cast<const uint32_t *>(live_lane + kTile * t + 32 * ct + 8 * g);
                    *reinterpret_cast<uint32_t *>(mine_lane + 32 * ct + 8 * g) = (packed ^ 0x80808080u) & keep;
                }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            // this tile's piece of every row: kSegs lanes per row, 8 bytes each
            const int seg = lane & (kSegs - 1), sub = lane / kSegs;
            const int row_seg = kSegs * t + seg;              // 8-byte segment of the whole row
#pragma unroll 4
            for (int j = 0; j < 32; j += kWave / kSegs) {
                const int local = j + sub;
                const int64_t row = row0 + local;
                uint2 v = *reinterpret_cast<const uint2 *>(mine + local * kStride + 8 * seg);
                const uint32_t row_scale = *reinterpret_cast<const uint32_t *>(mine + local * kStride + kTile);
                if (p.seven_bit) {
                    if (kSegs == 16 && p.escape) {
                        // a byte fits 7 bits when its bits 7 and 6 agree
                        const bool misfit = (((v.x ^ (v.x << 1)) | (v.y ^ (v.y << 1))) & 0x80808080u) != 0u;
                        const uint64_t any = __ballot(misfit);
                        const uint32_t four = ((any & 0xffffull) != 0ull ? 1u : 0u) | ((any & 0xffff0000ull) != 0ull ? 2u : 0u) |
                                              ((any & 0xffff00000000ull) != 0ull ? 4u : 0u) | ((any >> 48) != 0ull ? 8u : 0u);
                        escaped |= four << j;
                    }
                    // carrier bytes: byte 0 of segment i carries bit i (i < 32); rows of 16 lanes carry
                    // bits 16..31 in byte 4
                    if (row_seg < 32) v.x = (v.x & ~0x80u) | (((row_scale >> row_seg) & 1u) << 7);
                    if (P == 128) v.y = (v.y & ~0x80u) | (((row_scale >> (16 + seg)) & 1u) << 7);
                } else if (p.tail_scale) {
                    if (t == n_tiles - 1 && seg == kSegs - 1) v.y = row_scale;
                } else if (p.last_bytes) {
                    if (kSegs == 8 && p.escape) {
                        // 8-bit values: 0x80 and 0x7f are where the conversion saturates, so a row
                        // holding either is taken as not fitting (dead positions hold 0)
                        const uint32_t lo_x = v.x ^ 0x80808080u, hi_x = v.x ^ 0x7f7f7f7fu;
                        const uint32_t lo_y = v.y ^ 0x80808080u, hi_y = v.y ^ 0x7f7f7f7fu;
                        const uint32_t zero = ((lo_x - 0x01010101u) & ~lo_x) | ((hi_x - 0x01010101u) & ~hi_x) |
                                              ((lo_y - 0x01010101u) & ~lo_y) | ((hi_y - 0x01010101u) & ~hi_y);
                        const uint64_t any = __ballot((zero & 0x80808080u) != 0u);
                        uint32_t eight = 0;
#pragma unroll
                        for (int r = 0; r < 8; ++r) eight |= ((any >> (8 * r)) & 0xffull) != 0ull ? (1u << r) : 0u;
                        escaped |= eight << j;
                    }
                    // rows of 8 lanes: byte i of the scale is the last byte of lane 4 + i
                    if (seg >= kSegs - 4) v.y = (v.y & 0x00ffffffu) | (((row_scale >> (8 * (seg - (kSegs - 4)))) & 0xffu) << 24);
                }
                if (row < m) *reinterpret_cast<uint2 *>(rows + row * P + kTile * t + 8 * seg) = v;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();                  // the buffer is rewritten by the next tile
        }
        if (escaped != 0u) {
            if (escape_flag != nullptr) *escape_flag = 1;
            // the main rows are complete in memory before their carrier bytes are written again
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            uint32_t todo = escaped;
            while (todo != 0u) {
                const int local = __builtin_amdgcn_readfirstlane(__builtin_ctz(todo));
                todo &= todo - 1u;
                const int64_t row = row0 + local;
                if (row >= m) continue;
                const uint64_t *bits_of_row = a + row * lda;  // uniform: every lane reads the same words
                for (int pos = lane; pos < P; pos += kWave) {
                    int pop = 0;
                    for (int q = 0; q < p.n_steps; ++q) {
                        const uint64_t f = bits_of_row[q];
                        pop += __popc((static_cast<uint32_t>(f) ^ wbits[(2 * q) * P + pos]) & fp4_rows_valid(p.k_bits, q, 0));
                        pop += __popc((static_cast<uint32_t>(f >> 32) ^ wbits[(2 * q + 1) * P + pos]) &
                                      fp4_rows_valid(p.k_bits, q, 1));
                    }
                    const int value = live[pos] != 0 ? (p.k_bits >> 1) - pop : 0;
                    if (p.alt_half)
                        static_cast<__half *>(alt_rows)[row * P + pos] = __float2half(static_cast<float>(value));
                    else
                        static_cast<signed char *>(alt_rows)[row * P + pos] = static_cast<signed char>(value);
                    const int segment = pos >> 3, offset = pos & 7;
                    if (p.last_bytes) {
                        // the NaN scale, byte by byte, behind the values of the last four lanes
                        if (offset == 7 && segment >= P / 8 - 4)
                            rows[row * P + pos] = static_cast<unsigned char>((0x7fc00000u >> (8 * (segment - (P / 8 - 4)))) & 0xffu);
                        continue;
                    }
                    int bit = -1;
                    if (offset == 0 && segment < 32) bit = segment;
                    else if (offset == 4 && P == 128) bit = 16 + segment;
                    if (bit >= 0)
                        rows[row * P + pos] = static_cast<unsigned char>((static_cast<uint32_t>(value) & 0x7fu) |
                                                                        (((0x7fc00000u >> bit) & 1u) << 7));
                }
            }
        }
    }
}

// Product rows of `layout` on the FP4 matrix cores: one byte per value, 64 / 128 / 256 / 512 stored
// positions, K <= 1024 with the packed weights fitting 64 KB of LDS beside the row tiles, more
// than 32768 rows.  Returns BIGCN_EINVAL without launching anything when the shape is not covered.
bool fp4_rows_covers(int64_t m, int64_t k_bits, const RowLayout &layout)
{
    const int pos = layout.positions();
    if (layout.kind != kI8 || k_bits > 1024 || m <= 32768) return false;
    if (pos != 64 && pos != 128 && pos != 256 && pos != 512) return false;
    if (pos == 64 && (layout.embed_scale == kScaleInTopBits || layout.groups != 8)) return false;
    if (layout.embed_scale == kScaleInLastBytes && pos != 64) return false;
    if (layout.escape && layout.alt_kind != kI8 && layout.alt_kind != kF16) return false;
    if (layout.escape && layout.embed_scale == kScaleInLastBytes && layout.alt_kind != kF16) return false;
    if (layout.escape && layout.embed_scale != kScaleInTopBits && layout.embed_scale != kScaleInLastBytes) return false;
    return fp4_rows_lds_bytes(pos, (layout.k_eff + 63) / 64) <= 64 * 1024;
}

// blocks of the kernel that a compute unit holds at once (asked once per LDS size)
template <int P, int kMaxSteps>
static int launch_fp4_rows(const uint64_t *a_bits, int64_t m, int64_t lda, const uint64_t *b_bits, int64_t ldb,
                           const float *scale, const Fp4RowsParams &p, void *c_rows, void *alt_rows, hipStream_t stream,
                           int *escape_flag)
{
    const size_t lds_bytes = fp4_rows_lds_bytes(P, p.n_steps);
    static std::atomic<int> known[257];
    const size_t slot = lds_bytes / 256;
    int per_cu = known[slot].load(std::memory_order_relaxed);
    if (per_cu == 0) {
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, bitgemm_fp4_rows_kernel<P, kMaxSteps>, kBlock,
                                                         lds_bytes) != hipSuccess || per_cu < 1) {
            (void)hipGetLastError();                          // the query's failure is not the launch's
            per_cu = 1;
        }
        known[slot].store(per_cu, std::memory_order_relaxed);
    }
    // the blocks stay for the whole call (each loads the weights once): as many as are resident at once
    int64_t blocks = (m + 127) / 128;
    if (blocks > static_cast<int64_t>(compute_units()) * per_cu) blocks = static_cast<int64_t>(compute_units()) * per_cu;
    hipLaunchKernelGGL((bitgemm_fp4_rows_kernel<P, kMaxSteps>), dim3(static_cast<unsigned>(blocks)), dim3(kBlock), lds_bytes,
                       stream, a_bits, m, lda, b_bits, ldb, scale, p, static_cast<unsigned char *>(c_rows), alt_rows, escape_flag);
    return check_launch();
}

int launch_bitgemm_fp4_rows(const uint64_t *a_bits, int64_t m, int64_t lda, const uint64_t *b_bits, int64_t n,
                            int64_t ldb, int64_t k_bits, const float *src_scale, void *c_rows, void *alt_rows,
                            RowLayout layout, hipStream_t stream, int *escape_flag)
{
    if (!fp4_rows_covers(m, k_bits, layout)) return BIGCN_EINVAL;
    if (layout.escape && alt_rows == nullptr) return BIGCN_ENULL;
    if (layout.embed_scale != kScaleSeparate && src_scale == nullptr) return BIGCN_ENULL;
    Fp4RowsParams p;
    p.positions = layout.positions();
    p.groups = layout.groups;
    p.vec = layout.vec;
    p.n = static_cast<int>(n);
    p.k_bits = layout.k_eff;
    p.n_steps = (layout.k_eff + 63) / 64;
    p.seven_bit = layout.embed_scale == kScaleInTopBits ? 1 : 0;
    p.tail_scale = layout.embed_scale == kScaleInTail ? 1 : 0;
    p.last_bytes = layout.embed_scale == kScaleInLastBytes ? 1 : 0;
    p.escape = layout.escape;
    p.alt_half = layout.alt_kind == kF16 ? 1 : 0;
    const float *scale = layout.embed_scale != kScaleSeparate ? src_scale : nullptr;
    // K' <= 256 has an instantiation of its own (four K steps unrolled) only for rows of 64 and 128
    // positions: for wider rows the general one needs fewer registers and is the faster
    // (c5, 256 positions: 0.18 / 0.25 ms against 0.21 / 0.28 ms for its layers of 100 and 256 bits).
    const bool narrow = p.n_steps <= 4;
    switch (p.positions) {
    case 64:
        return narrow ? launch_fp4_rows<64, 4>(a_bits, m, lda, b_bits, ldb, scale, p, c_rows, alt_rows, stream, escape_flag)
                      : launch_fp4_rows<64, 16>(a_bits, m, lda, b_bits, ldb, scale, p, c_rows, alt_rows, stream, escape_flag);
    case 128:
        return narrow ? launch_fp4_rows<128, 4>(a_bits, m, lda, b_bits, ldb, scale, p, c_rows, alt_rows, stream, escape_flag)
                      : launch_fp4_rows<128, 16>(a_bits, m, lda, b_bits, ldb, scale, p, c_rows, alt_rows, stream, escape_flag);
    case 256:
        return launch_fp4_rows<256, 16>(a_bits, m, lda, b_bits, ldb, scale, p, c_rows, alt_rows, stream, escape_flag);
    default:
        return launch_fp4_rows<512, 16>(a_bits, m, lda, b_bits, ldb, scale, p, c_rows, alt_rows, stream, escape_flag);
    }
}

// One-byte product rows in column order (position = column, no scale inside the row) on the same
// kernel: the consumers that read a row's columns next to each other (the Bi-GAT kernels).
bool fp4_natural_covers(int64_t m, int64_t k_bits, int positions)
{
    if (k_bits > 255 || m <= 32768) return false;
    if (positions != 64 && positions != 128 && positions != 256 && positions != 512) return false;
    return fp4_rows_lds_bytes(positions, static_cast<int>((k_bits + 63) / 64)) <= 64 * 1024;
}

int launch_bitgemm_fp4_natural(const uint64_t *a_bits, int64_t m, int64_t lda, const uint64_t *b_bits, int64_t n,
                               int64_t ldb, int64_t k_bits, void *rows, int positions, hipStream_t stream)
{
    if (!fp4_natural_covers(m, k_bits, positions) || n > positions) return BIGCN_EINVAL;
    Fp4RowsParams p;
    p.positions = positions;
    p.groups = positions;             // position p holds column p / vec + groups (p % vec) = p
    p.vec = 1;
    p.n = static_cast<int>(n);
    p.k_bits = static_cast<int>(k_bits);
    p.n_steps = static_cast<int>((k_bits + 63) / 64);
    p.seven_bit = 0;
    p.tail_scale = 0;
    p.last_bytes = 0;
    p.escape = 0;
    p.alt_half = 0;
    switch (positions) {
    case 64:
        return launch_fp4_rows<64, 4>(a_bits, m, lda, b_bits, ldb, nullptr, p, rows, nullptr, stream, nullptr);
    case 128:
        return launch_fp4_rows<128, 4>(a_bits, m, lda, b_bits, ldb, nullptr, p, rows, nullptr, stream, nullptr);
    case 256:
        return launch_fp4_rows<256, 16>(a_bits, m, lda, b_bits, ldb, nullptr, p, rows, nullptr, stream, nullptr);
    default:
        return launch_fp4_rows<512, 16>(a_bits, m, lda, b_bits, ldb, nullptr, p, rows, nullptr, stream, nullptr);
    }
}

}  // namespace bigcn
