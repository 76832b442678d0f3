// Kernel 2: binary matrix product  c_ij = K - 2*popcount(a_i xor b_j)  with the fused
// rescale  zeta_ij = beta_i * alpha_j * c_ij  (Sec. 4.2.3: XNOR + bit count in place of the
// floating-point inner product of two +-1 vectors).
//
// Mapping (wave64, integer VALU path): the 64 lanes of a wavefront own 64 * VB output
// columns of a row block; the packed rows of B for those columns live in LDS as
// [word][lane + 64 v] so that a wavefront reads 512 contiguous bytes per access; the
// wavefront walks R rows of A at a time, and because all 64 lanes work on the same row of
// A its words are wave-uniform (scalar loads, XOR with a scalar operand).  Per 64 binary
// multiply-accumulates a lane issues two v_xor_b32 and two v_bcnt_u32_b32 (the bit count
// accumulates for free), which is the integer-VALU roofline of the operation.
//
// Which columns a lane owns is a parameter (ColumnMap), so that the values a lane produces
// are consecutive in the destination: row-major columns l, l+64, ... for the public entry
// point, and the interleaved product-row layout of the fused forward otherwise.
#include "bigcn_internal.h"

namespace bigcn {

bool prefer_mfma(int64_t m, int64_t n, int64_t k_bits);

// Lane l, local index v (0..VB-1), column block y:
//   value index inside the stored row   vv  = per_group * (l / groups) + y * VB + v
//   output column                       col = (l % groups) + groups * vv
//   stored position                     pos = (l % groups) * vec + vv
// The public entry point uses groups = 64, per_group = vec = VB * gridDim.y, i.e.
// col = l + 64 * (y * VB + v), and ignores pos.
struct ColumnMap {
    int groups;
    int vec;
    int per_group;   // values of one lane across all column blocks
};

// ---- epilogues ---------------------------------------------------------------------------
// Public entry point: int32 accumulators and / or rescaled fp32, row-major.
struct EpilogueApi {
    const float *a_scale;
    const float *b_scale;
    int32_t *acc;
    int64_t ld_acc;
    float *out;
    int64_t ld_out;
    int k_bits;
    template <int VB>
    struct Lane {
        float b_scale[VB];   // per-lane constants: the scales of this lane's columns
    };
    template <int VB>
    __device__ __forceinline__ void init(const int (&col)[VB], int /*pos0*/, int n, Lane<VB> &c) const
    {
#pragma unroll
        for (int v = 0; v < VB; ++v)
            c.b_scale[v] = (out != nullptr && col[v] >= 0 && col[v] < n) ? b_scale[col[v]] : 0.0f;
    }
    // per-row value needed by store(): fetched when the row block starts, not when it ends
    __device__ __forceinline__ float row_value(int64_t row) const { return out != nullptr ? a_scale[row] : 0.0f; }
    // start value of the bit counters (store() receives counters that include it)
    __device__ __forceinline__ int pop_init() const { return 0; }
    template <int VB>
    __device__ __forceinline__ void store(const Lane<VB> &ctx, int64_t row, float sa, const int (&col)[VB],
                                          int /*pos0*/, bool /*any*/, int n, const int (&pop)[VB]) const
    {
#pragma unroll
        for (int v = 0; v < VB; ++v) {
            const int j = col[v];
            if (j >= 0 && j < n) {
                const int c = k_bits - 2 * pop[v];
                if (acc != nullptr) acc[row * ld_acc + j] = c;
                if (out != nullptr) out[row * ld_out + j] = sa * ctx.b_scale[v] * static_cast<float>(c);
            }
        }
    }
};

// Fused forward: one product row per node in a RowLayout.  T = int8_t stores
// floor(K'/2) - pop, T = __half / float store K' - 2 pop; a lane's VB values are consecutive.
template <typename T>
struct EpilogueLayout {
    T *rows;
    int positions;
    int k_eff;
    const float *embed;      // non-null (int8 rows only): scale[row] is stored inside the row,
    int top_bits_shift;      //   0: in its last 4 bytes; 3: bit i in the top bit of position 8 i (i < 32) and,
    int top_bits_groups;     //   for rows of 16 lanes, bits 16..31 in the top bit of position 8 (i - 16) + 4;
                             //   -1: byte i at position 8 (groups - 4 + i) + 7 (rows of 8 lanes x 8 values)
    void *alt_rows;          // escape layouts: rows with a value outside [-64, 63] are written here (one
    int alt_half;            // byte per value, or one fp16 when alt_half) and get a NaN scale in the
                             // main array; else nullptr
    int *escape_flag;        // nullable: set to 1 whenever a row goes to alt_rows
    template <int VB>
    struct Lane {
        int top_bit;         // which bit of the scale this lane's first value carries, or -1
    };
    template <int VB>
    __device__ __forceinline__ void init(const int (&)[VB], int pos0, int, Lane<VB> &c) const
    {
        // a lane's values are consecutive positions starting at a multiple of VB, and carriers sit
        // on multiples of 4 (of 8 when VB = 8), so only a lane's first value can be a carrier
        c.top_bit = -1;
        if (top_bits_shift > 0 && embed != nullptr) {
            const int segment = pos0 >> 3, offset = pos0 & 7;
            if (offset == 0 && segment < 32) c.top_bit = segment;
            else if (offset == 4 && top_bits_groups == 16) c.top_bit = 16 + segment;
        }
    }
    __device__ __forceinline__ float row_value(int64_t row) const { return embed != nullptr ? embed[row] : 0.0f; }
    // 7-bit layouts (scale in the top bits) count from 63 - floor(K'/2): the stored value
    // floor(K'/2) - popcount is then 63 - counter.  It fits 7 bits exactly when the counter lies in
    // [0, 127], i.e. has no bit above bit 6 (one OR over a lane's counters and one test decide it),
    // and its 7-bit two's-complement code is then simply counter ^ 0x3f, so four counters are
    // packed into bytes first and complemented, sign-extended and stamped as one word.
    __device__ __forceinline__ int pop_init() const { return top_bits_shift > 0 ? 63 - (k_eff >> 1) : 0; }
    template <int VB>
    __device__ __forceinline__ void store(const Lane<VB> &ctx, int64_t row, float row_scale, const int (&col)[VB],
                                          int pos0, bool any, int n, const int (&pop)[VB]) const
    {
        if (!any) return;
        if constexpr (sizeof(T) == 1) {
            if (top_bits_shift > 0) {
                store_seven_bit<VB>(ctx, row, row_scale, col, pos0, n, pop);
                return;
            }
        }
        alignas(16) T tmp[VB];
        const int bias = pop_init();
        const int half_k = (k_eff >> 1) + bias;             // value = half_k - (counter incl. bias)
#pragma unroll
        for (int v = 0; v < VB; ++v) {
            const bool live = col[v] >= 0 && col[v] < n;
            if constexpr (sizeof(T) == 1) {
                tmp[v] = static_cast<T>(live ? half_k - pop[v] : 0);
            } else {
                const int value = k_eff - 2 * pop[v];
                tmp[v] = static_cast<T>(live ? static_cast<float>(value) : 0.0f);
            }
        }
        if constexpr (sizeof(T) == 1) {
            if (alt_rows != nullptr) {
                // 8-bit rows of more than 256 input bits (fp16 alternates; the scale sits in the
                // last bytes).  One wavefront holds the whole row: if any value lies outside
                // [-127, 126] (the range the matrix-core kernel can tell from a saturated byte) the
                // row goes to the alternate array and the main array gets a NaN scale
                bool misfit = false;
#pragma unroll
                for (int v = 0; v < VB; ++v) {
                    const int value = half_k - pop[v];
                    misfit = misfit || (col[v] >= 0 && col[v] < n && (value < -127 || value > 126));
                }
                if (__ballot(misfit) != 0ull) {
                    if (escape_flag != nullptr) *escape_flag = 1;
                    alignas(16) __half wide[VB];
#pragma unroll
                    for (int v = 0; v < VB; ++v)
                        wide[v] = __float2half((col[v] >= 0 && col[v] < n) ? static_cast<float>(half_k - pop[v]) : 0.0f);
                    EpilogueLayout<__half>::template write_values<VB>(static_cast<__half *>(alt_rows) + row * positions + pos0,
                                                                      wide);
                    row_scale = __uint_as_float(0x7fc00000u);
                }
            }
            if (embed != nullptr && top_bits_shift == 0) {
                const uint32_t bits = __float_as_uint(row_scale);
#pragma unroll
                for (int v = 0; v < VB; ++v) {
                    const int byte = pos0 + v - (positions - 4);
                    if (byte >= 0) tmp[v] = static_cast<T>((bits >> (8 * byte)) & 0xffu);
                }
            } else if (embed != nullptr && top_bits_shift < 0) {
                const uint32_t bits = __float_as_uint(row_scale);
#pragma unroll
                for (int v = 0; v < VB; ++v) {
                    const int p = pos0 + v, byte = (p >> 3) - (top_bits_groups - 4);
                    if ((p & 7) == 7 && byte >= 0) tmp[v] = static_cast<T>((bits >> (8 * byte)) & 0xffu);
                }
            } else if (ctx.top_bit >= 0) {
                const uint32_t bit = (__float_as_uint(row_scale) >> ctx.top_bit) & 1u;
                tmp[0] = static_cast<T>((static_cast<uint32_t>(tmp[0]) & 0x7fu) | (bit << 7));
            }
        }
        write_values<VB>(rows + row * positions + pos0, tmp);
    }
    // store() for the 7-bit layouts (see pop_init).
    template <int VB>
    __device__ __forceinline__ void store_seven_bit(const Lane<VB> &ctx, int64_t row, float row_scale,
                                                    const int (&col)[VB], int pos0, int n,
                                                    const int (&pop)[VB]) const
    {
        uint32_t c[VB];
        uint32_t spread = 0;
#pragma unroll
        for (int v = 0; v < VB; ++v) {
            const bool live = col[v] >= 0 && col[v] < n;
            c[v] = live ? static_cast<uint32_t>(pop[v]) : 63u;       // a dead position stores 0
            spread |= c[v];
        }
        if (alt_rows != nullptr) {
            // one wavefront holds the whole row: if any value needs the eighth bit the row goes to
            // the alternate array (bytes or fp16) and the main array gets a NaN scale
            if (__ballot((spread & ~127u) != 0u) != 0ull) {
                if (escape_flag != nullptr) *escape_flag = 1;
                if (alt_half) {
                    alignas(16) __half tmp[VB];
#pragma unroll
                    for (int v = 0; v < VB; ++v)
                        tmp[v] = __float2half(static_cast<float>(63 - static_cast<int>(c[v])));
                    EpilogueLayout<__half>::template write_values<VB>(
                        static_cast<__half *>(alt_rows) + row * positions + pos0, tmp);
                } else {
                    alignas(16) T tmp[VB];
#pragma unroll
                    for (int v = 0; v < VB; ++v) tmp[v] = static_cast<T>(63 - static_cast<int>(c[v]));
                    write_values<VB>(static_cast<T *>(alt_rows) + row * positions + pos0, tmp);
                }
                row_scale = __uint_as_float(0x7fc00000u);
            }
        }
        constexpr int kWords = VB > 4 ? VB / 4 : 1;
        uint32_t words[kWords];
#pragma unroll
        for (int q = 0; q < kWords; ++q) {
            uint32_t x = 0;
#pragma unroll
            for (int e = 0; e < 4 && 4 * q + e < VB; ++e) x |= (c[4 * q + e] & 0xffu) << (8 * e);
            x ^= 0x3f3f3f3fu;
            x = (x & 0x7f7f7f7fu) | ((x & 0x40404040u) << 1);          // copy bit 6 into bit 7
            words[q] = x;
        }
        if (ctx.top_bit >= 0) {
            const uint32_t bit = (__float_as_uint(row_scale) >> ctx.top_bit) & 1u;
            words[0] = (words[0] & ~0x80u) | (bit << 7);
        }
        T *p = rows + row * positions + pos0;
        if constexpr (VB == 8) *reinterpret_cast<uint2 *>(p) = make_uint2(words[0], words[1]);
        else if constexpr (VB == 4) *reinterpret_cast<uint32_t *>(p) = words[0];
        else if constexpr (VB == 2) *reinterpret_cast<uint16_t *>(p) = static_cast<uint16_t>(words[0]);
        else *reinterpret_cast<uint8_t *>(p) = static_cast<uint8_t>(words[0]);
    }
    template <int VB>
    static __device__ __forceinline__ void write_values(T *p, const T (&tmp)[VB])
    {
        constexpr int kBytes = sizeof(T) * VB;
        if constexpr (kBytes == 16) *reinterpret_cast<uint4 *>(p) = *reinterpret_cast<const uint4 *>(tmp);
        else if constexpr (kBytes == 8) *reinterpret_cast<uint2 *>(p) = *reinterpret_cast<const uint2 *>(tmp);
        else if constexpr (kBytes == 4) *reinterpret_cast<uint32_t *>(p) = *reinterpret_cast<const uint32_t *>(tmp);
        else if constexpr (kBytes == 2) *reinterpret_cast<uint16_t *>(p) = *reinterpret_cast<const uint16_t *>(tmp);
        else if constexpr (kBytes == 32) {
            reinterpret_cast<uint4 *>(p)[0] = reinterpret_cast<const uint4 *>(tmp)[0];
            reinterpret_cast<uint4 *>(p)[1] = reinterpret_cast<const uint4 *>(tmp)[1];
        } else {
#pragma unroll
            for (int v = 0; v < VB; ++v) p[v] = tmp[v];
        }
    }
};

// Stage the packed rows of B for the columns of column block y into LDS ([n_words][64*VB]; slot c
// belongs to lane c % 64), with last_mask applied to the last word; ends with a barrier.
template <int VB>
__device__ __forceinline__ void stage_b_block(uint64_t *lds_b, const uint64_t *__restrict__ b, int n, int64_t ldb,
                                              int n_words, uint32_t last_mask, const ColumnMap &map, int y)
{
    constexpr int CB = 64 * VB;
    constexpr int kBatch = 4;         // loads of a thread in flight together
    const int total = CB * n_words;
    for (int idx0 = threadIdx.x; idx0 < total; idx0 += kBlock * kBatch) {
        uint64_t word[kBatch];
        int slot[kBatch];
#pragma unroll
        for (int q = 0; q < kBatch; ++q) {
            const int idx = idx0 + q * kBlock;
            const int c = idx / n_words;
            const int w = idx - c * n_words;
            const int l = c & 63, v = c >> 6;
            const int vv = map.per_group * (l / map.groups) + y * VB + v;
            const int j = (l % map.groups) + map.groups * vv;
            word[q] = (idx < total && vv < map.vec && j < n) ? b[static_cast<int64_t>(j) * ldb + w] : 0ull;
            if (w == n_words - 1) word[q] &= (static_cast<uint64_t>(last_mask) << 32) | 0xffffffffull;
            slot[q] = idx < total ? w * CB + c : -1;
        }
#pragma unroll
        for (int q = 0; q < kBatch; ++q)
            if (slot[q] >= 0) lds_b[slot[q]] = word[q];
    }
    __syncthreads();
}

// The output columns of a lane's VB values in column block y (-1: none), whether it has any,
// and (returned) the stored position of its first value.
template <int VB>
__device__ __forceinline__ int lane_columns(const ColumnMap &map, int y, int lane, int (&col)[VB], bool &any)
{
    any = false;
#pragma unroll
    for (int v = 0; v < VB; ++v) {
        const int vv = map.per_group * (lane / map.groups) + y * VB + v;
        col[v] = vv < map.vec ? (lane % map.groups) + map.groups * vv : -1;
        any = any || vv < map.vec;
    }
    return (lane % map.groups) * map.vec + map.per_group * (lane / map.groups) + y * VB;
}

// ---- the kernel -----------------------------------------------------------------------------
// grid.x walks row blocks (grid-stride), grid.y is the column block.  last_mask is ANDed onto
// the high half of the last word of both operands (all ones, or bit 31 cleared to leave the
// last of 64*n_words bits out of the count).
template <int VB, int R, class Epilogue>
__global__ __launch_bounds__(kBlock) void bitgemm_kernel(
    const uint64_t *__restrict__ a, int64_t m, int64_t lda, const uint64_t *__restrict__ b, int n,
    int64_t ldb, int n_words, uint32_t last_mask, ColumnMap map, Epilogue epi)
{
    extern __shared__ uint64_t lds_b[];          // [n_words][64*VB]
    constexpr int CB = 64 * VB;
    const int y = blockIdx.y;
    stage_b_block<VB>(lds_b, b, n, ldb, n_words, last_mask, map, y);
    const uint2 *lds_b2 = reinterpret_cast<const uint2 *>(lds_b);

    const int lane = lane_id();
    int col[VB];
    bool any;
    const int pos0 = lane_columns<VB>(map, y, lane, col, any);
    typename Epilogue::template Lane<VB> ctx;
    epi.template init<VB>(col, pos0, n, ctx);

    const int64_t wave = static_cast<int64_t>(blockIdx.x) * kWavesPerBlock + wave_in_block();
    const int64_t n_waves = static_cast<int64_t>(gridDim.x) * kWavesPerBlock;

    for (int64_t row0 = wave * R; row0 < m; row0 += n_waves * R) {
        int pop[R][VB];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int v = 0; v < VB; ++v) pop[r][v] = epi.pop_init();

        const uint32_t *arow[R];
        float row_value[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int64_t row = row0 + r < m ? row0 + r : m - 1;   // clamp: tail rows recompute the last row
            arow[r] = reinterpret_cast<const uint32_t *>(a + row * lda);
            row_value[r] = epi.row_value(row);
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
            if (w + WC == n_words) {
#pragma unroll
                for (int r = 0; r < R; ++r) aw[r][2 * WC - 1] &= last_mask;
            }
#pragma unroll
            for (int u = 0; u < WC; ++u) {
                uint2 bw[VB];
#pragma unroll
                for (int v = 0; v < VB; ++v) bw[v] = lds_b2[(w + u) * CB + lane + 64 * v];
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int v = 0; v < VB; ++v) {
                        pop[r][v] = __popc(aw[r][2 * u] ^ bw[v].x) + pop[r][v];
                        pop[r][v] = __popc(aw[r][2 * u + 1] ^ bw[v].y) + pop[r][v];
                    }
            }
        }
        for (; w < n_words; ++w) {
            uint2 bw[VB];
#pragma unroll
            for (int v = 0; v < VB; ++v) bw[v] = lds_b2[w * CB + lane + 64 * v];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const uint32_t lo = arow[r][2 * w];
                uint32_t hi = arow[r][2 * w + 1];
                if (w == n_words - 1) hi &= last_mask;
#pragma unroll
                for (int v = 0; v < VB; ++v) {
                    pop[r][v] = __popc(lo ^ bw[v].x) + pop[r][v];
                    pop[r][v] = __popc(hi ^ bw[v].y) + pop[r][v];
                }
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (row0 + r >= m) break;                               // wave-uniform
            epi.template store<VB>(ctx, row0 + r, row_value[r], col, pos0, any, n, pop[r]);
        }
    }
}

// ---- rows of at most four packed words (K <= 256) ------------------------------------------
// With so few words per row the scalar loads of A above are a chain of short, dependent fetches
// and the kernel waits on memory latency.  Here a wavefront fetches the packed words (and the
// per-row epilogue value) of 64 rows with coalesced vector loads, lane l holding row l, and the
// next 64 rows are already in flight while the current ones are processed; a row's words reach
// the scalar registers by lane broadcast.  B lives in registers (VB columns x NW words per lane).
template <int VB, int NW, class Epilogue>
__global__ __launch_bounds__(kBlock) void bitgemm_rows_kernel(
    const uint64_t *__restrict__ a, int64_t m, int64_t lda, const uint64_t *__restrict__ b, int n,
    int64_t ldb, uint32_t last_mask, ColumnMap map, Epilogue epi)
{
    constexpr int R = 4;                          // rows per inner step (share the loop overhead)
    const int y = blockIdx.y;
    const int lane = lane_id();
    int col[VB];
    bool any = false;
    uint32_t bw[VB][2 * NW];
#pragma unroll
    for (int v = 0; v < VB; ++v) {
        const int vv = map.per_group * (lane / map.groups) + y * VB + v;
        col[v] = vv < map.vec ? (lane % map.groups) + map.groups * vv : -1;
        any = any || vv < map.vec;
        const bool live = col[v] >= 0 && col[v] < n;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            uint64_t word = live ? b[static_cast<int64_t>(col[v]) * ldb + w] : 0ull;
            if (w == NW - 1) word &= (static_cast<uint64_t>(last_mask) << 32) | 0xffffffffull;
            bw[v][2 * w] = static_cast<uint32_t>(word);
            bw[v][2 * w + 1] = static_cast<uint32_t>(word >> 32);
        }
    }
    const int pos0 = (lane % map.groups) * map.vec + map.per_group * (lane / map.groups) + y * VB;
    typename Epilogue::template Lane<VB> ctx;
    epi.template init<VB>(col, pos0, n, ctx);

    const int64_t wave = static_cast<int64_t>(blockIdx.x) * kWavesPerBlock + wave_in_block();
    const int64_t n_waves = static_cast<int64_t>(gridDim.x) * kWavesPerBlock;

    // fetch of the 64 rows starting at `base`: lane l reads row base + l (clamped to the last row)
    uint32_t aw[2 * NW], aw_next[2 * NW];
    float rv, rv_next;
    auto fetch = [&](int64_t base, uint32_t (&dst)[2 * NW], float &value) {
        const int64_t row = base + lane < m ? base + lane : m - 1;
        const uint2 *src = reinterpret_cast<const uint2 *>(a + row * lda);
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const uint2 word = src[w];
            dst[2 * w] = word.x;
            dst[2 * w + 1] = w == NW - 1 ? (word.y & last_mask) : word.y;
        }
        value = epi.row_value(row);
    };
    int64_t base = wave * kWave;
    if (base < m) fetch(base, aw, rv);
    for (; base < m; base += n_waves * kWave) {
        const int64_t next = base + n_waves * kWave;
        if (next < m) fetch(next, aw_next, rv_next);          // in flight during this batch
        const int rows_here = static_cast<int>(m - base < kWave ? m - base : kWave);
        for (int r0 = 0; r0 < rows_here; r0 += R) {
            int pop[R][VB];
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int v = 0; v < VB; ++v) pop[r][v] = epi.pop_init();
            float value[R];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int src = r0 + r < rows_here ? r0 + r : rows_here - 1;
                value[r] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, rv), src));
#pragma unroll
                for (int q = 0; q < 2 * NW; ++q) {
                    const uint32_t word = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(aw[q]), src));
#pragma unroll
                    for (int v = 0; v < VB; ++v) pop[r][v] = __popc(word ^ bw[v][q]) + pop[r][v];
                }
            }
#pragma unroll
            for (int r = 0; r < R; ++r) {
                if (r0 + r >= rows_here) break;                 // wave-uniform
                epi.template store<VB>(ctx, base + r0 + r, value[r], col, pos0, any, n, pop[r]);
            }
        }
#pragma unroll
        for (int q = 0; q < 2 * NW; ++q) aw[q] = aw_next[q];
        rv = rv_next;
    }
}

// ---- few rows (small graphs) ---------------------------------------------------------------
// With a few thousand rows neither kernel fills the chip and the time of a launch is the latency
// of one wavefront's chain of dependent steps.  Here a wavefront owns one row at a time: lane l
// fetches word 64 c + l of the row (one coalesced load per 4096 bits), the words reach the scalar
// registers by lane broadcast, and B is staged in LDS as above.
template <int VB, class Epilogue>
__global__ __launch_bounds__(kBlock) void bitgemm_small_kernel(
    const uint64_t *__restrict__ a, int64_t m, int64_t lda, const uint64_t *__restrict__ b, int n,
    int64_t ldb, int n_words, uint32_t last_mask, ColumnMap map, Epilogue epi)
{
    extern __shared__ uint64_t lds_b[];          // [n_words][64*VB]
    constexpr int CB = 64 * VB;
    const int y = blockIdx.y;
    stage_b_block<VB>(lds_b, b, n, ldb, n_words, last_mask, map, y);
    const uint2 *lds_b2 = reinterpret_cast<const uint2 *>(lds_b);

    const int lane = lane_id();
    int col[VB];
    bool any;
    const int pos0 = lane_columns<VB>(map, y, lane, col, any);
    typename Epilogue::template Lane<VB> ctx;
    epi.template init<VB>(col, pos0, n, ctx);

    const int64_t wave = static_cast<int64_t>(blockIdx.x) * kWavesPerBlock + wave_in_block();
    const int64_t n_waves = static_cast<int64_t>(gridDim.x) * kWavesPerBlock;
    // the first 64 words of the next row are fetched while the current row is processed
    auto fetch = [&](int64_t row, int c0) {
        const int w = c0 + lane;
        uint2 words = (row < m && w < n_words) ? reinterpret_cast<const uint2 *>(a + row * lda)[w] : make_uint2(0u, 0u);
        if (w == n_words - 1) words.y &= last_mask;
        return words;
    };
    uint2 head = fetch(wave, 0);
    for (int64_t row = wave; row < m; row += n_waves) {
        const float row_value = epi.row_value(row);
        uint2 mine = head;
        head = fetch(row + n_waves, 0);
        int pop[VB];
#pragma unroll
        for (int v = 0; v < VB; ++v) pop[v] = epi.pop_init();
        for (int c0 = 0; c0 < n_words; c0 += kWave) {
            if (c0 > 0) mine = fetch(row, c0);
            const int cnt = n_words - c0 < kWave ? n_words - c0 : kWave;      // wave-uniform
            for (int t = 0; t < cnt; ++t) {
                const uint32_t lo = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(mine.x), t));
                const uint32_t hi = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(mine.y), t));
#pragma unroll
                for (int v = 0; v < VB; ++v) {
                    const uint2 bw = lds_b2[(c0 + t) * CB + lane + 64 * v];
                    pop[v] = __popc(lo ^ bw.x) + pop[v];
                    pop[v] = __popc(hi ^ bw.y) + pop[v];
                }
            }
        }
        epi.template store<VB>(ctx, row, row_value, col, pos0, any, n, pop);
    }
}

// The same for the first layer of a small graph, with the binarisation folded in: the wavefront
// reads its row of the fp32 input itself (lane l reads column 64 w + l), the 64-bit ballot of
// "x >= threshold" is word w of the row (already wave-uniform: no broadcast), and the row scale
// mean |(x - shift) mul| times the optional per-row factor is known when the row ends, in time for
// the epilogue.  One launch instead of two and no packed input written or read.
// fold_last: the row's last bit is left out of the product (last_mask) and carried by the sign of
// the stored scale, as the binarise+pack kernel does.
template <int VB, class Epilogue>
__global__ __launch_bounds__(kBlock) void pack_bitgemm_small_kernel(
    const float *__restrict__ x, int64_t m, int64_t ld_x, int k_bits, const float *__restrict__ shift,
    const float *__restrict__ mul, const float *__restrict__ row_mul, int fold_last, float *__restrict__ scale,
    const uint64_t *__restrict__ b, int n, int64_t ldb, uint32_t last_mask, ColumnMap map, Epilogue epi)
{
    extern __shared__ uint64_t lds_b[];          // [n_words][64*VB]
    constexpr int CB = 64 * VB;
    constexpr int U = 4;                         // row loads in flight
    const int n_words = (k_bits + 63) >> 6;
    const int y = blockIdx.y;
    stage_b_block<VB>(lds_b, b, n, ldb, n_words, last_mask, map, y);
    const uint2 *lds_b2 = reinterpret_cast<const uint2 *>(lds_b);

    const int lane = lane_id();
    int col[VB];
    bool any;
    const int pos0 = lane_columns<VB>(map, y, lane, col, any);
    typename Epilogue::template Lane<VB> ctx;
    epi.template init<VB>(col, pos0, n, ctx);
    const float inv_cols = 1.0f / static_cast<float>(k_bits);

    const int64_t wave = static_cast<int64_t>(blockIdx.x) * kWavesPerBlock + wave_in_block();
    const int64_t n_waves = static_cast<int64_t>(gridDim.x) * kWavesPerBlock;
    for (int64_t row = wave; row < m; row += n_waves) {
        const float *xr = x + row * ld_x;
        int pop[VB];
#pragma unroll
        for (int v = 0; v < VB; ++v) pop[v] = epi.pop_init();
        float sum = 0.0f;
        uint64_t last_word = 0;
        for (int w0 = 0; w0 < n_words; w0 += U) {
            float xv[U], th[U], ml[U];
            bool in[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = 64 * (w0 + u) + lane;
                in[u] = c < k_bits;
                xv[u] = in[u] ? xr[c] : 0.0f;
                th[u] = (shift != nullptr && in[u]) ? shift[c] : 0.0f;
                ml[u] = (mul != nullptr && in[u]) ? mul[c] : 1.0f;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int w = w0 + u;
                if (w >= n_words) break;                      // wave-uniform
                const uint64_t word = __ballot(in[u] && xv[u] >= th[u]);
                sum += in[u] ? fabsf((xv[u] - th[u]) * ml[u]) : 0.0f;
                last_word = word;
                const uint32_t lo = static_cast<uint32_t>(word);
                uint32_t hi = static_cast<uint32_t>(word >> 32);
                if (w == n_words - 1) hi &= last_mask;
#pragma unroll
                for (int v = 0; v < VB; ++v) {
                    const uint2 bw = lds_b2[w * CB + lane + 64 * v];
                    pop[v] = __popc(lo ^ bw.x) + pop[v];
                    pop[v] = __popc(hi ^ bw.y) + pop[v];
                }
            }
        }
        sum = wave_sum_dpp(sum);          // the same order of additions as the stand-alone binarisation
        float s = sum * inv_cols;
        if (row_mul != nullptr) s *= row_mul[row];
        if (fold_last && ((last_word >> ((k_bits - 1) & 63)) & 1ull) == 0) s = -s;
        if (lane == 0 && y == 0) scale[row] = s;
        epi.template store<VB>(ctx, row, s, col, pos0, any, n, pop);
    }
}

template <int VB, class Epilogue>
static int launch_pack_bitgemm_small(const float *x, int64_t m, int64_t ld_x, int64_t k_bits, const float *shift,
                                     const float *mul, const float *row_mul, int fold_last, float *scale,
                                     const uint64_t *b, int64_t n, int64_t ldb, uint32_t last_mask, ColumnMap map,
                                     int col_blocks, const Epilogue &epi, hipStream_t stream)
{
    const int n_words = static_cast<int>((k_bits + 63) / 64);
    const size_t lds = static_cast<size_t>(64) * VB * n_words * sizeof(uint64_t);
    int64_t blocks = (m + kWavesPerBlock - 1) / kWavesPerBlock;
    const int64_t cus = compute_units();
    const int64_t cap = cus * 8 / col_blocks > cus ? cus * 8 / col_blocks : cus;
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL((pack_bitgemm_small_kernel<VB, Epilogue>), dim3(static_cast<unsigned>(blocks), col_blocks),
                       dim3(kBlock), lds, stream, x, m, ld_x, static_cast<int>(k_bits), shift, mul, row_mul, fold_last,
                       scale, b, static_cast<int>(n), ldb, last_mask, map, epi);
    return check_launch();
}

// Row counts up to which bitgemm_small_kernel is used (one wavefront per row still fits the
// resident wavefronts of the chip a few times over).
constexpr int64_t kSmallRows = 32768;

template <int VB, class Epilogue>
static int launch_bitgemm_small(const uint64_t *a, int64_t m, int64_t lda, const uint64_t *b, int64_t n,
                                int64_t ldb, int64_t k_bits, uint32_t last_mask, ColumnMap map,
                                int col_blocks, const Epilogue &epi, hipStream_t stream)
{
    const int n_words = static_cast<int>((k_bits + 63) / 64);
    const size_t lds = static_cast<size_t>(64) * VB * n_words * sizeof(uint64_t);
    // one row per wavefront up to 8 workgroups per compute unit; more rows share the staged B
    int64_t blocks = (m + kWavesPerBlock - 1) / kWavesPerBlock;
    const int64_t cus = compute_units();
    const int64_t cap = cus * 8 / col_blocks > cus ? cus * 8 / col_blocks : cus;
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL((bitgemm_small_kernel<VB, Epilogue>), dim3(static_cast<unsigned>(blocks), col_blocks),
                       dim3(kBlock), lds, stream, a, m, lda, b, static_cast<int>(n), ldb, n_words,
                       last_mask, map, epi);
    return check_launch();
}

template <int VB, int NW, class Epilogue>
static int launch_bitgemm_rows(const uint64_t *a, int64_t m, int64_t lda, const uint64_t *b, int64_t n,
                               int64_t ldb, uint32_t last_mask, ColumnMap map, int col_blocks,
                               const Epilogue &epi, hipStream_t stream)
{
    int64_t blocks = (m + kBlock - 1) / kBlock;               // 64 rows per wavefront and batch
    const int64_t cus = compute_units();
    const int64_t cap = cus * 8 / col_blocks > cus ? cus * 8 / col_blocks : cus;
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL((bitgemm_rows_kernel<VB, NW, Epilogue>), dim3(static_cast<unsigned>(blocks), col_blocks),
                       dim3(kBlock), 0, stream, a, m, lda, b, static_cast<int>(n), ldb, last_mask, map, epi);
    return check_launch();
}

template <int VB, int R, class Epilogue>
static int launch_bitgemm(const uint64_t *a, int64_t m, int64_t lda, const uint64_t *b, int64_t n,
                          int64_t ldb, int64_t k_bits, uint32_t last_mask, ColumnMap map,
                          int col_blocks, const Epilogue &epi, hipStream_t stream)
{
    const int n_words = static_cast<int>((k_bits + 63) / 64);
    const size_t lds = static_cast<size_t>(64) * VB * n_words * sizeof(uint64_t);
    // one row block per wavefront until the chip is full, then grid-stride: every workgroup
    // stages its B block once, so no more workgroups are launched than can be resident
    // (8 per CU, fewer when the staged block is large; 160 KB of LDS per CU)
    int64_t row_blocks = (m + R - 1) / R;
    int64_t blocks = (row_blocks + kWavesPerBlock - 1) / kWavesPerBlock;
    int64_t resident = lds > 0 ? static_cast<int64_t>((160 * 1024) / lds) : 8;
    resident = resident > 8 ? 8 : (resident < 1 ? 1 : resident);
    int64_t cap = static_cast<int64_t>(compute_units()) * resident / col_blocks;
    if (cap < 256) cap = 256;
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL((bitgemm_kernel<VB, R, Epilogue>), dim3(static_cast<unsigned>(blocks), col_blocks),
                       dim3(kBlock), lds, stream, a, m, lda, b, static_cast<int>(n), ldb, n_words,
                       last_mask, map, epi);
    return check_launch();
}

// per_lane values of a lane are split into column blocks of VB values so that the B block
// fits the 64 KB of LDS a workgroup may use: 64 * VB * n_words * 8 <= 65536  <=>
// VB * n_words <= 128.
template <class Epilogue>
static int dispatch_bitgemm(int per_lane, int groups, int vec, const uint64_t *a, int64_t m, int64_t lda,
                            const uint64_t *b, int64_t n, int64_t ldb, int64_t k_bits,
                            uint32_t last_mask, const Epilogue &epi, hipStream_t stream)
{
    const int n_words = static_cast<int>((k_bits + 63) / 64);
    int vb = per_lane >= 8 ? 8 : (per_lane >= 4 ? 4 : (per_lane >= 2 ? 2 : 1));
    while (vb > 1 && vb * n_words > 128) vb >>= 1;
    const int col_blocks = (per_lane + vb - 1) / vb;
    if (col_blocks > 65535) return BIGCN_ESHAPE;           // grid limit of the second dimension
    const ColumnMap map{groups, vec, per_lane};
    if (m <= kSmallRows) {
        if (vb == 8) return launch_bitgemm_small<8>(a, m, lda, b, n, ldb, k_bits, last_mask, map, col_blocks, epi, stream);
        if (vb == 4) return launch_bitgemm_small<4>(a, m, lda, b, n, ldb, k_bits, last_mask, map, col_blocks, epi, stream);
        if (vb == 2) return launch_bitgemm_small<2>(a, m, lda, b, n, ldb, k_bits, last_mask, map, col_blocks, epi, stream);
        return launch_bitgemm_small<1>(a, m, lda, b, n, ldb, k_bits, last_mask, map, col_blocks, epi, stream);
    }
    if (n_words <= 4 && vb <= 4) {
        // K <= 256: batched rows, B in registers
#define BIGCN_ROWS_CASE(VV, WW)                                                                                \
    if (vb == VV && n_words == WW)                                                                             \
        return launch_bitgemm_rows<VV, WW>(a, m, lda, b, n, ldb, last_mask, map, col_blocks, epi, stream)
        BIGCN_ROWS_CASE(4, 1); BIGCN_ROWS_CASE(4, 2); BIGCN_ROWS_CASE(4, 3); BIGCN_ROWS_CASE(4, 4);
        BIGCN_ROWS_CASE(2, 1); BIGCN_ROWS_CASE(2, 2); BIGCN_ROWS_CASE(2, 3); BIGCN_ROWS_CASE(2, 4);
        BIGCN_ROWS_CASE(1, 1); BIGCN_ROWS_CASE(1, 2); BIGCN_ROWS_CASE(1, 3); BIGCN_ROWS_CASE(1, 4);
#undef BIGCN_ROWS_CASE
    }
    if (vb == 8) return launch_bitgemm<8, 2>(a, m, lda, b, n, ldb, k_bits, last_mask, map, col_blocks, epi, stream);
    if (vb == 4) return launch_bitgemm<4, 4>(a, m, lda, b, n, ldb, k_bits, last_mask, map, col_blocks, epi, stream);
    if (vb == 2) return launch_bitgemm<2, 4>(a, m, lda, b, n, ldb, k_bits, last_mask, map, col_blocks, epi, stream);
    return launch_bitgemm<1, 4>(a, m, lda, b, n, ldb, k_bits, last_mask, map, col_blocks, epi, stream);
}

int launch_bitgemm_layout(const uint64_t *a_bits, int64_t m, int64_t lda, const uint64_t *b_bits,
                          int64_t n, int64_t ldb, int64_t k_bits, const float *src_scale, void *c_rows,
                          void *alt_rows, RowLayout layout, hipStream_t stream, int *escape_flag)
{
    if (m == 0 || n == 0) return BIGCN_OK;
    if (layout.escape && alt_rows == nullptr) return BIGCN_ENULL;
    // a stored row is spread over all 64 lanes: each lane produces positions/64 consecutive values
    const int per_lane = layout.positions() >= 64 ? layout.positions() / 64 : 1;
    const uint32_t last_mask = layout.fold_last ? 0x7fffffffu : 0xffffffffu;
    if (layout.kind == kI8) {
        EpilogueLayout<int8_t> epi{static_cast<int8_t *>(c_rows), layout.positions(), layout.k_eff,
                                   layout.embed_scale != kScaleSeparate ? src_scale : nullptr,
                                   layout.embed_scale == kScaleInTopBits ? 3 : (layout.embed_scale == kScaleInLastBytes ? -1 : 0), layout.groups,
                                   layout.escape ? alt_rows : nullptr, layout.alt_kind == kF16 ? 1 : 0, escape_flag};
        // the escape decision is taken by the one wavefront that holds the whole row
        if (layout.escape && (per_lane > 8 || per_lane * ((k_bits + 63) / 64) > 128)) return BIGCN_EINVAL;
        if (layout.escape && layout.alt_kind != kI8 && layout.alt_kind != kF16) return BIGCN_EINVAL;
        if (layout.escape && layout.embed_scale != kScaleInTopBits &&
            (layout.embed_scale != kScaleInLastBytes || layout.alt_kind != kF16))
            return BIGCN_EINVAL;
        return dispatch_bitgemm(per_lane, layout.groups, layout.vec, a_bits, m, lda, b_bits, n, ldb, k_bits,
                                last_mask, epi, stream);
    }
    if (layout.kind == kF16) {
        EpilogueLayout<__half> epi{static_cast<__half *>(c_rows), layout.positions(), layout.k_eff, nullptr, 0, 0, nullptr, 0, nullptr};
        return dispatch_bitgemm(per_lane, layout.groups, layout.vec, a_bits, m, lda, b_bits, n, ldb, k_bits,
                                last_mask, epi, stream);
    }
    EpilogueLayout<float> epi{static_cast<float *>(c_rows), layout.positions(), layout.k_eff, nullptr, 0, 0, nullptr, 0, nullptr};
    return dispatch_bitgemm(per_lane, layout.groups, layout.vec, a_bits, m, lda, b_bits, n, ldb, k_bits,
                            last_mask, epi, stream);
}

// Binarisation of the fp32 input fused into the first layer's bit-GEMM (graphs of at most
// kSmallRows nodes): writes the product rows of `layout` and the source scales, nothing else.
// Returns BIGCN_EINVAL when the shape is not covered (the caller then runs the two kernels).
// Whether launch_pack_bitgemm_layout takes the shape: a small graph, and a row's products within
// one wavefront's column block (several blocks would each re-read the fp32 row).
bool pack_bitgemm_covers(int64_t m, int64_t k_bits, const RowLayout &layout)
{
    if (m > kSmallRows) return false;
    const int per_lane = layout.positions() >= 64 ? layout.positions() / 64 : 1;
    const int n_words = static_cast<int>((k_bits + 63) / 64);
    int vb = per_lane >= 8 ? 8 : (per_lane >= 4 ? 4 : (per_lane >= 2 ? 2 : 1));
    while (vb > 1 && vb * n_words > 128) vb >>= 1;
    return (per_lane + vb - 1) / vb == 1;
}

int launch_pack_bitgemm_layout(const float *x, int64_t m, int64_t ld_x, const float *shift, const float *mul,
                               const float *row_mul, float *scale, const uint64_t *b_bits, int64_t n, int64_t ldb,
                               int64_t k_bits, void *c_rows, void *alt_rows, RowLayout layout, hipStream_t stream)
{
    if (m == 0 || n == 0) return BIGCN_OK;
    if (!pack_bitgemm_covers(m, k_bits, layout)) return BIGCN_EINVAL;
    if (layout.escape && alt_rows == nullptr) return BIGCN_ENULL;
    const int per_lane = layout.positions() >= 64 ? layout.positions() / 64 : 1;
    const int n_words = static_cast<int>((k_bits + 63) / 64);
    int vb = per_lane >= 8 ? 8 : (per_lane >= 4 ? 4 : (per_lane >= 2 ? 2 : 1));
    while (vb > 1 && vb * n_words > 128) vb >>= 1;
    const int col_blocks = 1;
    const uint32_t last_mask = layout.fold_last ? 0x7fffffffu : 0xffffffffu;
    const ColumnMap map{layout.groups, layout.vec, per_lane};
#define BIGCN_PACK_GEMM(EPI)                                                                                       \
    switch (vb) {                                                                                                  \
    case 8: return launch_pack_bitgemm_small<8>(x, m, ld_x, k_bits, shift, mul, row_mul, layout.fold_last, scale,  \
                                                b_bits, n, ldb, last_mask, map, col_blocks, EPI, stream);          \
    case 4: return launch_pack_bitgemm_small<4>(x, m, ld_x, k_bits, shift, mul, row_mul, layout.fold_last, scale,  \
                                                b_bits, n, ldb, last_mask, map, col_blocks, EPI, stream);          \
    case 2: return launch_pack_bitgemm_small<2>(x, m, ld_x, k_bits, shift, mul, row_mul, layout.fold_last, scale,  \
                                                b_bits, n, ldb, last_mask, map, col_blocks, EPI, stream);          \
    default: return launch_pack_bitgemm_small<1>(x, m, ld_x, k_bits, shift, mul, row_mul, layout.fold_last, scale, \
                                                 b_bits, n, ldb, last_mask, map, col_blocks, EPI, stream);         \
    }
    if (layout.kind == kI8) {
        if (layout.escape && layout.alt_kind != kI8 && layout.alt_kind != kF16) return BIGCN_EINVAL;
        // the scale is computed inside the kernel: `embed` only says that the layout wants it in the row
        EpilogueLayout<int8_t> epi{static_cast<int8_t *>(c_rows), layout.positions(), layout.k_eff,
                                   layout.embed_scale != kScaleSeparate ? scale : nullptr,
                                   layout.embed_scale == kScaleInTopBits ? 3 : (layout.embed_scale == kScaleInLastBytes ? -1 : 0), layout.groups,
                                   layout.escape ? alt_rows : nullptr, layout.alt_kind == kF16 ? 1 : 0, nullptr};
        BIGCN_PACK_GEMM(epi)
    }
    if (layout.kind == kF16) {
        EpilogueLayout<__half> epi{static_cast<__half *>(c_rows), layout.positions(), layout.k_eff, nullptr, 0, 0, nullptr, 0, nullptr};
        BIGCN_PACK_GEMM(epi)
    }
    EpilogueLayout<float> epi{static_cast<float *>(c_rows), layout.positions(), layout.k_eff, nullptr, 0, 0, nullptr, 0, nullptr};
    BIGCN_PACK_GEMM(epi)
#undef BIGCN_PACK_GEMM
}

// Product rows in column order (stored position = output column) for consumers that read a row's
// columns next to each other: lane l produces positions [per_lane l, per_lane (l + 1)).  One
// byte per product stores floor(K/2) - popcount (K <= 255), fp16 / fp32 store K - 2 popcount.
// last_mask is ANDed onto the upper half of the last packed word of both operands (0x7fffffff
// leaves bit 63 out: a layer of 256 bits whose last bit is carried outside the stored value).
int launch_bitgemm_natural(const uint64_t *a_bits, int64_t m, int64_t lda, const uint64_t *b_bits, int64_t n,
                           int64_t ldb, int64_t k_bits, void *rows, int positions, RowKind kind,
                           hipStream_t stream, uint32_t last_mask)
{
    if (m == 0 || n == 0) return BIGCN_OK;
    if (positions < n || positions % 8 != 0 || (positions >= 64 && positions % 64 != 0)) return BIGCN_EINVAL;
    if (kind == kI8 && k_bits > 255) return BIGCN_EINVAL;
    const int per_lane = positions >= 64 ? positions / 64 : 1;
    const int k = static_cast<int>(k_bits);
    if (kind == kI8) {
        EpilogueLayout<int8_t> epi{static_cast<int8_t *>(rows), positions, k, nullptr, 0, 0, nullptr, 0, nullptr};
        return dispatch_bitgemm(per_lane, 1, positions, a_bits, m, lda, b_bits, n, ldb, k_bits, last_mask, epi, stream);
    }
    if (kind == kF16) {
        EpilogueLayout<__half> epi{static_cast<__half *>(rows), positions, k, nullptr, 0, 0, nullptr, 0, nullptr};
        return dispatch_bitgemm(per_lane, 1, positions, a_bits, m, lda, b_bits, n, ldb, k_bits, last_mask, epi, stream);
    }
    EpilogueLayout<float> epi{static_cast<float *>(rows), positions, k, nullptr, 0, 0, nullptr, 0, nullptr};
    return dispatch_bitgemm(per_lane, 1, positions, a_bits, m, lda, b_bits, n, ldb, k_bits, last_mask, epi, stream);
}

// Shapes on which the matrix cores measured faster than XOR + bit count (the FP4 path is the
// faster of the two matrix-core paths on all of them): enough inner dimension to pay for the
// expansion of the bits and enough rows and columns to fill the tiles.
bool prefer_mfma(int64_t m, int64_t n, int64_t k_bits)
{
    return k_bits >= 512 && n >= 48 && m >= 16384;
}

}  // namespace bigcn

extern "C" int bigcn_binary_gemm_variant(const uint64_t *a_bits, const float *a_scale, int64_t m,
                                         int64_t lda_words, const uint64_t *b_bits, const float *b_scale,
                                         int64_t n, int64_t ldb_words, int64_t k_bits, int32_t *acc,
                                         int64_t ld_acc, float *out, int64_t ld_out, int variant,
                                         void *stream)
{
    if (variant < BIGCN_GEMM_AUTO || variant > BIGCN_GEMM_FP4) return BIGCN_EINVAL;
    if (a_bits == nullptr || b_bits == nullptr) return BIGCN_ENULL;
    if (acc == nullptr && out == nullptr) return BIGCN_ENULL;
    if (out != nullptr && (a_scale == nullptr || b_scale == nullptr)) return BIGCN_ENULL;
    if (m < 0 || n < 0 || k_bits <= 0) return BIGCN_EINVAL;
    const int64_t n_words = (k_bits + 63) / 64;
    if (lda_words < n_words || ldb_words < n_words) return BIGCN_EINVAL;
    if (acc != nullptr && ld_acc < n) return BIGCN_EINVAL;
    if (out != nullptr && ld_out < n) return BIGCN_EINVAL;
    if (k_bits > BIGCN_MAX_K_BITS || n > BIGCN_MAX_GEMM_N) return BIGCN_ESHAPE;
    if (m == 0 || n == 0) return BIGCN_OK;
    if (variant == BIGCN_GEMM_FP4 || (variant == BIGCN_GEMM_AUTO && bigcn::prefer_mfma(m, n, k_bits)))
        return bigcn::launch_bitgemm_fp4(a_bits, a_scale, m, lda_words, b_bits, b_scale, n, ldb_words, k_bits,
                                         acc, ld_acc, out, ld_out, bigcn::as_stream(stream));
    if (variant == BIGCN_GEMM_MFMA)
        return bigcn::launch_bitgemm_mfma(a_bits, a_scale, m, lda_words, b_bits, b_scale, n, ldb_words, k_bits,
                                          acc, ld_acc, out, ld_out, bigcn::as_stream(stream));
    bigcn::EpilogueApi epi{a_scale, b_scale, acc, ld_acc, out, ld_out, static_cast<int>(k_bits)};
    // row-major output: lane l owns columns l, l + 64, ...
    const int per_lane = static_cast<int>((n + 63) / 64);
    return bigcn::dispatch_bitgemm(per_lane, 64, per_lane, a_bits, m, lda_words, b_bits, n, ldb_words,
                                   k_bits, 0xffffffffu, epi, bigcn::as_stream(stream));
}

extern "C" int bigcn_binary_gemm(const uint64_t *a_bits, const float *a_scale, int64_t m,
                                 int64_t lda_words, const uint64_t *b_bits, const float *b_scale,
                                 int64_t n, int64_t ldb_words, int64_t k_bits, int32_t *acc,
                                 int64_t ld_acc, float *out, int64_t ld_out, void *stream)
{
    return bigcn_binary_gemm_variant(a_bits, a_scale, m, lda_words, b_bits, b_scale, n, ldb_words, k_bits,
                                     acc, ld_acc, out, ld_out, BIGCN_GEMM_AUTO, stream);
}
