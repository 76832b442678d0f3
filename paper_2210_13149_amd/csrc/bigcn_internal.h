// Internal declarations shared by the HIP translation units of libbigcn (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stddef.h>
#include <stdint.h>

#include "bigcn.h"

namespace bigcn {

constexpr int kWave = 64;          // CDNA wavefront width
constexpr int kBlock = 256;        // threads per workgroup used by every kernel here
constexpr int kWavesPerBlock = kBlock / kWave;

// Rows at least this long are aggregated by a whole workgroup instead of one wavefront: by the
// Bi-GAT kernels (kBlockRowDegree) and by the aggregation of the Bi-GCN path (kSplitRowDegree: a
// workgroup per row costs a start-up per row, which rows of a few hundred neighbours do not repay;
// on the 232965-node workload, whose rows average 492 neighbours, 1024 instead of 256 saves 6-10 %
// of an aggregation, and the largest workload does not notice).
constexpr int64_t kBlockRowDegree = 256;
constexpr int64_t kSplitRowDegree = 1024;

inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

// Compute units of the current device (256 on MI355X), asked once per device; launch sizes that
// aim at "all compute units" use it instead of a literal.
inline int compute_units()
{
    static int known[64];
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= 64) return 256;
    if (known[device] == 0) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || cus <= 0) {
            (void)hipGetLastError();
            cus = 256;
        }
        known[device] = cus;
    }
    return known[device];
}

inline int check_launch()
{
    return hipGetLastError() == hipSuccess ? BIGCN_OK : BIGCN_EHIP;
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// Wave-uniform index of this thread's wavefront inside its workgroup, as a scalar value.
__device__ __forceinline__ int wave_in_block()
{
    return __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x) >> 6);
}

// Sum over the 64 lanes of a wavefront in a fixed butterfly order (every lane gets the sum).
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1)
        v += __shfl_xor(v, off, kWave);
    return v;
}

// The same total by data-parallel moves inside the vector ALU (no LDS traffic; a sixth of the
// latency of the butterfly above): lanes of a quad, of a row of 16, then rows 0 -> 1, 2 -> 3 and
// lanes 0..31 -> 32..63; lane 63 ends with the total, which every lane receives.  Fixed order.
// Used for the row scale of the binarisation (Sec. 4.1), where one sum per 100..600 values is taken.
__device__ __forceinline__ float wave_sum_dpp(float v)
{
#define BIGCN_DPP_ADD(CTRL, ROWS)                                                                        \
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROWS, 0xf, false))
    BIGCN_DPP_ADD(0xb1, 0xf);      // quad_perm [1, 0, 3, 2]
    BIGCN_DPP_ADD(0x4e, 0xf);      // quad_perm [2, 3, 0, 1]
    BIGCN_DPP_ADD(0x141, 0xf);     // row_half_mirror
    BIGCN_DPP_ADD(0x140, 0xf);     // row_mirror: every lane of a row of 16 holds the row's sum
    BIGCN_DPP_ADD(0x142, 0xa);     // row_bcast 15: rows 1 and 3 add the sum of the row before them
    BIGCN_DPP_ADD(0x143, 0xc);     // row_bcast 31: rows 2 and 3 add lane 31 (rows 0 + 1)
#undef BIGCN_DPP_ADD
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

// Layout in which the fused forward keeps the integer products C of one node.
// `groups` lanes hold `vec` consecutive stored values each; stored position g*vec + v holds
// output column g + groups*v.  With this interleaving one ballot per v yields `groups`
// consecutive sign bits of the next layer's packed activation.
//
// Storage kinds (all exact):
//   kI8  (K <= 256): q = floor(K'/2) - popcount over the first K' bits, so that the product
//         over those bits is 2q + (K' mod 2).  K' = K, except K = 256 (and K = 128 with the scale
//         in the top bits) where K' = K - 1 and the contribution of the last bit,
//         f_{k,K-1} * b_{K-1,j}, is carried separately: the sign f_{k,K-1} rides on the sign of the
//         node's stored scale, b_{K-1,j} is a per-column constant.  q always fits int8.
//   kF16 (K <= 2048): the product itself; every integer of magnitude <= 2048 is exact in fp16.
//   kF32 : the product as fp32.
enum RowKind { kI8 = 0, kF16 = 1, kF32 = 2 };

// Where the aggregation finds a node's fp32 source scale (kI8 rows may carry it themselves, so
// that no second cache line is gathered per neighbour):
//   kScaleSeparate   an array of n floats, gathered through the column index;
//   kScaleInTail     the last 4 bytes of the stored row (rows with at least 4 spare positions);
//   kScaleInTopBits  the stored values use 7 bits (always true for K' <= 127; checked per row
//                    otherwise, see `escape`): bit i of the scale is the top bit of the first
//                    byte of lane i's segment, i < 32 (rows of 32 or 64 lanes).
//   kScaleInLastBytes  64-byte rows of 40..60 columns (8 lanes of 8 values): the last value of
//                    each of the last four lanes belongs to a column past the last one; byte i
//                    of the scale is stored there (lane 4 + i).  Keeps such rows in half a cache
//                    line's worth of lanes instead of widening them to 16 lanes for a tail.
enum ScalePlace { kScaleSeparate = 0, kScaleInTail = 1, kScaleInTopBits = 2, kScaleInLastBytes = 3 };

struct RowLayout {
    int groups;      // lanes that share one stored row (power of two, 2..64)
    int vec;         // values per lane (4 or 8)
    int kind;        // RowKind
    int k_eff;       // K': bits covered by the stored value
    int fold_last;   // 1: bit K-1 is excluded from the stored value (kI8 with K = 256, or K = 128
                     //    when the scale sits in the top bits)
    int embed_scale; // ScalePlace
    int escape;      // 1 (kScaleInTopBits, K' > 127): a row whose values do not all fit 7 bits carries
                     //    a NaN scale; its values live in an alternate row array (same positions,
                     //    element kind alt_kind) and its scale in the per-node array
    int alt_kind;    // RowKind of the alternate array: kI8 (K <= 256), kF16 (K <= 4096: |value| <=
                     //    2048 is exact in fp16), kF32
    __host__ __device__ int positions() const { return groups * vec; }
    __host__ __device__ int elem_bytes() const { return kind == kI8 ? 1 : (kind == kF16 ? 2 : 4); }
    __host__ __device__ int64_t row_bytes() const { return static_cast<int64_t>(positions()) * elem_bytes(); }
    __host__ __device__ int64_t alt_row_bytes() const
    {
        return static_cast<int64_t>(positions()) * (alt_kind == kI8 ? 1 : (alt_kind == kF16 ? 2 : 4));
    }
    // sum_k w_k c_kj = mul * sum_k w_k stored_kj + bias * sum_k w_k (+ last-bit term)
    __host__ __device__ float mul() const { return kind == kI8 ? 2.0f : 1.0f; }
    __host__ __device__ float bias() const { return kind == kI8 ? static_cast<float>(k_eff & 1) : 0.0f; }
};

// Layout used for a layer with d_out columns and d_in input bits.
RowLayout choose_layout(int64_t d_in, int64_t d_out);

// ---- internal launchers (defined in the .hip files) ------------------------------------
// pack: as bigcn_pack, plus an optional per-row factor folded into the scale.
// fold_last_sign: the stored scale additionally carries the sign of the row's last column.
// clear_flag (DEVICE, nullable): an int that the launch sets to 0 (see FusedSpmmArgs::escape_flag).
int launch_pack(const float *x, int64_t rows, int64_t cols, int64_t row_stride,
                int64_t col_stride, const float *shift, const float *mul, const float *row_mul,
                int fold_last_sign, uint64_t *bits, int64_t ld_words, float *scale,
                hipStream_t stream, int *clear_flag = nullptr);

// Stored source scale of rows that are already packed: beta[i] * row_mul[i] (row_mul nullable),
// negated when fold_last_sign is set and the row's last bit (column cols-1) is 0.
int launch_source_scale(const float *beta, const float *row_mul, const uint64_t *bits, int64_t ld_words,
                        int64_t cols, int fold_last_sign, float *scale, int64_t rows, hipStream_t stream,
                        int *clear_flag = nullptr);

// bit-GEMM writing the integer products in a RowLayout (fused forward).
// src_scale (m floats) is copied into the rows when the layout embeds the scale.
// alt_rows (escape layouts only): receives the rows that do not fit 7 bits, one byte or fp16 per value
// (layout.alt_kind).  escape_flag (DEVICE, nullable): set to 1 when any row went to alt_rows; never
// cleared here.
int launch_bitgemm_layout(const uint64_t *a_bits, int64_t m, int64_t lda, const uint64_t *b_bits,
                          int64_t n, int64_t ldb, int64_t k_bits, const float *src_scale, void *c_rows,
                          void *alt_rows, RowLayout layout, hipStream_t stream, int *escape_flag = nullptr);

// First layer of a small graph: binarise the fp32 rows of x and multiply in one launch; writes
// the product rows and scale[i] = row_mul[i] * beta_i (negated for a folded last bit of -1).
// BIGCN_EINVAL: shape not covered (more than 32768 rows, or a row wider than one wavefront's
// column block); nothing was launched.
bool pack_bitgemm_covers(int64_t m, int64_t k_bits, const RowLayout &layout);
int launch_pack_bitgemm_layout(const float *x, int64_t m, int64_t ld_x, const float *shift, const float *mul,
                               const float *row_mul, float *scale, const uint64_t *b_bits, int64_t n, int64_t ldb,
                               int64_t k_bits, void *c_rows, void *alt_rows, RowLayout layout, hipStream_t stream);

// bit-GEMM writing the integer products of a row in column order (`positions` stored values per
// row, a multiple of 8 and >= n; multiples of 64 from 64 on): one byte per product holds
// floor(K/2) - popcount (K <= 255 only), fp16 / fp32 hold K - 2 popcount.
int launch_bitgemm_natural(const uint64_t *a_bits, int64_t m, int64_t lda, const uint64_t *b_bits, int64_t n,
                           int64_t ldb, int64_t k_bits, void *rows, int positions, RowKind kind,
                           hipStream_t stream, uint32_t last_mask = 0xffffffffu);

// Matrix-core (int8 MFMA) variant of the public bit-GEMM: same arguments and results.
int launch_bitgemm_mfma(const uint64_t *a_bits, const float *a_scale, int64_t m, int64_t lda,
                        const uint64_t *b_bits, const float *b_scale, int64_t n, int64_t ldb,
                        int64_t k_bits, int32_t *acc, int64_t ld_acc, float *out, int64_t ld_out,
                        hipStream_t stream);

// The same on the FP4 path of the block-scaled matrix cores (unit scales).
int launch_bitgemm_fp4(const uint64_t *a_bits, const float *a_scale, int64_t m, int64_t lda,
                       const uint64_t *b_bits, const float *b_scale, int64_t n, int64_t ldb,
                       int64_t k_bits, int32_t *acc, int64_t ld_acc, float *out, int64_t ld_out,
                       hipStream_t stream);

// The FP4 path with one 128 x 128 tile per wavefront and no LDS stage (shapes bound by the
// multiplies): fp4_tile_covers says whether launch_bitgemm_fp4 hands the shape to it.
bool fp4_tile_covers(int64_t m, int64_t n, int64_t k_bits, int64_t ld_acc, int64_t ld_out, int64_t lda, int64_t ldb);
int launch_bitgemm_fp4_tile(const uint64_t *a_bits, const float *a_scale, int64_t m, int64_t lda,
                            const uint64_t *b_bits, const float *b_scale, int64_t n, int64_t ldb,
                            int64_t k_bits, int32_t *acc, int64_t ld_acc, float *out, int64_t ld_out,
                            hipStream_t stream);

// Product rows of a one-byte RowLayout on the FP4 matrix cores (K <= 1024, 64 / 128 / 256 / 512 stored
// positions, more than 32768 rows): fp4_rows_covers says whether the shape is taken.
bool fp4_rows_covers(int64_t m, int64_t k_bits, const RowLayout &layout);
int launch_bitgemm_fp4_rows(const uint64_t *a_bits, int64_t m, int64_t lda, const uint64_t *b_bits, int64_t n,
                            int64_t ldb, int64_t k_bits, const float *src_scale, void *c_rows, void *alt_rows,
                            RowLayout layout, hipStream_t stream, int *escape_flag = nullptr);

// The same kernel writing one-byte rows in column order (position = column, nothing but the
// values in the row; K <= 255): what launch_bitgemm_natural writes, for more than 32768 rows of
// 64 / 128 / 256 / 512 positions.
bool fp4_natural_covers(int64_t m, int64_t k_bits, int positions);
int launch_bitgemm_fp4_natural(const uint64_t *a_bits, int64_t m, int64_t lda, const uint64_t *b_bits, int64_t n,
                               int64_t ldb, int64_t k_bits, void *rows, int positions, hipStream_t stream);

// Aggregation of layer l fused with the rescale and with the binarisation of layer l+1.
// Bi-GCN: dst_mul = next_row_mul = D^-1/2 and no own-row term.  Bi-GraphSAGE (mean aggregator):
// dst_mul = 1/|N_i|, next_row_mul = nullptr, and the own-row term is described by self_*.
struct FusedSpmmArgs {
    const bigcn_plan *plan;
    const int64_t *row_ptr;
    const int32_t *col_idx;
    const float *dst_mul;       // n: factor of the neighbour sum of node i
    const float *src_scale;     // n: weight of source node k (its beta_k, times D^-1/2 for Bi-GCN;
                                //    negative when the layout folds the last bit and that bit is -1)
    const void *c_rows;         // n rows in `layout`
    RowLayout layout;
    const float *alpha;         // d_out
    int64_t d_out;
    const uint64_t *w_bits;     // this layer's packed weights (for the last-bit term)
    int64_t w_ld_words;
    int64_t d_in;
    // last layer: fp32 logits
    float *logits;
    int64_t ld_logits;
    // hidden layer: packed signs + scale of the next layer's input
    const float *next_shift;    // d_out, nullable
    const float *next_mul;      // d_out, nullable
    uint64_t *next_bits;
    int64_t next_ld_words;
    float *next_scale;          // n: next_row_mul[i] * beta_i of the next layer
    const float *next_row_mul;  // n, nullable (= 1)
    int next_fold_last_sign;    // the next layer's layout has fold_last: sign the stored scale
    // own-row term, all nullptr when absent
    const void *alt_rows;       // escape layouts: the rows that did not fit 7 bits (bytes or fp16: alt_kind)
    const void *alt_self_rows;  //   (same for the own-row array)
    const void *self_rows;      // n rows in `layout`: products with the second weight matrix
    const float *self_alpha;    // d_out
    const uint64_t *self_w_bits;// packed second weight matrix (for its last-bit term), stride w_ld_words
    // escape layouts: *escape_flag == 0 (DEVICE, nullable) promises that no row of c_rows / self_rows
    // went to the alternate arrays; the aggregation is then launched twice, gated on the flag: the
    // kernel without the per-row test and the one with it.  clear_flag (DEVICE, nullable) is set to
    // 0 by this launch: the flag of the layer that follows.
    const int *escape_flag;
    int *clear_flag;
};
int launch_fused_spmm(const FusedSpmmArgs &args, hipStream_t stream);

}  // namespace bigcn

// The plan: row order by decreasing length (device copy) and the split between rows handled
// by a whole workgroup and rows handled by one wavefront.
// One entry of the plan's row list: a row and where its entries lie in the CSR arrays, so that the
// aggregation finds them with one 16-byte load instead of a load of the row number followed by a
// load of its two row pointers (one dependent memory access fewer per row: 2-4 us of a launch on
// the graphs of a few thousand nodes, whose time is a chain of such accesses).
struct bigcn_plan_entry {
    int64_t first;       // row_ptr[row]
    int32_t row;
    int32_t count;       // row_ptr[row + 1] - row_ptr[row]
};

struct bigcn_plan {
    int64_t n;
    int64_t nnz;
    int device;
    int compute_units;       // of `device`, read when the plan was created
    int32_t *row_order;      // DEVICE, n entries
    bigcn_plan_entry *entries; // DEVICE, n entries: the same order with the rows' extents
    int64_t n_block_rows;    // the first n_block_rows entries of row_order have degree >= kBlockRowDegree
    int64_t n_split_rows;    // ... the first n_split_rows entries degree >= kSplitRowDegree
    int64_t max_degree;
};
