// Kernel 2 on the FP4 matrix cores, large-tile form: the +-1 inner products of Sec. 4.2.3,
// c_ij = sum_k F_ik B_kj, for shapes that are bound by the multiplies (many rows, more than 64
// columns, K of 512 bits or more).
//
// One wavefront owns a tile of 128 rows x 128 columns (4 x 4 multiplies of 32 x 32 x 64 per 64
// bits of K, v_mfma_scale_f32_32x32x64_f8f6f4 with both operands FP4 E2M1 and unit scales) and
// runs alone on its SIMD: 256 accumulator registers, every expanded operand feeds four
// multiplies.  The operands are not staged in LDS and there is no barrier.  K is walked in
// chunks of 256 bits; lane (i, h) (i = lane % 32, h = lane / 32) loads, for each of its four
// rows 32 rt + i and its four columns 32 ct + i, the 16 bytes [32 chunk + 16 h, +16) of the
// packed row straight from global memory (the two lanes of a row read 32 consecutive bytes; a
// 128-byte line serves four chunks and stays in L2 meanwhile), two chunks ahead of the one being
// multiplied.  The order of the k values inside a multiply is free as long as both operands
// agree, so multiply t of a chunk simply takes dword t of every lane's 16 bytes.
//
// Codes: the 32 bits x of a dword become four operand dwords, operand dword d taking the bits
// d, d + 4, ..., d + 28 of x where they stand.  Both operands are coded as the *negated* sign
// (sign bit of the code = the bit itself, so a set bit, +1, becomes a negative code): the
// products are the same, and the sign needs no complement.  The magnitudes are chosen per
// operand dword so that a code is at most one shift away from the bits: rows use 2 / 1 / 0.5 / 1
// for d = 0..3 and columns 0.5 / 1 / 2 / 1, every product is exactly +-1, and the fp32
// accumulators hold c_ij itself (integers below 2^24: exact).
// The last, partial chunk of K is loaded dword by dword up to bit K, and the row codes of the
// positions at and beyond K are cleared (FP4 zero), so that they add nothing.
#include <algorithm>

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

// mag[0..2]: the codes of 2.0 / 1.0 / 0.5 in every nibble (registers, see lshl_or).
// Rows: magnitudes 2 / 1 / 0.5 / 1 for operand dwords 0..3; columns: 0.5 / 1 / 2 / 1.
template <bool kColumn>
__device__ __forceinline__ v8i codes(uint32_t x, const uint32_t (&mag)[3])
{
    v8i op;
    op[0] = static_cast<int>(lshl_or(x & 0x11111111u, 3, mag[kColumn ? 2 : 0]));
    op[1] = static_cast<int>(lshl_or(x & 0x22222222u, 2, mag[1]));
    op[2] = static_cast<int>(lshl_or(x & 0x44444444u, 1, mag[kColumn ? 0 : 2]));
    op[3] = static_cast<int>(and_or(x, 0x88888888u, mag[1]));
    op[4] = op[5] = op[6] = op[7] = 0;
    return op;
}

struct Chunk {
    Bits128 a[4];
    Bits128 b[4];
};

}  // namespace

// One staged result row: 128 columns as int16 (|c| <= K <= 8192), position 4 i + ct holding column
// 32 ct + i, so that the four accumulator registers (ct = 0..3) a lane holds for one row and one
// i are 8 consecutive bytes.
constexpr int kStageRowBytes = kTileCols * 2;
constexpr int kStageBytes = kTileRows * kStageRowBytes;       // 32 KB per wavefront
constexpr int kSlices = kTileRows / 8;                        // a slice = 8 rows = one drain step

struct TileArgs {
    const uint64_t *a;
    int64_t m, lda;
    const uint64_t *b;
    int n;
    int64_t ldb;
    int k_bits;
    const float *a_scale, *b_scale;
    int32_t *acc_out;
    int64_t ld_acc;
    float *out;
    int64_t ld_out;
    int64_t n_tiles;
    int col_tiles;
};

// Persistent wavefronts: wavefront w of the launch takes tiles w, w + W, w + 2 W, ... (tile index =
// row tile * column tiles + column tile, so that the wavefronts of a workgroup that share rows
// read them at about the same time).  The results of a tile do not go to global memory when the
// tile ends: the wavefront converts them, parks them in its own 32 KB of LDS and writes them out
// slice by slice between the multiplies of the *next* tile (a wavefront may have only 64 memory
// operations in flight: storing 256 registers in one go runs at the speed of the memory system
// with the matrix cores idle, and all wavefronts would do so at the same time).  No barrier
// anywhere: a wavefront only ever reads LDS that it wrote itself.
//
// With one wavefront per SIMD nothing hides an instruction that is not issued next to a multiply,
// so the loop over K is one basic block: chunk loads past the end are clamped to the last chunk
// instead of skipped, and the stores of a slice are buffer stores whose offset is moved out of
// the descriptor's range when there is nothing to store (no slice left, a row past m, a column
// past n): the hardware drops those, no branch and no change of the execution mask is needed.
// kDrains slices are written out per chunk (1, 2 or 4: enough for the 16 slices of a tile when K
// has at least 16, 8 or 4 chunks; what is left is written out after the loop).
constexpr uint32_t kOutOfRange = 0x80000000u;                 // beyond any descriptor built below
constexpr int kBufferFlags = 0x00020000;                      // raw buffer, 32-bit data format
constexpr int kStorePolicy = 2;                               // non-temporal: the results are written once and not read here
                                                              // (measured: 0.175 -> 0.148 ms at M = 262144, n = 256, K = 4096)

template <bool kAcc, bool kOut, int kDrains>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(1, 1))) void bitgemm_fp4_tile_kernel(TileArgs p)
{
    __shared__ __attribute__((aligned(16))) unsigned char stage_all[kWavesPerBlock][kStageBytes];
    const int lane = lane_id();
    const int wave = wave_in_block();
    const int i32 = lane & 31;
    const int half = lane >> 5;
    unsigned char *stage = stage_all[wave];
    const int k_bits = p.k_bits;
    const int n_full = k_bits / kChunkBits;                   // chunks that lie wholly below K
    const bool partial = n_full * kChunkBits < k_bits;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kWavesPerBlock;

    // the codes of 2.0 / 1.0 / 0.5 in every nibble, kept in vector registers (opaque to the
    // compiler so that they are not folded back into literals)
    uint32_t mag[3] = {0x44444444u, 0x22222222u, 0x11111111u};
#pragma unroll
    for (int d = 0; d < 3; ++d) asm volatile("" : "+v"(mag[d]));

    // The tile being multiplied.  Addresses are a wave-uniform base (first row / column of the tile)
    // plus 32-bit byte offsets of this lane's four rows and four columns (clamped: results of
    // clamped rows / columns are never written out): eight registers instead of sixteen.
    int64_t row0 = 0;
    int col0 = 0;
    const unsigned char *a_base = nullptr, *b_base = nullptr;
    uint32_t a_off[4], b_off[4];
    auto set_tile = [&](int64_t t) {
        row0 = (t / p.col_tiles) * kTileRows;
        col0 = static_cast<int>(t % p.col_tiles) * kTileCols;
        a_base = reinterpret_cast<const unsigned char *>(p.a + row0 * p.lda);
        b_base = reinterpret_cast<const unsigned char *>(p.b + static_cast<int64_t>(col0) * p.ldb);
        const int rows_here = static_cast<int>(min(static_cast<int64_t>(kTileRows), p.m - row0));
        const int cols_here = min(kTileCols, p.n - col0);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int r = min(32 * q + i32, rows_here - 1), cc = min(32 * q + i32, cols_here - 1);
            a_off[q] = static_cast<uint32_t>(r) * static_cast<uint32_t>(p.lda) * 8u + 16u * half;
            b_off[q] = static_cast<uint32_t>(cc) * static_cast<uint32_t>(p.ldb) * 8u + 16u * half;
        }
    };
    // chunk c (wholly below K; the caller keeps c < n_full): 16 bytes per row / column and lane
    auto load = [&](int c, Chunk &s) {
        const unsigned char *ac = a_base + 32 * c, *bc = b_base + 32 * c;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            s.a[q] = *reinterpret_cast<const Bits128 *>(ac + a_off[q]);
            s.b[q] = *reinterpret_cast<const Bits128 *>(bc + b_off[q]);
        }
    };
    // the partial chunk at the end of K: dword by dword, nothing is read at or beyond bit K
    // (dwords wholly beyond K are zero; the positions beyond K are taken out in multiply())
    auto load_partial = [&](Chunk &s) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int left = k_bits - (kChunkBits * n_full + 128 * half + 32 * u);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                s.a[q].d[u] = 0u;
                s.b[q].d[u] = 0u;
            }
            if (left > 0) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    s.a[q].d[u] = *reinterpret_cast<const uint32_t *>(a_base + 32 * n_full + 4 * u + a_off[q]);
                    s.b[q].d[u] = *reinterpret_cast<const uint32_t *>(b_base + 32 * n_full + 4 * u + b_off[q]);
                }
            }
        }
    };

    // The tile whose results sit in LDS: slices [slice, kSlices) are still to be written out.
    // Slice s: lane (r = lane / 8, g = lane % 8) takes row 8 s + r and the 32 staged bytes
    // [32 g, 32 g + 32) of it = columns 32 ct + 4 g + e, e = 0..3, for the four ct: four stores of
    // 16 bytes per output array, eight lanes covering one 128-byte line each.  The descriptors
    // start at the tile's first row (column 0) and end behind its last existing row.
    int slice = kSlices;
    __amdgpu_buffer_rsrc_t acc_rsrc = __builtin_amdgcn_make_buffer_rsrc(p.acc_out, 0, 0, kBufferFlags);
    __amdgpu_buffer_rsrc_t out_rsrc = __builtin_amdgcn_make_buffer_rsrc(p.out, 0, 0, kBufferFlags);
    int64_t done_row0 = 0;
    const int dr = lane >> 3, dg = lane & 7;
    uint32_t acc_lane = kOutOfRange, out_lane = kOutOfRange;  // byte offset of (row dr, this lane's first column)
    int b_scale_col = 0;                                      // that column, clamped, for b_scale
    // drain_read(s) fetches what slice s needs (two LDS reads; the row scale for fp32 output) and
    // drain_store writes it out: in the K loop the reads are issued with the chunk loads, a whole
    // chunk of multiplies ahead of the stores that use them.
    struct Parked {
        uint4 lo, hi;
        float sa;
        int s;
    };
    auto drain_read = [&](int s) {
        Parked d;
        d.s = s;
        const int s_in = s < kSlices ? s : kSlices - 1;       // LDS reads stay inside the stage
        const uint4 *src = reinterpret_cast<const uint4 *>(stage + (8 * s_in + dr) * kStageRowBytes + 32 * dg);
        d.lo = src[0];
        d.hi = src[1];
        d.sa = 0.0f;
        if (kOut) {
            int64_t row = done_row0 + 8 * s_in + dr;
            if (row >= p.m) row = p.m - 1;
            d.sa = p.a_scale[row];
        }
        return d;
    };
    auto drain_store = [&](const Parked &d) {
        const int s = d.s;
        const int s_in = s < kSlices ? s : kSlices - 1;
        const uint32_t w[8] = {d.lo.x, d.lo.y, d.lo.z, d.lo.w, d.hi.x, d.hi.y, d.hi.z, d.hi.w};   // w[2 e + ct / 2]: ct even | odd
        const bool live = s < kSlices;                        // uniform
        const float sa = d.sa;
#pragma unroll
        for (int ct = 0; ct < 4; ++ct) {
            typedef int v4i __attribute__((ext_vector_type(4)));
            typedef float v4f __attribute__((ext_vector_type(4)));
            v4i c;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t pair = w[2 * e + (ct >> 1)];
                c[e] = (ct & 1) ? (static_cast<int>(pair) >> 16) : static_cast<int>(static_cast<int16_t>(pair & 0xffffu));
            }
            // columns past n: this lane's four columns 32 ct + 4 g .. + 3 exist all or not at all (n % 4 == 0)
            const bool col_ok = b_scale_col + 32 * ct < p.n;
            if (kAcc) {
                const uint32_t off = (live && col_ok) ? acc_lane + static_cast<uint32_t>(8 * s_in) * static_cast<uint32_t>(p.ld_acc) * 4u + 128u * ct
                                                      : kOutOfRange;
                __builtin_amdgcn_raw_buffer_store_b128(c, acc_rsrc, static_cast<int>(off), 0, kStorePolicy);
            }
            if (kOut) {
                int j = b_scale_col + 32 * ct;
                if (j + 3 >= p.n) j = p.n - 4;
                struct __attribute__((aligned(4))) F4 { float v[4]; };
                const F4 sb = *reinterpret_cast<const F4 *>(p.b_scale + j);
                v4f o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = sa * sb.v[e] * static_cast<float>(c[e]);
                const uint32_t off = (live && col_ok) ? out_lane + static_cast<uint32_t>(8 * s_in) * static_cast<uint32_t>(p.ld_out) * 4u + 128u * ct
                                                      : kOutOfRange;
                __builtin_amdgcn_raw_buffer_store_b128(o, out_rsrc, static_cast<int>(off), 0, kStorePolicy);
            }
        }
    };
    auto drain = [&](int s) { drain_store(drain_read(s)); };

    int64_t tile = static_cast<int64_t>(blockIdx.x) * kWavesPerBlock + wave;
    Chunk s0, s1, s2;
    if (tile < p.n_tiles) {
        set_tile(tile);
        if (n_full > 0) load(0, s0);
        if (n_full > 1) load(1, s1);
    }
    while (tile < p.n_tiles) {                                // wave-uniform
        v16f acc[4][4];
#pragma unroll
        for (int rt = 0; rt < 4; ++rt)
#pragma unroll
            for (int ct = 0; ct < 4; ++ct)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[rt][ct][r] = 0.0f;

        v8i ca[4], cb[4];
        // Bits of this lane's dword u of the partial chunk that lie below K.
        auto partial_keep = [&](int u) {
            const int left = k_bits - (kChunkBits * n_full + 128 * half + 32 * u);
            return left >= 32 ? 0xffffffffu : (left <= 0 ? 0u : ((1u << left) - 1u));
        };
        // The operand codes of one step from its four row and four column dwords.  keep: the bits
        // that lie below K (all ones except in the partial chunk); the row codes of the others are
        // cleared (FP4 zero), nibble i of operand dword d standing for bit 4 i + d.
        auto expand = [&](const uint32_t (&aw)[4], const uint32_t (&bw)[4], uint32_t keep, v8i (&oa)[4], v8i (&ob)[4]) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                oa[q] = codes<false>(aw[q], mag);
                ob[q] = codes<true>(bw[q], mag);
            }
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const int keep_codes = static_cast<int>(((keep >> d) & 0x11111111u) * 0xfu);
#pragma unroll
                for (int q = 0; q < 4; ++q) oa[q][d] &= keep_codes;
            }
        };
        auto expand_step = [&](const Chunk &s, int u, uint32_t keep, v8i (&oa)[4], v8i (&ob)[4]) {
            const uint32_t aw[4] = {s.a[0].d[u], s.a[1].d[u], s.a[2].d[u], s.a[3].d[u]};
            const uint32_t bw[4] = {s.b[0].d[u], s.b[1].d[u], s.b[2].d[u], s.b[3].d[u]};
            expand(aw, bw, keep, oa, ob);
        };
        // Sixteen multiplies of one step.  The codes they use were built during the step before
        // (see multiply below), so the compiler can place the vector instructions of the next
        // step between them: built in one piece ahead of their own multiplies the same
        // instructions leave the matrix pipe idle meanwhile (a launch of nothing but expansion and
        // multiplies loses a sixth that way and nothing when they alternate).
        auto multiply16 = [&](const v8i (&oa)[4], const v8i (&ob)[4]) {
#pragma unroll
            for (int rt = 0; rt < 4; ++rt)
#pragma unroll
                for (int ct = 0; ct < 4; ++ct)
                    acc[rt][ct] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(oa[rt], ob[ct], acc[rt][ct], 4, 4, 0,
                                                                                 0x7f7f7f7f, 0, 0x7f7f7f7f);
        };
        // One chunk: on entry (ca, cb) hold the codes of its step 0; every step builds the codes
        // of the step after it while it multiplies, the last one those of step 0 of the chunk that
        // follows (its dwords next_a / next_b; anything valid when nothing follows), which are in
        // (ca, cb) again on exit: four steps, two code sets in turn, nothing is copied and there is
        // no branch.  masked: the partial chunk.
        v8i na[4], nb[4];
        auto multiply = [&](const Chunk &s, bool masked, const uint32_t (&next_a)[4], const uint32_t (&next_b)[4],
                            uint32_t next_keep) {
            expand_step(s, 1, masked ? partial_keep(1) : 0xffffffffu, na, nb);
            multiply16(ca, cb);
            expand_step(s, 2, masked ? partial_keep(2) : 0xffffffffu, ca, cb);
            multiply16(na, nb);
            expand_step(s, 3, masked ? partial_keep(3) : 0xffffffffu, na, nb);
            multiply16(ca, cb);
            expand(next_a, next_b, next_keep, ca, cb);
            multiply16(na, nb);
        };
        auto multiply_then = [&](const Chunk &s, const Chunk &next) {      // whole chunk followed by a whole chunk
            const uint32_t aw[4] = {next.a[0].d[0], next.a[1].d[0], next.a[2].d[0], next.a[3].d[0]};
            const uint32_t bw[4] = {next.b[0].d[0], next.b[1].d[0], next.b[2].d[0], next.b[3].d[0]};
            multiply(s, false, aw, bw, 0xffffffffu);
        };

        // Three register sets in rotation, chunk c + 2 requested before chunk c is multiplied; the
        // loop body is three whole chunks so that the sets keep their names (no copies) and the
        // loop has one exit (the 256 accumulators must not meet at a join of several paths); the
        // one or two chunks left over are already in s0 / s1 when the loop ends.
        const int last = n_full - 1;
        Parked parked[kDrains];
        int c = 0;
        expand_step(s0, 0, 0xffffffffu, ca, cb);
        for (; c + 3 <= n_full; c += 3) {
            load(min(c + 2, last), s2);
#pragma unroll
            for (int q = 0; q < kDrains; ++q) parked[q] = drain_read(slice + q);
            __builtin_amdgcn_sched_barrier(0);        // the requests stay ahead of the multiplies
            multiply_then(s0, s1);
#pragma unroll
            for (int q = 0; q < kDrains; ++q) drain_store(parked[q]);
            slice += kDrains;
            load(min(c + 3, last), s0);
#pragma unroll
            for (int q = 0; q < kDrains; ++q) parked[q] = drain_read(slice + q);
            __builtin_amdgcn_sched_barrier(0);        // the requests stay ahead of the multiplies
            multiply_then(s1, s2);
#pragma unroll
            for (int q = 0; q < kDrains; ++q) drain_store(parked[q]);
            slice += kDrains;
            load(min(c + 4, last), s1);
#pragma unroll
            for (int q = 0; q < kDrains; ++q) parked[q] = drain_read(slice + q);
            __builtin_amdgcn_sched_barrier(0);        // the requests stay ahead of the multiplies
            multiply_then(s2, s0);                    // s0: chunk c + 3, or the last one again (then unused)
#pragma unroll
            for (int q = 0; q < kDrains; ++q) drain_store(parked[q]);
            slice += kDrains;
        }
        // What is left: up to two whole chunks (s0, s1) and the partial one (s2).  The codes of the
        // first of them are built here, outside any multiply; which chunk follows which is chosen
        // by selecting its dwords, not by branching.
        const bool left0 = c < n_full, left1 = c + 1 < n_full;
        if (partial) load_partial(s2);
        uint32_t first_a[4], first_b[4], after0_a[4], after0_b[4], part_a[4], part_b[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            part_a[q] = s2.a[q].d[0];
            part_b[q] = s2.b[q].d[0];
            first_a[q] = left0 ? s0.a[q].d[0] : part_a[q];
            first_b[q] = left0 ? s0.b[q].d[0] : part_b[q];
            after0_a[q] = left1 ? s1.a[q].d[0] : part_a[q];
            after0_b[q] = left1 ? s1.b[q].d[0] : part_b[q];
        }
        expand(first_a, first_b, left0 ? 0xffffffffu : partial_keep(0), ca, cb);
        if (left0) multiply(s0, false, after0_a, after0_b, left1 ? 0xffffffffu : partial_keep(0));
        if (left1) multiply(s1, false, part_a, part_b, partial_keep(0));
        if (partial) multiply(s2, true, part_a, part_b, 0xffffffffu);
        while (slice < kSlices) drain(slice++);               // short K: what the chunks did not cover

        // the tile just multiplied becomes the one to write out
        {
            done_row0 = row0;
            const int64_t rows_here = min(static_cast<int64_t>(kTileRows), p.m - row0);
            const int first_col = col0 + 4 * dg;
            b_scale_col = first_col;
            if (kAcc) {
                acc_rsrc = __builtin_amdgcn_make_buffer_rsrc(p.acc_out + row0 * p.ld_acc, 0,
                                                             static_cast<int>(rows_here * p.ld_acc * 4), kBufferFlags);
                acc_lane = (static_cast<uint32_t>(dr) * static_cast<uint32_t>(p.ld_acc) + static_cast<uint32_t>(first_col)) * 4u;
            }
            if (kOut) {
                out_rsrc = __builtin_amdgcn_make_buffer_rsrc(p.out + row0 * p.ld_out, 0,
                                                             static_cast<int>(rows_here * p.ld_out * 4), kBufferFlags);
                out_lane = (static_cast<uint32_t>(dr) * static_cast<uint32_t>(p.ld_out) + static_cast<uint32_t>(first_col)) * 4u;
            }
        }
        // the next tile's first two chunks are requested before this tile's results are converted
        tile += stride;
        if (tile < p.n_tiles) {
            set_tile(tile);
            if (n_full > 0) load(0, s0);
            if (n_full > 1) load(1, s1);
        }

        // convert and park: accumulator register r of lane (i, h) holds row 8 (r / 4) + 4 h + r % 4 of
        // its 32 x 32 block and column i
#pragma unroll
        for (int rt = 0; rt < 4; ++rt) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = 32 * rt + 8 * (r >> 2) + 4 * half + (r & 3);
                int c4[4];
#pragma unroll
                for (int ct = 0; ct < 4; ++ct) c4[ct] = static_cast<int>(acc[rt][ct][r]);
                uint2 packed;
                packed.x = __builtin_amdgcn_perm(static_cast<uint32_t>(c4[1]), static_cast<uint32_t>(c4[0]), 0x05040100u);
                packed.y = __builtin_amdgcn_perm(static_cast<uint32_t>(c4[3]), static_cast<uint32_t>(c4[2]), 0x05040100u);
                *reinterpret_cast<uint2 *>(stage + row * kStageRowBytes + 8 * i32) = packed;
            }
        }
        slice = 0;
    }
    while (slice < kSlices) drain(slice++);                   // the last tile of this wavefront
}

// Shapes the tile kernel takes: enough columns to fill most of a 128-column tile, enough K for
// the multiplies to dominate; columns in whole groups of four (a lane writes four at a time) and
// leading dimensions (of the outputs and of the packed operands) small enough for 32-bit byte
// offsets inside a tile.
bool fp4_tile_covers(int64_t m, int64_t n, int64_t k_bits, int64_t ld_acc, int64_t ld_out, int64_t lda, int64_t ldb)
{
    if (lda >= (1 << 21) || ldb >= (1 << 21)) return false;
    return n > 64 && n % 4 == 0 && k_bits >= 512 && m >= 4096 && ld_acc < (1 << 21) && ld_out < (1 << 21);
}

template <bool kAcc, bool kOut>
static void launch_tile(dim3 grid, int n_chunks, hipStream_t stream, const TileArgs &p)
{
    if (n_chunks >= 16)
        hipLaunchKernelGGL((bitgemm_fp4_tile_kernel<kAcc, kOut, 1>), grid, dim3(kBlock), 0, stream, p);
    else if (n_chunks >= 8)
        hipLaunchKernelGGL((bitgemm_fp4_tile_kernel<kAcc, kOut, 2>), grid, dim3(kBlock), 0, stream, p);
    else
        hipLaunchKernelGGL((bitgemm_fp4_tile_kernel<kAcc, kOut, 4>), grid, dim3(kBlock), 0, stream, p);
}

int launch_bitgemm_fp4_tile(const uint64_t *a_bits, const float *a_scale, int64_t m, int64_t lda,
                            const uint64_t *b_bits, const float *b_scale, int64_t n, int64_t ldb,
                            int64_t k_bits, int32_t *acc, int64_t ld_acc, float *out, int64_t ld_out,
                            hipStream_t stream)
{
    static_assert(BIGCN_MAX_K_BITS <= 32767, "results are parked as int16");
    if (!fp4_tile_covers(m, n, k_bits, acc != nullptr ? ld_acc : 0, out != nullptr ? ld_out : 0, lda, ldb)) return BIGCN_EINVAL;
    const int64_t row_tiles = (m + kTileRows - 1) / kTileRows;
    const int64_t col_tiles = (n + kTileCols - 1) / kTileCols;
    TileArgs p{a_bits, m, lda, b_bits, static_cast<int>(n), ldb, static_cast<int>(k_bits), a_scale, b_scale,
               acc, ld_acc, out, ld_out, row_tiles * col_tiles, static_cast<int>(col_tiles)};
    // one workgroup (four wavefronts, one per SIMD) per compute unit
    const int cus = bigcn::compute_units();
    const dim3 grid(static_cast<unsigned>(std::min<int64_t>(cus, (p.n_tiles + kWavesPerBlock - 1) / kWavesPerBlock)));
    const int n_chunks = static_cast<int>(k_bits / kChunkBits);
    if (acc != nullptr && out != nullptr) launch_tile<true, true>(grid, n_chunks, stream, p);
    else if (acc != nullptr) launch_tile<true, false>(grid, n_chunks, stream, p);
    else launch_tile<false, true>(grid, n_chunks, stream, p);
    return check_launch();
}

// Nothing but multiplies: the rate at which one wavefront per SIMD issues independent
// 32 x 32 x 64 FP4 multiplies on this device, with operands of pseudo-random +-1 codes (what the
// tile kernel above could reach if loads, code expansion and stores were free).  kExpand: the
// eight operands of every sixteen multiplies are expanded from packed bits (codes() above, one
// rotate to vary the bits) while the sixteen multiplies before them run, three vector instructions
// after every multiply: what the kernel could reach if only loads and stores were free.  (Expanded
// in one piece ahead of their own multiplies the same instructions cost a sixth more.)
template <bool kExpand>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(1, 1))) void fp4_multiply_rate_kernel(
    float *sink, int iterations)
{
    __shared__ unsigned char whole_cu[131072];               // one workgroup per compute unit, as the tile kernel
    if (iterations < 0) whole_cu[threadIdx.x] = 1;           // never: keeps the allocation
    uint32_t mag[3] = {0x44444444u, 0x22222222u, 0x11111111u};
#pragma unroll
    for (int d = 0; d < 3; ++d) asm volatile("" : "+v"(mag[d]));
    v16f acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;
    v8i a[4], b[4];
    uint32_t xa[4], xb[4];
    uint32_t x = 0x9e3779b9u * (blockIdx.x * kBlock + threadIdx.x + 1u);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        x ^= x << 13; x ^= x >> 17; x ^= x << 5;
        xa[q] = x;
        x ^= x << 13; x ^= x >> 17; x ^= x << 5;
        xb[q] = x;
        a[q] = codes<false>(xa[q], mag);
        b[q] = codes<true>(xb[q], mag);
    }
    // two operand sets in turn (the loop body is two steps, so that neither is ever copied): the
    // set of the next step is built while the current one is multiplied
    v8i a2[4], b2[4];
    auto step = [&](v8i (&ma)[4], v8i (&mb)[4], v8i (&na)[4], v8i (&nb)[4]) {
        if (kExpand) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                xa[q] = __builtin_amdgcn_alignbit(xa[q], xa[q], 1);
                xb[q] = __builtin_amdgcn_alignbit(xb[q], xb[q], 3);
                na[q] = codes<false>(xa[q], mag);
                nb[q] = codes<true>(xb[q], mag);
            }
        }
#pragma unroll
        for (int rt = 0; rt < 4; ++rt)
#pragma unroll
            for (int ct = 0; ct < 4; ++ct)
                acc[4 * rt + ct] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ma[rt], mb[ct], acc[4 * rt + ct], 4, 4, 0,
                                                                                   0x7f7f7f7f, 0, 0x7f7f7f7f);
        if (kExpand) {
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);      // one multiply,
                __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);      // three vector instructions
            }
        }
    };
    for (int it = 0; it + 2 <= iterations; it += 2) {
        if (kExpand) {
            step(a, b, a2, b2);
            step(a2, b2, a, b);
        } else {
            step(a, b, a, b);
            step(a, b, a, b);
        }
    }
    if (iterations & 1) step(a, b, a2, b2);
    float total = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) total += acc[i][r];
    sink[blockIdx.x * kBlock + threadIdx.x] = total;
}

static int launch_multiply_rate(bool expand, int iterations, float *sink, int64_t sink_floats, int64_t *multiply_accumulates,
                                void *stream)
{
    if (sink == nullptr || multiply_accumulates == nullptr) return BIGCN_ENULL;
    if (iterations <= 0 || iterations > (1 << 20)) return BIGCN_EINVAL;
    const int cus = compute_units();
    if (sink_floats < static_cast<int64_t>(cus) * kBlock) return BIGCN_EWORKSPACE;
    if (expand)
        hipLaunchKernelGGL(fp4_multiply_rate_kernel<true>, dim3(cus), dim3(kBlock), 0, as_stream(stream), sink, iterations);
    else
        hipLaunchKernelGGL(fp4_multiply_rate_kernel<false>, dim3(cus), dim3(kBlock), 0, as_stream(stream), sink, iterations);
    *multiply_accumulates = static_cast<int64_t>(cus) * kWavesPerBlock * iterations * 16 * (32 * 32 * 64);
    return check_launch();
}

}  // namespace bigcn

extern "C" int bigcn_probe_fp4_multiply_rate(int iterations, float *sink, int64_t sink_floats,
                                             int64_t *multiply_accumulates, void *stream)
{
    return bigcn::launch_multiply_rate(false, iterations, sink, sink_floats, multiply_accumulates, stream);
}

extern "C" int bigcn_probe_fp4_expand_multiply_rate(int iterations, float *sink, int64_t sink_floats,
                                                    int64_t *multiply_accumulates, void *stream)
{
    return bigcn::launch_multiply_rate(true, iterations, sink, sink_floats, multiply_accumulates, stream);
}
