// Kernel 3: aggregation with the normalised adjacency, H = A~ Z (Sec. 4.2.3), as a CSR
// sparse-dense product, and its fused form used by the layer driver.
//
// The kernel is a gather: for every stored neighbour k of node i one dense row of Z is read
// from HBM and accumulated in fp32.  Mapping for wave64:
//   * a stored row of Z occupies `G` lanes x `V` consecutive values (one 8- or 16-byte load
//     per lane), so a wavefront covers 64/G neighbours per load instruction when rows are
//     narrow, and one neighbour when a row spans all 64 lanes;
//   * column indices (and the per-neighbour weights) of up to 64 neighbours are fetched with
//     one coalesced load and handed out by lane broadcast, so the inner loop issues only row
//     loads and FMAs, four row loads in flight per wavefront;
//   * rows are taken in order of decreasing length (plan): the longest rows are started
//     first and each is shared by the four wavefronts of a workgroup (partial sums combined
//     through LDS in a fixed order); every other row is owned by one wavefront.
// All sums are evaluated in a fixed order, so results are bit-identical from run to run.
#include <type_traits>

#include "bigcn_internal.h"

namespace bigcn {

// Where the per-neighbour weight comes from: all ones, a per-entry array, a per-node array
// gathered through the column index, the last four bytes of the gathered row itself, or the top
// bits of the first byte of each lane's segment of the gathered row (7-bit products).
// kWeightTopBitsEscape: as kWeightTopBits for layers whose products usually, but not provably,
// fit 7 bits: a row that does not is stored with a NaN scale, and its true values (one byte each)
// and scale are fetched from an alternate row array and the per-node scale array.
enum WeightMode {
    kWeightOne = 0, kWeightVals = 1, kWeightGather = 2, kWeightEmbedded = 3, kWeightTopBits = 4,
    kWeightTopBitsEscape = 5,        // alternate rows hold one byte per value
    kWeightTopBitsEscapeF16 = 6,     // ... one fp16 per value (layers of more than 256 input bits)
    kWeightLastBytes = 7,            // rows of 8 lanes: byte i of the weight is the last byte of lane 4 + i
    kWeightLastBytesEscapeF16 = 8    // ... with 8-bit products of more than 256 input bits: a row with a product
                                     //     outside [-127, 126] carries a NaN scale and lives as fp16 in the alternate array
};
__host__ __device__ constexpr bool top_bit_weights(int wm) { return wm >= kWeightTopBits && wm <= kWeightTopBitsEscapeF16; }
__host__ __device__ constexpr bool escape_weights(int wm)
{
    return wm == kWeightTopBitsEscape || wm == kWeightTopBitsEscapeF16 || wm == kWeightLastBytesEscapeF16;
}
__host__ __device__ constexpr bool last_byte_weights(int wm) { return wm == kWeightLastBytes || wm == kWeightLastBytesEscapeF16; }
__host__ __device__ constexpr bool half_alternates(int wm) { return wm == kWeightTopBitsEscapeF16 || wm == kWeightLastBytesEscapeF16; }
__host__ __device__ constexpr bool fused_weights(int wm) { return wm >= kWeightGather; }
__host__ __device__ constexpr bool row_weights(int wm) { return wm >= kWeightEmbedded; }

// ---- one stored row segment: V values of T per lane, loaded as one vector ------------------
template <typename T, int V>
struct Segment;

template <>
struct Segment<float, 1> {
    float raw;
    __device__ __forceinline__ void load(const char *p) { raw = *reinterpret_cast<const float *>(p); }
    __device__ __forceinline__ void fma(float w, float (&acc)[1]) const { acc[0] = fmaf(w, raw, acc[0]); }
};
template <>
struct Segment<float, 4> {
    float4 raw;
    __device__ __forceinline__ void load(const char *p) { raw = *reinterpret_cast<const float4 *>(p); }
    __device__ __forceinline__ void fma(float w, float (&acc)[4]) const
    {
        acc[0] = fmaf(w, raw.x, acc[0]);
        acc[1] = fmaf(w, raw.y, acc[1]);
        acc[2] = fmaf(w, raw.z, acc[2]);
        acc[3] = fmaf(w, raw.w, acc[3]);
    }
};
template <>
struct Segment<float, 8> {
    float4 lo, hi;
    __device__ __forceinline__ void load(const char *p)
    {
        lo = *reinterpret_cast<const float4 *>(p);
        hi = *reinterpret_cast<const float4 *>(p + 16);
    }
    __device__ __forceinline__ void fma(float w, float (&acc)[8]) const
    {
        acc[0] = fmaf(w, lo.x, acc[0]);
        acc[1] = fmaf(w, lo.y, acc[1]);
        acc[2] = fmaf(w, lo.z, acc[2]);
        acc[3] = fmaf(w, lo.w, acc[3]);
        acc[4] = fmaf(w, hi.x, acc[4]);
        acc[5] = fmaf(w, hi.y, acc[5]);
        acc[6] = fmaf(w, hi.z, acc[6]);
        acc[7] = fmaf(w, hi.w, acc[7]);
    }
};
template <>
struct Segment<__half, 4> {
    uint2 raw;
    __device__ __forceinline__ void load(const char *p) { raw = *reinterpret_cast<const uint2 *>(p); }
    __device__ __forceinline__ void fma(float w, float (&acc)[4]) const
    {
        const __half2 a = *reinterpret_cast<const __half2 *>(&raw.x);
        const __half2 b = *reinterpret_cast<const __half2 *>(&raw.y);
        acc[0] = fmaf(w, __low2float(a), acc[0]);
        acc[1] = fmaf(w, __high2float(a), acc[1]);
        acc[2] = fmaf(w, __low2float(b), acc[2]);
        acc[3] = fmaf(w, __high2float(b), acc[3]);
    }
};
template <>
struct Segment<__half, 8> {
    uint4 raw;
    __device__ __forceinline__ void load(const char *p) { raw = *reinterpret_cast<const uint4 *>(p); }
    __device__ __forceinline__ void fma(float w, float (&acc)[8]) const
    {
        const __half2 *h = reinterpret_cast<const __half2 *>(&raw);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            acc[2 * q] = fmaf(w, __low2float(h[q]), acc[2 * q]);
            acc[2 * q + 1] = fmaf(w, __high2float(h[q]), acc[2 * q + 1]);
        }
    }
};
// four signed bytes -> fp32 (sign-extending bit-field extract, then convert), multiplied and
// accumulated.  kCarrier: the first byte holds a 7-bit value under a foreign top bit (a bit of
// the row's scale) and is sign-extended from its bit 6.
template <bool kCarrier>
__device__ __forceinline__ void fma_bytes(float w, uint32_t word, float *acc)
{
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int value = (kCarrier && e == 0) ? (static_cast<int>(word << 25) >> 25)
                                               : (static_cast<int>(word << (24 - 8 * e)) >> 24);
        acc[e] = fmaf(w, static_cast<float>(value), acc[e]);
    }
}
template <>
struct Segment<int8_t, 8> {
    uint2 raw;
    __device__ __forceinline__ void load(const char *p) { raw = *reinterpret_cast<const uint2 *>(p); }
    __device__ __forceinline__ void fma(float w, float (&acc)[8]) const
    {
        fma_bytes<false>(w, raw.x, acc);
        fma_bytes<false>(w, raw.y, acc + 4);
    }
    // rows that carry scale bits in the top bit of the first byte (and, kMiddle, of the fifth)
    template <bool kMiddle>
    __device__ __forceinline__ void fma_carrier(float w, float (&acc)[8]) const
    {
        fma_bytes<true>(w, raw.x, acc);
        fma_bytes<kMiddle>(w, raw.y, acc + 4);
    }
    __device__ __forceinline__ uint32_t tail() const { return raw.y; }
    __device__ __forceinline__ uint32_t head() const { return raw.x; }
    __device__ __forceinline__ uint32_t middle() const { return raw.y; }
    __device__ __forceinline__ void clear() { raw = make_uint2(0u, 0u); }
};
// The fp32 weight stored inside a loaded row, handed to every lane of the row's group.
//   kWeightEmbedded: the row's last four bytes, held by the last lane of the group;
//   kWeightLastBytes: rows of 8 lanes; byte i of the weight is the last byte of lane 4 + i;
//   kWeightTopBits:  bit i of the weight is the top bit of the first byte of lane i's segment
//                    (groups of 32 or 64 lanes; groups of 16 lanes keep bits 16..31 in the top
//                    bit of the fifth byte); one ballot per carrier byte collects the bits of all
//                    rows that a load instruction covers.  The carrier bytes keep the foreign bit:
//                    accumulate_segment sign-extends them from bit 6.
template <typename T, int G, int V, int WM>
__device__ __forceinline__ float row_weight(Segment<T, V> &seg, int lane, bool loaded)
{
    if constexpr (sizeof(T) == 1 && WM == kWeightEmbedded) {
        return __uint_as_float(static_cast<uint32_t>(__shfl(static_cast<int>(seg.tail()), lane | (G - 1), kWave)));
    } else if constexpr (sizeof(T) == 1 && last_byte_weights(WM)) {
        static_assert(sizeof(T) != 1 || !last_byte_weights(WM) || (G == 8 && V == 8), "rows of 8 lanes x 8 values");
        // lanes 4..7 of a row are one quad: each of them collects the four bytes by quad
        // broadcasts (data-parallel moves, no LDS traffic), then one shuffle hands the word of
        // lane 4 to the row's eight lanes
        const int top = static_cast<int>(seg.tail() >> 24);
        const uint32_t b0 = static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, top, 0x00, 0xf, 0xf, false));
        const uint32_t b1 = static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, top, 0x55, 0xf, 0xf, false));
        const uint32_t b2 = static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, top, 0xaa, 0xf, 0xf, false));
        const uint32_t b3 = static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, top, 0xff, 0xf, 0xf, false));
        const int word = static_cast<int>(b0 | (b1 << 8) | (b2 << 16) | (b3 << 24));
        return __uint_as_float(static_cast<uint32_t>(__shfl(word, (lane & ~(G - 1)) + G - 4, kWave)));
    } else if constexpr (sizeof(T) == 1 && top_bit_weights(WM)) {
        const uint64_t bits = __ballot(loaded && (seg.head() & 0x80u) != 0);
        if constexpr (G >= 32) {
            const uint32_t mine = (G == kWave || lane < 32) ? static_cast<uint32_t>(bits) : static_cast<uint32_t>(bits >> 32);
            return __uint_as_float(mine);
        } else {
            const uint64_t high = __ballot(loaded && (seg.middle() & 0x80u) != 0);
            const int shift = lane & ~(G - 1);           // first lane of this lane's group (G = 16)
            const uint32_t mine = (static_cast<uint32_t>(bits >> shift) & 0xffffu) |
                                  ((static_cast<uint32_t>(high >> shift) & 0xffffu) << 16);
            return __uint_as_float(mine);
        }
    } else {
        return 0.0f;
    }
}

// Per-node accumulators of a lane: V positions of the weighted row sum, plus (fused path only)
// the sum of the weight magnitudes and the sum of the signed weights.
template <int V>
struct RowAcc {
    float pos[V];
    float sum_abs;      // sum_k |w_k|
    float sum_signed;   // sum_k w_k   (the sign of w_k carries the last input bit of node k)
    __device__ __forceinline__ void clear()
    {
#pragma unroll
        for (int v = 0; v < V; ++v) pos[v] = 0.0f;
        sum_abs = 0.0f;
        sum_signed = 0.0f;
    }
};

// Address of a lane's segment of stored row k: one 32 x 32 -> 64 bit multiply-add onto the array's
// wave-uniform base (row indices and row strides are below 2^32; the launchers check the stride).
// A 24-bit multiply with a 32-bit offset was measured on arrays below 4 GiB: 0.5 % faster, not
// worth a second set of kernels.
struct RowBase {
    const char *base;      // wave-uniform
    uint32_t lane_off;     // byte offset of this lane's segment inside a row
};
__device__ __forceinline__ const char *row_address(const RowBase &rb, int k, uint32_t row_bytes)
{
    return rb.base + rb.lane_off + static_cast<uint64_t>(static_cast<uint32_t>(k)) * row_bytes;
}

// acc += w * (the V values of a loaded segment); rows with the scale in their top bits keep the
// scale bits in their carrier bytes (first byte; fifth byte too for rows of 16 lanes).
template <typename T, int G, int V, int WM>
__device__ __forceinline__ void accumulate_segment(const Segment<T, V> &seg, float w, float (&acc)[V])
{
    if constexpr (sizeof(T) == 1 && top_bit_weights(WM)) seg.template fma_carrier<(G < 32)>(w, acc);
    else seg.fma(w, acc);
}

// The weight a loaded row carries; with the escape modes also the rare replacement of a row that
// did not fit 7 bits (NaN scale): its values come from the alternate array and its scale from the
// per-node array.  The alternate values (one byte or fp16 each) are accumulated here (with |w|,
// as the caller would) and the segment is cleared.  Executed by all
// lanes; `loaded` says whether this lane's segment was fetched; alt_row_bytes = bytes of an
// alternate row, alt_lane_base already points at this lane's first value.
template <typename T, int G, int V, int WM>
__device__ __forceinline__ float resolve_row(Segment<T, V> &seg, int lane, bool loaded, int k,
                                             const RowBase &alt_lane_base, uint32_t alt_row_bytes,
                                             const float *__restrict__ weights, float (&acc)[V])
{
    float w = row_weight<T, G, V, WM>(seg, lane, loaded);
    if constexpr (escape_weights(WM) && sizeof(T) == 1) {
        const bool escaped = loaded && !(fabsf(w) <= 3.0e38f);      // NaN (or Inf) marks the row
        if (__ballot(escaped) != 0ull) {
            if (escaped) {
                const char *src = row_address(alt_lane_base, k, alt_row_bytes);
                w = weights[k];
                if constexpr (WM == kWeightTopBitsEscape) {
                    // full one-byte values: accumulated here, the 7-bit segment is cleared
                    Segment<T, V> alt;
                    alt.load(src);
                    alt.fma(fabsf(w), acc);
                    seg.clear();
                } else {
                    static_assert(V == 8, "fp16 alternates are read as one 16-byte vector per lane");
                    const float aw = fabsf(w);
                    const uint4 raw = *reinterpret_cast<const uint4 *>(src);
                    const __half2 *h = reinterpret_cast<const __half2 *>(&raw);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        acc[2 * q] = fmaf(aw, __low2float(h[q]), acc[2 * q]);
                        acc[2 * q + 1] = fmaf(aw, __high2float(h[q]), acc[2 * q + 1]);
                    }
                    seg.clear();
                }
            }
        }
    }
    return w;
}

// ---- accumulate the neighbours p0..p1-1 of one node (per lane: V positions) ---------------
// active: this lane's positions exist in the stored row (lanes past the row width never load);
// kAllActive: known at compile time to hold for every lane (stored rows of the fused path),
// which keeps the loop free of per-lane predication.
// In gather mode the row values are weighted by |w| and both sum |w| and sum w are kept.
template <typename T, int G, int V, int WM, bool kAllActive>
__device__ __forceinline__ void accumulate_range(const int32_t *__restrict__ col_idx,
                                                 const float *__restrict__ weights,
                                                 const RowBase &lane_base,
                                                 const RowBase &alt_lane_base, uint32_t row_bytes,
                                                 uint32_t alt_row_bytes, int64_t p0, int64_t p1, int lane,
                                                 bool active_in, RowAcc<V> &acc)
{
    const bool active = kAllActive || active_in;
    constexpr int S = kWave / G;      // neighbours covered by one load instruction
    constexpr int U = 4;              // load instructions in flight (4 measured best: more costs occupancy)
    const int slot = lane / G;

    for (int64_t pb = p0; pb < p1; pb += kWave) {
        const int cnt = static_cast<int>(p1 - pb < kWave ? p1 - pb : kWave);     // wave-uniform
        int k = 0;
        float wk = 0.0f;
        if (lane < cnt) {
            k = col_idx[pb + lane];
            if (WM == kWeightVals) wk = weights[pb + lane];
            else if (WM == kWeightGather) wk = weights[k];
            else if (WM == kWeightOne) wk = 1.0f;
        }
        int t = 0;
        // full groups: S*U neighbours, all present
        for (; t + S * U <= cnt; t += S * U) {
            Segment<T, V> seg[U];
            float w[U];
            int kk[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (S == 1) {
                    kk[u] = __builtin_amdgcn_readlane(k, t + u);
                    w[u] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wk), t + u));
                } else {
                    kk[u] = __shfl(k, t + u * S + slot, kWave);
                    w[u] = __shfl(wk, t + u * S + slot, kWave);
                }
                if (active) seg[u].load(row_address(lane_base, kk[u], row_bytes));
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (row_weights(WM))
                    w[u] = resolve_row<T, G, V, WM>(seg[u], lane, active, kk[u], alt_lane_base, alt_row_bytes, weights,
                                                    acc.pos);
                if (fused_weights(WM)) {
                    acc.sum_abs += fabsf(w[u]);
                    acc.sum_signed += w[u];
                    if (active) accumulate_segment<T, G, V, WM>(seg[u], fabsf(w[u]), acc.pos);
                } else {
                    if (active) accumulate_segment<T, G, V, WM>(seg[u], w[u], acc.pos);
                }
            }
        }
        // tail: fewer than S*U neighbours left in this batch; one predicated group so that
        // the remaining loads are still issued back to back
        if (t < cnt) {
            Segment<T, V> seg[U];
            float w[U];
            int kk[U];
            bool present[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int src = t + u * S + slot;
                present[u] = src < cnt;
                const int from = present[u] ? src : 0;
                kk[u] = __shfl(k, from, kWave);
                w[u] = __shfl(wk, from, kWave);
                if (active && present[u]) seg[u].load(row_address(lane_base, kk[u], row_bytes));
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                // the broadcast is executed by all lanes; slots without a neighbour discard it
                if (row_weights(WM))
                    w[u] = resolve_row<T, G, V, WM>(seg[u], lane, active && present[u], kk[u], alt_lane_base,
                                                    alt_row_bytes, weights, acc.pos);
                if (present[u]) {
                    if (fused_weights(WM)) {
                        acc.sum_abs += fabsf(w[u]);
                        acc.sum_signed += w[u];
                        if (active) accumulate_segment<T, G, V, WM>(seg[u], fabsf(w[u]), acc.pos);
                    } else {
                        if (active) accumulate_segment<T, G, V, WM>(seg[u], w[u], acc.pos);
                    }
                }
            }
        }
    }
}

// The node's own stored row (second product array of a layer with an own-row term), weighted by
// the node's own scale exactly as a neighbour's row would be: pos = |t| * stored, sums of t.
template <typename T, int G, int V, int WM>
__device__ __forceinline__ void load_own_row(const RowBase &own_lane_base,
                                             const RowBase &own_alt_lane_base, uint32_t row_bytes,
                                             uint32_t alt_row_bytes, const float *__restrict__ weights,
                                             int64_t row, int lane, bool active, RowAcc<V> &own)
{
    own.clear();
    Segment<T, V> seg;
    if (active) seg.load(row_address(own_lane_base, static_cast<int>(row), row_bytes));
    float t;
    if (row_weights(WM))
        t = resolve_row<T, G, V, WM>(seg, lane, active, static_cast<int>(row), own_alt_lane_base, alt_row_bytes,
                                     weights, own.pos);
    else t = weights[row];
    own.sum_abs = fabsf(t);
    own.sum_signed = t;
    if (active) accumulate_segment<T, G, V, WM>(seg, fabsf(t), own.pos);
}

// x + (x of lane ^ kOff): the partner's value comes by a swap of 32- or 16-lane rows or a
// rotation inside a row of 16 or a quad where the vector ALU can do that itself (kOff = 32, 16, 8, 2), by a
// shuffle through the LDS crossbar otherwise.  The same pairs are added either way.
template <int kOff>
__device__ __forceinline__ float add_xor_lane(float x)
{
    const unsigned bits = __float_as_uint(x);
    if constexpr (kOff == 32) {
        const auto r = __builtin_amdgcn_permlane32_swap(bits, bits, false, false);
        return __uint_as_float(r[0]) + __uint_as_float(r[1]);
    } else if constexpr (kOff == 16) {
        const auto r = __builtin_amdgcn_permlane16_swap(bits, bits, false, false);
        return __uint_as_float(r[0]) + __uint_as_float(r[1]);
    } else if constexpr (kOff == 8) {
        return x + __uint_as_float(static_cast<unsigned>(
                       __builtin_amdgcn_update_dpp(0, static_cast<int>(bits), 0x128, 0xf, 0xf, false)));   // row_ror:8
    } else if constexpr (kOff == 2) {
        return x + __uint_as_float(static_cast<unsigned>(
                       __builtin_amdgcn_update_dpp(0, static_cast<int>(bits), 0x4e, 0xf, 0xf, false)));    // quad_perm [2, 3, 0, 1]
    } else {
        return x + __shfl_xor(x, kOff, kWave);
    }
}

// Sum the partial results of the 64/G lane slots; afterwards every lane holds the total.
template <int G, int V, int WM, int kOff = G>
__device__ __forceinline__ void reduce_slots(RowAcc<V> &acc)
{
    if constexpr (kOff < kWave) {
#pragma unroll
        for (int v = 0; v < V; ++v) acc.pos[v] = add_xor_lane<kOff>(acc.pos[v]);
        if (fused_weights(WM)) {
            acc.sum_abs = add_xor_lane<kOff>(acc.sum_abs);
            acc.sum_signed = add_xor_lane<kOff>(acc.sum_signed);
        }
        reduce_slots<G, V, WM, 2 * kOff>(acc);
    }
}

// ---- epilogues ---------------------------------------------------------------------------------
// An epilogue has per-lane constants (`Lane<G, V>`: a struct of floats, computed once per
// workgroup by `init`) and a `finish` that turns the accumulators of one node into its outputs.

// Public SpMM: stored position == output column, fp32 row-major output.
struct EpiloguePlain {
    static constexpr bool kSelf = false;
    float *out;
    int64_t ld_out;
    int d;                 // valid positions
    int vector_store;      // 1: V floats of a lane can be written as one aligned vector
    template <int G, int V>
    struct Lane {};
    template <int G, int V>
    __device__ __forceinline__ void init(int, Lane<G, V> &) const {}
    template <int G, int V>
    __device__ __forceinline__ void finish(const Lane<G, V> &, int64_t row, int lane, const RowAcc<V> &acc,
                                           const RowAcc<V> &) const
    {
        if (lane >= G) return;
        float *dst = out + row * ld_out + lane * V;
        if (V == 4 && vector_store) {
            if (lane * V < d)
                *reinterpret_cast<float4 *>(dst) = make_float4(acc.pos[0], acc.pos[1], acc.pos[2], acc.pos[3]);
        } else {
#pragma unroll
            for (int v = 0; v < V; ++v)
                if (lane * V + v < d) dst[v] = acc.pos[v];
        }
    }
};

// Fused layer: stored position g*V + v holds column g + G*v of the stored products.  The
// neighbour sum of the true products is  mul * acc + bias * sum|w| + (+-1)_j * sum w  (the last
// term only with a folded last bit); it is rescaled by dst_mul_i * alpha_j and either written as
// fp32 output or turned directly into the packed signs and the scale of the next layer's input.
//   Bi-GCN (Sec. 4.2.3):        dst_mul = D^-1/2, the source weights carry D^-1/2 beta.
//   Bi-GraphSAGE (Sec. 4.4.2):  dst_mul = 1/|N_i|, the source weights carry beta, and the node's
//                               own product row (second weight matrix) is added: kSelfTerm.
template <bool kSelfTerm>
struct EpilogueFusedT {
    static constexpr bool kSelf = kSelfTerm;
    const float *dst_mul;
    const float *alpha;
    int d_out;
    float mul;
    float bias;
    const uint64_t *last_bit_word;   // &w_bits[(K-1)/64] of column 0, or nullptr without folded bit
    int64_t w_ld_words;
    int last_bit_shift;              // (K-1) % 64
    float *logits;
    int64_t ld_logits;
    const float *next_shift;
    const float *next_mul;
    uint64_t *next_bits;
    int64_t next_ld_words;
    float *next_scale;
    const float *next_row_mul;       // nullable: per-node factor folded into the next stored scale
    int next_fold_last_sign;
    // own-row term (kSelfTerm only): rows in the same layout, their column scales and last bits
    const char *self_rows;
    const char *alt_self_rows;       // own rows that did not fit 7 bits (escape layouts; bytes or fp16)
    const float *self_alpha;
    const uint64_t *self_last_bit_word;

    template <int G, int V>
    struct Lane {
        float alpha[V];      // 0 for columns past d_out
        float last[V];       // +-1: sign of the weight's last input bit, 0 without folded bit
        float shift[V];
        float mul[V];
        float self_alpha[kSelfTerm ? V : 1];
        float self_last[kSelfTerm ? V : 1];
    };
    template <int G, int V>
    __device__ __forceinline__ void init(int lane, Lane<G, V> &c) const
    {
        const int g = lane & (G - 1);
#pragma unroll
        for (int v = 0; v < V; ++v) {
            const int col = g + G * v;
            const bool in = col < d_out;
            c.alpha[v] = in ? alpha[col] : 0.0f;
            c.last[v] = 0.0f;
            if (in && last_bit_word != nullptr)
                c.last[v] = ((last_bit_word[col * w_ld_words] >> last_bit_shift) & 1ull) ? 1.0f : -1.0f;
            c.shift[v] = (in && next_shift != nullptr) ? next_shift[col] : 0.0f;
            c.mul[v] = (in && next_mul != nullptr) ? next_mul[col] : 1.0f;
            if constexpr (kSelfTerm) {
                c.self_alpha[v] = in ? self_alpha[col] : 0.0f;
                c.self_last[v] = 0.0f;
                if (in && self_last_bit_word != nullptr)
                    c.self_last[v] = ((self_last_bit_word[col * w_ld_words] >> last_bit_shift) & 1ull) ? 1.0f : -1.0f;
            }
        }
    }
    template <int G, int V>
    __device__ __forceinline__ void finish(const Lane<G, V> &c, int64_t row, int lane, const RowAcc<V> &acc,
                                           const RowAcc<V> &self) const
    {
        const float di = dst_mul[row];
        const int g = lane & (G - 1);
        const bool first_slot = lane < G;
        const float base = bias * acc.sum_abs;
        float h[V];
#pragma unroll
        for (int v = 0; v < V; ++v) {
            const float total = fmaf(mul, acc.pos[v], fmaf(c.last[v], acc.sum_signed, base));
            h[v] = di * c.alpha[v] * total;
            if constexpr (kSelfTerm) {
                // the node's own products, weighted by its own scale (sign = its last input bit)
                const float own = fmaf(mul, self.pos[v], fmaf(c.self_last[v], self.sum_signed, bias * self.sum_abs));
                h[v] = fmaf(c.self_alpha[v], own, h[v]);
            }
        }
        if (logits != nullptr) {
            if (first_slot) {
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    const int col = g + G * v;
                    if (col < d_out) logits[row * ld_logits + col] = h[v];
                }
            }
            return;
        }
        // binarise for the next layer: bit (G*v + g) of the row's bit string is column g + G*v
        constexpr int kWords = (G * V + 63) / 64;
        uint64_t words[kWords];
#pragma unroll
        for (int q = 0; q < kWords; ++q) words[q] = 0;
        float sum = 0.0f;
#pragma unroll
        for (int v = 0; v < V; ++v) {
            const int col = g + G * v;
            const bool valid = first_slot && col < d_out;
            const uint64_t mask = __ballot(valid && h[v] >= c.shift[v]);   // only the low G lanes can be set
            words[(G * v) / 64] |= mask << ((G * v) % 64);
            sum += valid ? fabsf((h[v] - c.shift[v]) * c.mul[v]) : 0.0f;
        }
        sum = wave_sum_dpp(sum);
        const int n_words = (d_out + 63) >> 6;
#pragma unroll
        for (int q = 0; q < kWords; ++q)
            if (lane == q && q < n_words) next_bits[row * next_ld_words + q] = words[q];
        if (lane == 0) {
            float s = sum / static_cast<float>(d_out);
            if (next_row_mul != nullptr) s *= next_row_mul[row];
            if (next_fold_last_sign) {
                uint64_t last = 0;
#pragma unroll
                for (int q = 0; q < kWords; ++q)
                    if (q == ((d_out - 1) >> 6)) last = words[q];
                if (((last >> ((d_out - 1) & 63)) & 1ull) == 0) s = -s;
            }
            next_scale[row] = s;
        }
    }
};

// The per-lane constants of an epilogue are needed once per node, after the gather; held in
// registers for the whole kernel they would cost occupancy in the loop that matters.  They are
// parked in LDS and fetched back by `finish`.  They depend on the lane's place in its group only,
// so G lanes' worth is kept ([constant][place]: the 64 lanes read G consecutive words, conflict-free).
template <class L, int G>
struct ParkedLane {
    static constexpr int kFloats = std::is_empty<L>::value ? 0 : static_cast<int>(sizeof(L) / sizeof(float));
    static __device__ __forceinline__ void park(const L &c, float *lds, int lane)
    {
        const float *src = reinterpret_cast<const float *>(&c);
        if (lane < G) {
#pragma unroll
            for (int k = 0; k < kFloats; ++k) lds[k * G + lane] = src[k];
        }
    }
    static __device__ __forceinline__ void fetch(L &c, const float *lds, int lane)
    {
        asm volatile("" ::: "memory");      // keep the reads here: not hoisted out of the row loop
        float *dst = reinterpret_cast<float *>(&c);
#pragma unroll
        for (int k = 0; k < kFloats; ++k) dst[k] = lds[k * G + (lane & (G - 1))];
    }
};

// ---- the kernel ------------------------------------------------------------------------------
// Rows are taken in plan order.  Workgroup b < n_block_rows owns one long row; every later
// workgroup owns rows_per_wave * 4 consecutive plan entries, wavefront w taking entries
// base + w, base + w + 4, ... (neighbouring entries have similar lengths).  A wavefront takes 16
// rows one after the other when there are enough rows to fill the chip several times over (the
// epilogue constants are fetched once per workgroup); on small graphs, where the time of a
// launch is the latency of one wavefront's chain of dependent loads, it takes fewer, down to one.
constexpr int kMaxRowsPerWave = 16;
static int rows_per_wave_for(int64_t wave_rows, int compute_units)
{
    // one row per wavefront until the rows fill the chip four times over (measured on the
    // 19717- and 232965-node workloads), then proportionally more
    const int64_t resident_waves = static_cast<int64_t>(compute_units) * 4 * 8;   // x SIMDs x wavefronts per SIMD
    const int64_t r = wave_rows / (4 * resident_waves);
    return static_cast<int>(r < 1 ? 1 : (r > kMaxRowsPerWave ? kMaxRowsPerWave : r));
}

// Wavefronts per SIMD the register allocation aims for.  The gather hides HBM latency with
// resident wavefronts, so the one-byte rows of the Bi-GCN path (which fit 64 registers without
// spilling) ask for the maximum of 8.  With an own-row term the second accumulator set does not
// fit 64 registers: 6 wavefronts (80 registers) measured best, 7 (72 registers) for
// full-wavefront rows with the escape test.  Wider element types keep the compiler's own choice.
template <typename T, int G, int V, int WM, class Epilogue>
constexpr int spmm_min_waves()
{
    if (sizeof(T) != 1 || V != 8) return 1;
    if (!Epilogue::kSelf) return 8;
    return (G == kWave && escape_weights(WM)) ? 7 : 6;
}

// gate_flag (nullable): the launch does nothing unless (*gate_flag != 0) == (run_if_set != 0).
// Escape layouts with one-byte alternates (rows that may carry a NaN scale and live in the
// alternate array) are launched twice on the flag that the bit-GEMM sets when a row went to the
// alternate array: once as the plain top-bits kernel, which runs when no row did, once with the
// per-row test, which runs otherwise; one of the two returns at once (1.3 % of a forward on the
// largest workload, where no row ever escapes).  clear_flag: the flag of the layer that follows,
// cleared here, i.e. after the kernels that read it in the previous call and before the bit-GEMM
// that may set it in this one.
template <typename T, int G, int V, int WM, class Epilogue>
__global__ __launch_bounds__(kBlock, (spmm_min_waves<T, G, V, WM, Epilogue>())) void spmm_kernel(
    const bigcn_plan_entry *__restrict__ entries, int64_t n, int64_t n_block_rows,
    const int64_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx,
    const float *__restrict__ weights, const char *__restrict__ rows, const char *__restrict__ alt_rows,
    uint32_t row_bytes, int valid_positions, int rows_per_wave, Epilogue epi,
    const int *__restrict__ gate_flag, int run_if_set, int *__restrict__ clear_flag)
{
    if (clear_flag != nullptr && blockIdx.x == 0 && threadIdx.x == 0) *clear_flag = 0;
    if (gate_flag != nullptr && (*gate_flag != 0) != (run_if_set != 0)) return;     // uniform over the launch
    constexpr int kAltElem = half_alternates(WM) ? 2 : static_cast<int>(sizeof(T));
    const uint32_t alt_row_bytes = row_bytes / sizeof(T) * kAltElem;
    constexpr bool kAllActive = fused_weights(WM);     // stored rows of the fused path fill G * V positions
    __shared__ float partial[kWavesPerBlock - 1][V + 2][G];     // after reduce_slots the lanes of one place in their groups agree
    const int lane = lane_id();
    const int wave = wave_in_block();
    const int g = lane & (G - 1);
    const bool active = kAllActive || g * V < valid_positions;
    const RowBase lane_base{rows, static_cast<uint32_t>(g * V * sizeof(T))};

    using LaneConsts = typename Epilogue::template Lane<G, V>;
    using Parked = ParkedLane<LaneConsts, G>;
    __shared__ float parked[Parked::kFloats > 0 ? Parked::kFloats * G : 1];
    {
        LaneConsts ctx;
        epi.template init<G, V>(lane, ctx);
        if (wave == 0) Parked::park(ctx, parked, lane);     // identical in all four wavefronts
        __syncthreads();
    }
    RowAcc<V> acc;
    RowAcc<V> own;      // only filled (and only read) by epilogues with an own-row term
    // alternate rows of nodes whose products did not fit 7 bits; only dereferenced by the escape modes
    const RowBase alt_lane_base{alt_rows, static_cast<uint32_t>(g * V * kAltElem)};
    RowBase own_lane_base{nullptr, 0u};
    RowBase own_alt_lane_base{nullptr, 0u};
    if constexpr (Epilogue::kSelf) {
        own_lane_base = RowBase{epi.self_rows, static_cast<uint32_t>(g * V * sizeof(T))};
        own_alt_lane_base = RowBase{epi.alt_self_rows, static_cast<uint32_t>(g * V * kAltElem)};
    }

    if (static_cast<int64_t>(blockIdx.x) < n_block_rows) {
        // one long row shared by the four wavefronts: contiguous quarters, multiples of 64
        const bigcn_plan_entry e = entries[blockIdx.x];
        const int64_t row = e.row;
        const int64_t p0 = e.first, p1 = e.first + e.count;
        int64_t chunk = (p1 - p0 + kWavesPerBlock - 1) / kWavesPerBlock;
        chunk = (chunk + kWave - 1) / kWave * kWave;
        int64_t q0 = p0 + wave * chunk;
        int64_t q1 = q0 + chunk;
        if (q0 > p1) q0 = p1;
        if (q1 > p1) q1 = p1;
        acc.clear();
        accumulate_range<T, G, V, WM, kAllActive>(col_idx, weights, lane_base, alt_lane_base, row_bytes, alt_row_bytes, q0, q1, lane,
                                                  active, acc);
        reduce_slots<G, V, WM>(acc);
        if (wave > 0 && lane < G) {
#pragma unroll
            for (int v = 0; v < V; ++v) partial[wave - 1][v][lane] = acc.pos[v];
            partial[wave - 1][V][lane] = acc.sum_abs;
            partial[wave - 1][V + 1][lane] = acc.sum_signed;
        }
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int w = 0; w < kWavesPerBlock - 1; ++w) {
#pragma unroll
                for (int v = 0; v < V; ++v) acc.pos[v] += partial[w][v][g];
                acc.sum_abs += partial[w][V][g];
                acc.sum_signed += partial[w][V + 1][g];
            }
            if constexpr (Epilogue::kSelf)
                load_own_row<T, G, V, WM>(own_lane_base, own_alt_lane_base, row_bytes, alt_row_bytes, weights, row, lane, active, own);
            LaneConsts ctx;
            Parked::fetch(ctx, parked, lane);
            epi.template finish<G, V>(ctx, row, lane, acc, own);
        }
        return;
    }
    const int64_t base = n_block_rows +
                         (static_cast<int64_t>(blockIdx.x) - n_block_rows) * (kWavesPerBlock * rows_per_wave);
    for (int j = 0; j < rows_per_wave; ++j) {
        const int64_t entry = base + wave + j * kWavesPerBlock;
        if (entry >= n) break;                                   // wave-uniform
        const bigcn_plan_entry e = entries[entry];
        const int64_t row = e.row;
        const int64_t p0 = e.first, p1 = e.first + e.count;
        acc.clear();
        if constexpr (Epilogue::kSelf)
            load_own_row<T, G, V, WM>(own_lane_base, own_alt_lane_base, row_bytes, alt_row_bytes, weights, row, lane, active, own);
        accumulate_range<T, G, V, WM, kAllActive>(col_idx, weights, lane_base, alt_lane_base, row_bytes, alt_row_bytes, p0, p1, lane,
                                                  active, acc);
        reduce_slots<G, V, WM>(acc);
        LaneConsts ctx;
        Parked::fetch(ctx, parked, lane);
        epi.template finish<G, V>(ctx, row, lane, acc, own);
    }
}

template <typename T, int G, int V, int WM, class Epilogue>
static int launch_spmm_one(const bigcn_plan *plan, const int64_t *row_ptr, const int32_t *col_idx,
                           const float *weights, const void *rows, int64_t row_bytes,
                           int valid_positions, const Epilogue &epi, hipStream_t stream,
                           const void *alt_rows, const int *gate_flag = nullptr, int run_if_set = 0,
                           int *clear_flag = nullptr)
{
    if (row_bytes <= 0 || row_bytes > 0x7fffffff) return BIGCN_EINVAL;
    if (escape_weights(WM) && (alt_rows == nullptr || weights == nullptr)) return BIGCN_ENULL;
    if (fused_weights(WM) && valid_positions != G * V) return BIGCN_EINVAL;
    const int64_t wave_rows = plan->n - plan->n_split_rows;
    int rows_per_wave = rows_per_wave_for(wave_rows, plan->compute_units);
    // the launch that only runs when a row escaped (almost never): a quarter of the workgroups, so
    // that returning at once costs a quarter
    if (gate_flag != nullptr && run_if_set != 0 && rows_per_wave == kMaxRowsPerWave) rows_per_wave *= 4;
    const int64_t per_block = kWavesPerBlock * rows_per_wave;
    const int64_t blocks = plan->n_split_rows + (wave_rows + per_block - 1) / per_block;
    if (blocks == 0) return BIGCN_OK;
    hipLaunchKernelGGL((spmm_kernel<T, G, V, WM, Epilogue>), dim3(static_cast<unsigned>(blocks)),
                       dim3(kBlock), 0, stream, plan->entries, plan->n, plan->n_split_rows, row_ptr,
                       col_idx, weights, static_cast<const char *>(rows), static_cast<const char *>(alt_rows),
                       static_cast<uint32_t>(row_bytes), valid_positions, rows_per_wave, epi, gate_flag, run_if_set, clear_flag);
    return check_launch();
}

template <typename T, int V, int WM, class Epilogue>
static int launch_spmm_groups(int groups, const bigcn_plan *plan, const int64_t *row_ptr,
                              const int32_t *col_idx, const float *weights, const void *rows,
                              int64_t row_bytes, int valid_positions, const Epilogue &epi,
                              hipStream_t stream, const void *alt_rows = nullptr, const int *gate_flag = nullptr,
                              int run_if_set = 0, int *clear_flag = nullptr)
{
#define BIGCN_SPMM_CASE(GG)                                                                          \
    case GG:                                                                                         \
        return launch_spmm_one<T, GG, V, WM>(plan, row_ptr, col_idx, weights, rows, row_bytes,      \
                                             valid_positions, epi, stream, alt_rows, gate_flag, run_if_set, clear_flag)
    switch (groups) {
        BIGCN_SPMM_CASE(2);
        BIGCN_SPMM_CASE(4);
        BIGCN_SPMM_CASE(8);
        BIGCN_SPMM_CASE(16);
        BIGCN_SPMM_CASE(32);
        BIGCN_SPMM_CASE(64);
    default:
        return BIGCN_EINVAL;
    }
#undef BIGCN_SPMM_CASE
}

static int groups_for(int64_t positions, int vec)
{
    int g = 2;
    while (g < 64 && static_cast<int64_t>(g) * vec < positions) g <<= 1;
    return g;
}

// Largest layer input for which products are stored in 7 bits with an fp16 alternate (see below);
// with positions <= 512 the bit-GEMM then still holds a whole row in one wavefront.
constexpr int64_t kMaxEscapeBits = 1024;

RowLayout choose_layout(int64_t d_in, int64_t d_out)
{
    RowLayout l;
    if (d_in <= 256) {
        l.kind = kI8;
        l.vec = 8;
        l.fold_last = d_in == 256 ? 1 : 0;
        l.k_eff = static_cast<int>(d_in) - l.fold_last;
    } else {
        l.kind = d_in <= 2048 ? kF16 : kF32;    // |c| <= d_in: integers up to 2048 are exact in fp16
        l.vec = d_out > 256 ? 8 : 4;
        l.fold_last = 0;
        l.k_eff = static_cast<int>(d_in);
    }
    l.groups = groups_for(d_out, l.vec);
    l.embed_scale = kScaleSeparate;
    l.escape = 0;
    l.alt_kind = kI8;
    if (l.kind != kI8 && d_in <= kMaxEscapeBits) {
        // 257..1024 input bits: the stored value floor(K/2) - popcount has standard deviation
        // sqrt(K)/2 <= 16 for uncorrelated signs, so a whole row still fits 7 bits per value nearly
        // always (+-4 sigma at K = 1024).  Same 7-bit rows with the scale in the top bits as for
        // 129..256 bits; the alternate array keeps rows that do not fit as fp16 (|value| <= 512).
        // Beyond 1024 bits too many rows would take the slow path and fp16 rows are kept.
        // Narrow outputs are widened to 16 lanes (128 bytes, one cache line) to have room for
        // the scale bits: cheaper than a second line per neighbour for a separate scale.
        l.kind = kI8;
        l.vec = 8;
        l.escape = 1;
        l.alt_kind = kF16;
        if (d_out <= 60) {
            // up to 60 columns: a 64-byte row of 8 lanes whose last four lanes keep a byte of the
            // scale each behind their values (columns 60..63 do not exist), so the values have all
            // 8 bits (+-11 sigma at K = 512) and a gathered row is half the bytes of the widened one
            l.groups = 8;
            l.embed_scale = kScaleInLastBytes;
            return l;
        }
        l.groups = groups_for(d_out, 8) < 16 ? 16 : groups_for(d_out, 8);
        l.embed_scale = kScaleInTopBits;
        return l;
    }
    if (l.kind == kI8) {
        // The last four stored values belong to the last lane of the group and hold columns
        // (G-1) + G*(V-4 .. V-1); when those lie past d_out the bytes are free for the scale.
        // A row of at most 64 bytes is widened to make room: up to 128 bytes a row costs one
        // cache line either way, and the separate scale gather (a second line) disappears.
        // 40..60 columns in a 64-byte row: the tail is taken (column 39 sits there), but the last
        // value of each of the last four lanes is free and holds one byte of the scale each.
        if (l.groups == 8 && d_out > l.groups * (l.vec - 3) - 1 && d_out <= l.positions() - 4) {
            l.embed_scale = kScaleInLastBytes;
            return l;
        }
        if (d_out > l.groups * (l.vec - 3) - 1 && l.positions() <= 64) l.groups *= 2;
        l.embed_scale = d_out <= l.groups * (l.vec - 3) - 1 ? kScaleInTail : kScaleSeparate;
        // Up to 128 input bits the stored value needs 7 bits (K = 128: with the last bit folded
        // out, floor(127/2) - popcount lies in [-64, 63]), so the top bit of a byte is free.  Rows
        // of at least 32 lanes carry the 32 bits of the scale there, one per lane, rows of 16 lanes
        // two per lane (first and fifth byte).
        if (l.embed_scale == kScaleSeparate && d_in <= 128 && l.groups >= 16) {
            if (d_in == 128) {
                l.fold_last = 1;
                l.k_eff = 127;
            }
            l.embed_scale = kScaleInTopBits;
        } else if (l.embed_scale == kScaleSeparate && l.groups >= 16) {
            // 129..256 input bits: a product needs 8 bits in the worst case, but a row of them
            // almost never does (the stored value has standard deviation sqrt(K)/2 <= 8 for
            // uncorrelated signs; 7 bits hold +-8 sigma).  Rows are written in the 7-bit form
            // when every value fits; a row that does not fit is marked by a NaN scale and kept in
            // one-byte form in an alternate array.  Exact either way.
            l.embed_scale = kScaleInTopBits;
            l.escape = 1;
        }
    }
    return l;
}

template <bool kSelfTerm>
static int launch_fused_spmm_t(const FusedSpmmArgs &a, hipStream_t stream)
{
    const RowLayout &l = a.layout;
    EpilogueFusedT<kSelfTerm> epi{};
    epi.dst_mul = a.dst_mul;
    epi.alpha = a.alpha;
    epi.d_out = static_cast<int>(a.d_out);
    epi.mul = l.mul();
    epi.bias = l.bias();
    epi.last_bit_word = l.fold_last ? a.w_bits + (a.d_in - 1) / 64 : nullptr;
    epi.w_ld_words = a.w_ld_words;
    epi.last_bit_shift = static_cast<int>((a.d_in - 1) % 64);
    epi.logits = a.logits;
    epi.ld_logits = a.ld_logits;
    epi.next_shift = a.next_shift;
    epi.next_mul = a.next_mul;
    epi.next_bits = a.next_bits;
    epi.next_ld_words = a.next_ld_words;
    epi.next_scale = a.next_scale;
    epi.next_row_mul = a.next_row_mul;
    epi.next_fold_last_sign = a.next_fold_last_sign;
    epi.self_rows = static_cast<const char *>(a.self_rows);
    epi.alt_self_rows = static_cast<const char *>(a.alt_self_rows);
    epi.self_alpha = a.self_alpha;
    epi.self_last_bit_word = (l.fold_last && a.self_w_bits != nullptr) ? a.self_w_bits + (a.d_in - 1) / 64 : nullptr;
    const int valid = l.positions();
    const int64_t rb = l.row_bytes();
#define BIGCN_FUSED(TT, VV)                                                                             \
    return launch_spmm_groups<TT, VV, kWeightGather>(l.groups, a.plan, a.row_ptr, a.col_idx, a.src_scale, \
                                                     a.c_rows, rb, valid, epi, stream, nullptr, nullptr, 0, \
                                                     a.clear_flag)
#define BIGCN_FUSED_EMBEDDED(TT, VV)                                                                    \
    return launch_spmm_groups<TT, VV, kWeightEmbedded>(l.groups, a.plan, a.row_ptr, a.col_idx, nullptr, \
                                                       a.c_rows, rb, valid, epi, stream, nullptr, nullptr, 0, \
                                                       a.clear_flag)
    if (l.kind == kI8 && l.embed_scale == kScaleInTopBits && l.escape) {
        if (l.groups < 16) return BIGCN_EINVAL;
        if (kSelfTerm && a.alt_self_rows == nullptr) return BIGCN_ENULL;
        if (l.alt_kind != kI8 && l.alt_kind != kF16) return BIGCN_EINVAL;
        if (a.escape_flag != nullptr) {
            // no row escaped: the plain top-bits kernel runs and the next launch returns at once
            const int rc = launch_spmm_groups<int8_t, 8, kWeightTopBits>(l.groups, a.plan, a.row_ptr, a.col_idx, nullptr,
                                                                         a.c_rows, rb, valid, epi, stream, nullptr,
                                                                         a.escape_flag, 0, a.clear_flag);
            if (rc != BIGCN_OK) return rc;
        }
        if (l.alt_kind == kF16)
            return launch_spmm_groups<int8_t, 8, kWeightTopBitsEscapeF16>(l.groups, a.plan, a.row_ptr, a.col_idx,
                                                                          a.src_scale, a.c_rows, rb, valid, epi,
                                                                          stream, a.alt_rows, a.escape_flag, 1,
                                                                          a.clear_flag);
        return launch_spmm_groups<int8_t, 8, kWeightTopBitsEscape>(l.groups, a.plan, a.row_ptr, a.col_idx,
                                                                   a.src_scale, a.c_rows, rb, valid, epi, stream,
                                                                   a.alt_rows, a.escape_flag, 1, a.clear_flag);
    }
    if (l.kind == kI8 && l.embed_scale == kScaleInTopBits) {
        if (l.groups < 16) return BIGCN_EINVAL;
        return launch_spmm_groups<int8_t, 8, kWeightTopBits>(l.groups, a.plan, a.row_ptr, a.col_idx, nullptr,
                                                             a.c_rows, rb, valid, epi, stream, nullptr, nullptr, 0,
                                                             a.clear_flag);
    }
    if (l.kind == kI8 && l.embed_scale == kScaleInTail) {
        BIGCN_FUSED_EMBEDDED(int8_t, 8);
    }
    if (l.kind == kI8 && l.embed_scale == kScaleInLastBytes && l.escape) {
        // 8-bit products of 257..1024 input bits: the plain kernel when no row escaped, else the one
        // with the per-row test (same gate as for the top-bits rows above)
        if (l.groups != 8 || l.vec != 8 || l.alt_kind != kF16) return BIGCN_EINVAL;
        if (kSelfTerm && a.alt_self_rows == nullptr) return BIGCN_ENULL;
        if (a.escape_flag != nullptr) {
            const int rc = launch_spmm_one<int8_t, 8, 8, kWeightLastBytes>(a.plan, a.row_ptr, a.col_idx, nullptr, a.c_rows, rb,
                                                                           valid, epi, stream, nullptr, a.escape_flag, 0,
                                                                           a.clear_flag);
            if (rc != BIGCN_OK) return rc;
        }
        return launch_spmm_one<int8_t, 8, 8, kWeightLastBytesEscapeF16>(a.plan, a.row_ptr, a.col_idx, a.src_scale, a.c_rows, rb,
                                                                        valid, epi, stream, a.alt_rows, a.escape_flag, 1,
                                                                        a.clear_flag);
    }
    if (l.kind == kI8 && l.embed_scale == kScaleInLastBytes) {
        if (l.groups != 8 || l.vec != 8) return BIGCN_EINVAL;
        return launch_spmm_one<int8_t, 8, 8, kWeightLastBytes>(a.plan, a.row_ptr, a.col_idx, nullptr, a.c_rows, rb, valid,
                                                             epi, stream, nullptr, nullptr, 0, a.clear_flag);
    }
    if (l.kind == kI8) {
        BIGCN_FUSED(int8_t, 8);
    }
    if (l.kind == kF16) {
        if (l.vec == 8) BIGCN_FUSED(__half, 8);
        BIGCN_FUSED(__half, 4);
    }
    if (l.vec == 8) BIGCN_FUSED(float, 8);
    BIGCN_FUSED(float, 4);
#undef BIGCN_FUSED
#undef BIGCN_FUSED_EMBEDDED
}

int launch_fused_spmm(const FusedSpmmArgs &a, hipStream_t stream)
{
    if (a.self_rows != nullptr) return launch_fused_spmm_t<true>(a, stream);
    return launch_fused_spmm_t<false>(a, stream);
}

}  // namespace bigcn

using namespace bigcn;

extern "C" int bigcn_spmm(const bigcn_plan *plan, const int64_t *row_ptr, const int32_t *col_idx,
                          const float *vals, int64_t n, const float *z, int64_t d, int64_t ld_z,
                          float *out, int64_t ld_out, void *stream)
{
    if (plan == nullptr || row_ptr == nullptr || col_idx == nullptr || z == nullptr || out == nullptr)
        return BIGCN_ENULL;
    if (n != plan->n || d <= 0 || ld_z < d || ld_out < d) return BIGCN_EINVAL;
    if (n == 0) return BIGCN_OK;
    hipStream_t s = as_stream(stream);
    // 16-byte loads need aligned rows of a multiple of four columns; otherwise one float per lane
    const bool vec4 = (d % 4 == 0) && (ld_z % 4 == 0) && (reinterpret_cast<uintptr_t>(z) % 16 == 0);
    const bool vec_store = (ld_out % 4 == 0) && (reinterpret_cast<uintptr_t>(out) % 16 == 0);
    const int64_t pass_cols = vec4 ? 256 : 64;
    for (int64_t c0 = 0; c0 < d; c0 += pass_cols) {
        const int64_t dc = d - c0 < pass_cols ? d - c0 : pass_cols;
        EpiloguePlain epi{out + c0, ld_out, static_cast<int>(dc), vec_store ? 1 : 0};
        const void *rows = z + c0;
        int rc;
        if (vec4) {
            const int g = groups_for(dc, 4);
            rc = vals != nullptr
                     ? launch_spmm_groups<float, 4, kWeightVals>(g, plan, row_ptr, col_idx, vals, rows, ld_z * 4,
                                                                 static_cast<int>(dc), epi, s)
                     : launch_spmm_groups<float, 4, kWeightOne>(g, plan, row_ptr, col_idx, nullptr, rows, ld_z * 4,
                                                                static_cast<int>(dc), epi, s);
        } else {
            const int g = groups_for(dc, 1);
            rc = vals != nullptr
                     ? launch_spmm_groups<float, 1, kWeightVals>(g, plan, row_ptr, col_idx, vals, rows, ld_z * 4,
                                                                 static_cast<int>(dc), epi, s)
                     : launch_spmm_groups<float, 1, kWeightOne>(g, plan, row_ptr, col_idx, nullptr, rows, ld_z * 4,
                                                                static_cast<int>(dc), epi, s);
        }
        if (rc != BIGCN_OK) return rc;
    }
    return BIGCN_OK;
}
