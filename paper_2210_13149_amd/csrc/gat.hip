// One Bi-GAT layer (Sec. 4.4.1): z_j = W~ (*) h~_j by the binarise+pack and bit-GEMM kernels
// (Sec. 4.2), then, per head,
//   e_ij = LeakyReLU(a_src . z_i + a_dst . z_j),  a_ij = softmax_{j in N_i} e_ij,
//   out_i = sum_{j in N_i} a_ij z_j.
// The attention vectors are not binarised.
//
// Compact path (every head a multiple of 8 columns wide): the bit-GEMM leaves the integer
// products of a node as one compact row in column order (one byte per product up to 256 input
// bits, the last of 256 bits carried on the sign of the node's scale; fp16 up to 2048, fp32
// beyond); the row scale beta_j and the scores t_j = a_dst . z_j sit together in a small
// per-node record (256-column one-byte rows whose values all fit 7 bits carry that record in
// their spare top bits instead, so that a neighbour costs the two cache lines of its row and no
// other).  The aggregation makes ONE pass over the neighbours of
// a node: per batch of 64 neighbours the running maximum of e_ij is raised and the accumulators
// rescaled (once per batch and head), so no separate maximum pass gathers the records twice.
// Long rows are shared by the four wavefronts of a workgroup and merged through LDS.  Sums are
// taken in a fixed order (run-to-run identical).
//
// Plain path (any head width): z kept in fp32 rows, a maximum pass and an accumulation pass.
#include "bigcn_internal.h"

namespace bigcn {

constexpr int kGatMaxV = 8;              // columns per lane: d_out <= 512

// s[i][h], t[i][h]: one wavefront per node, lane l takes columns l, l + 64, ...
template <int H>
__global__ __launch_bounds__(kBlock) void gat_scores_plain_kernel(const float *__restrict__ z, int64_t n, int d_out, int d_head,
                                                            const float *__restrict__ a_src,
                                                            const float *__restrict__ a_dst, float *__restrict__ s,
                                                            float *__restrict__ t)
{
    const int lane = lane_id();
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * kWavesPerBlock + wave_in_block();
    const int64_t n_waves = static_cast<int64_t>(gridDim.x) * kWavesPerBlock;
    for (int64_t i = wave; i < n; i += n_waves) {
        float ps[H], pt[H];
#pragma unroll
        for (int h = 0; h < H; ++h) { ps[h] = 0.0f; pt[h] = 0.0f; }
        for (int c = lane; c < d_out; c += kWave) {
            const float v = z[i * d_out + c];
            const int hc = c / d_head;
            const float as = a_src[c], ad = a_dst[c];          // (heads, d_head) row-major = column order
#pragma unroll
            for (int h = 0; h < H; ++h) {
                ps[h] += hc == h ? as * v : 0.0f;
                pt[h] += hc == h ? ad * v : 0.0f;
            }
        }
#pragma unroll
        for (int h = 0; h < H; ++h) {
            const float ss = wave_sum(ps[h]), tt = wave_sum(pt[h]);
            if (lane == 0) {
                s[i * H + h] = ss;
                t[i * H + h] = tt;
            }
        }
    }
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
    return v;
}

__device__ __forceinline__ float leaky(float e, float slope) { return e > 0.0f ? e : slope * e; }

// One wavefront per node, nodes in plan order (longest rows first).
template <int H>
__global__ __launch_bounds__(kBlock) void gat_aggregate_plain_kernel(const int32_t *__restrict__ row_order, int64_t n,
                                                               const int64_t *__restrict__ row_ptr,
                                                               const int32_t *__restrict__ col_idx,
                                                               const float *__restrict__ z, int d_out, int d_head,
                                                               const float *__restrict__ s, const float *__restrict__ t,
                                                               float slope, float *__restrict__ out, int64_t ld_out)
{
    constexpr int U = 4;
    const int lane = lane_id();
    const int64_t entry = static_cast<int64_t>(blockIdx.x) * kWavesPerBlock + wave_in_block();
    if (entry >= n) return;                                    // wave-uniform
    const int64_t row = row_order[entry];
    const int64_t p0 = row_ptr[row], p1 = row_ptr[row + 1];

    int head_of[kGatMaxV];
    bool col_in[kGatMaxV];
#pragma unroll
    for (int v = 0; v < kGatMaxV; ++v) {
        const int c = lane + kWave * v;
        col_in[v] = c < d_out;
        head_of[v] = col_in[v] ? c / d_head : 0;
    }
    float si[H];
#pragma unroll
    for (int h = 0; h < H; ++h) si[h] = s[row * H + h];

    // pass 1: row maximum of e_ij per head
    float m[H];
#pragma unroll
    for (int h = 0; h < H; ++h) m[h] = -INFINITY;
    for (int64_t p = p0 + lane; p < p1; p += kWave) {
        const int64_t k = col_idx[p];
#pragma unroll
        for (int h = 0; h < H; ++h) m[h] = fmaxf(m[h], leaky(si[h] + t[k * H + h], slope));
    }
#pragma unroll
    for (int h = 0; h < H; ++h) m[h] = wave_max(m[h]);

    // pass 2: weights exp(e_ij - max), their sum, and the weighted rows
    float acc[kGatMaxV];
#pragma unroll
    for (int v = 0; v < kGatMaxV; ++v) acc[v] = 0.0f;
    float lsum[H];
#pragma unroll
    for (int h = 0; h < H; ++h) lsum[h] = 0.0f;

    for (int64_t pb = p0; pb < p1; pb += kWave) {
        const int cnt = static_cast<int>(p1 - pb < kWave ? p1 - pb : kWave);
        int k = 0;
        float pe[H];
#pragma unroll
        for (int h = 0; h < H; ++h) pe[h] = 0.0f;
        if (lane < cnt) {
            k = col_idx[pb + lane];
#pragma unroll
            for (int h = 0; h < H; ++h) {
                pe[h] = expf(leaky(si[h] + t[static_cast<int64_t>(k) * H + h], slope) - m[h]);
                lsum[h] += pe[h];
            }
        }
        for (int u0 = 0; u0 < cnt; u0 += U) {
            float zv[U][kGatMaxV];
            float w[U][H];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int src = u0 + u < cnt ? u0 + u : cnt - 1;          // tail repeats a valid lane with weight 0
                const int kk = __builtin_amdgcn_readlane(k, src);
#pragma unroll
                for (int h = 0; h < H; ++h) {
                    const float ph = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, pe[h]), src));
                    w[u][h] = u0 + u < cnt ? ph : 0.0f;
                }
                const float *zr = z + static_cast<int64_t>(kk) * d_out + lane;
#pragma unroll
                for (int v = 0; v < kGatMaxV; ++v) zv[u][v] = col_in[v] ? zr[kWave * v] : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int v = 0; v < kGatMaxV; ++v) {
                    float wv = w[u][0];
#pragma unroll
                    for (int h = 1; h < H; ++h) wv = head_of[v] == h ? w[u][h] : wv;
                    acc[v] = fmaf(wv, zv[u][v], acc[v]);
                }
        }
    }
    float inv[H];
#pragma unroll
    for (int h = 0; h < H; ++h) {
        const float l = wave_sum(lsum[h]);
        inv[h] = l > 0.0f ? 1.0f / l : 0.0f;
    }
#pragma unroll
    for (int v = 0; v < kGatMaxV; ++v) {
        if (!col_in[v]) continue;
        float iv = inv[0];
#pragma unroll
        for (int h = 1; h < H; ++h) iv = head_of[v] == h ? inv[h] : iv;
        out[row * ld_out + lane + kWave * v] = acc[v] * iv;
    }
}


// ---- compact path --------------------------------------------------------------------------
// Eight stored values of a row -> fp32, multiplied and accumulated.
template <typename T>
struct GatSegment;
template <>
struct GatSegment<int8_t> {
    uint2 raw;
    __device__ __forceinline__ void load(const char *p) { raw = *reinterpret_cast<const uint2 *>(p); }
    __device__ __forceinline__ float get(int v) const
    {
        const uint32_t word = v < 4 ? raw.x : raw.y;
        return static_cast<float>(static_cast<int>(word << (24 - 8 * (v & 3))) >> 24);
    }
};
template <>
struct GatSegment<__half> {
    uint4 raw;
    __device__ __forceinline__ void load(const char *p) { raw = *reinterpret_cast<const uint4 *>(p); }
    __device__ __forceinline__ float get(int v) const
    {
        const __half2 pair = reinterpret_cast<const __half2 *>(&raw)[v >> 1];
        return (v & 1) ? __high2float(pair) : __low2float(pair);
    }
};
template <>
struct GatSegment<float> {
    float4 lo, hi;
    __device__ __forceinline__ void load(const char *p)
    {
        lo = *reinterpret_cast<const float4 *>(p);
        hi = *reinterpret_cast<const float4 *>(p + 16);
    }
    __device__ __forceinline__ float get(int v) const
    {
        const float4 q = v < 4 ? lo : hi;
        return (v & 3) == 0 ? q.x : ((v & 3) == 1 ? q.y : ((v & 3) == 2 ? q.z : q.w));
    }
};

// Floats per record {beta, t[0..H-1]}, padded to whole 16-byte vectors: a neighbour's record is
// read with aligned vector loads that never straddle a cache line (one load for up to three
// heads, where three scalar loads asked the texture path for the same line three times).
template <int H>
constexpr int gat_record_floats() { return (H + 1 + 3) / 4 * 4; }

// select x[h] for a head index known only at run time (H is small)
template <int H>
__device__ __forceinline__ float pick(const float (&x)[H], int h)
{
    float r = x[0];
#pragma unroll
    for (int q = 1; q < H; ++q) r = h == q ? x[q] : r;
    return r;
}

// Shapes whose kernels can carry the record inside the row (the launcher decides per call).
template <typename T, int G, int H>
constexpr bool gat_embeds() { return sizeof(T) == 1 && G == 32 && H <= 2; }

constexpr float kLog2e = 1.44269504088896340736f;

// Scores of the compact path.  Stored value q of column c stands for the product
// mul * q + bias (mul = 2, bias = K mod 2 for one-byte rows; 1, 0 otherwise), so
//   s_i[h] = beta_i * (mul * sum_c a_src[c] alpha[c] q_ic + bias * sum_c a_src[c] alpha[c])
// over the columns c of head h; t_i[h] likewise with a_dst.  A wavefront takes 64 / G nodes at a
// time, lane g of a node's G lanes holding columns 8 g .. 8 g + 7 (all in one head).  When a head
// spans a power-of-two number of lanes its sums are a butterfly inside that lane group;
// otherwise one masked sum over the wavefront per head (one node at a time).
// record[i] = {beta_i, t_i[0..H-1]} at a stride of gat_record_floats<H>() floats.
// Record inside the row (one-byte rows of 256 columns, one or two heads, every stored value
// within 7 bits: always so up to 127 input bits, else checked by gat_fit_kernel): the record goes
// into the row itself instead.  Lane g of the
// row's 32 lanes gives bit g of beta_i to the top bit of its byte 3, bit g of t_i[0] log2(e) to
// the top bit of byte 7 and bit g of t_i[1] log2(e) to the top bit of byte 2 (see
// gat_aggregate_embedded_kernel).
template <typename T, int G, int H>
__global__ __launch_bounds__(kBlock) void gat_scores_kernel(char *__restrict__ rows, uint32_t row_bytes, int64_t n,
                                                            int d_out, int d_head, float mul, float bias,
                                                            const float *__restrict__ beta,
                                                            const float *__restrict__ alpha,
                                                            const float *__restrict__ a_src,
                                                            const float *__restrict__ a_dst, float *__restrict__ s,
                                                            float *__restrict__ record, int embed_mode,
                                                            const int *__restrict__ misfit,
                                                            const float *__restrict__ last_sign)
{
    constexpr int V = 8;
    // embed_mode 0: records beside the rows; 1: inside the rows; 2: inside unless *misfit is set
    const int embed = embed_mode == 1 || (embed_mode == 2 && *misfit == 0) ? 1 : 0;
    const int lane = lane_id();
    const int g = lane & (G - 1);
    const int lanes_per_head = d_head / V;
    const bool butterfly = (lanes_per_head & (lanes_per_head - 1)) == 0;         // wave-uniform
    const int nodes_per_step = butterfly ? kWave / G : 1;
    const int slot = lane / G;
    const int my_head = g / lanes_per_head;                    // >= H: lanes past the last head
    const bool live = my_head < H && slot < nodes_per_step;
    // last_sign (layers of 256 input bits kept in one-byte rows): the stored values cover the first
    // 255 bits; the last one contributes f_i b_c to the product, f_i = the sign of beta[i] and
    // b_c = last_sign[c], so s_i[h] gains beta_i * sum_c a_src[c] alpha[c] b_c (signed beta_i) and
    // the other terms take |beta_i|.
    float ca[V], cd[V];
    float sum_a = 0.0f, sum_d = 0.0f, last_a = 0.0f, last_d = 0.0f;
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const int c = g * V + v;
        const bool in = live && c < d_out;
        const float al = in ? alpha[c] : 0.0f;
        const float lb = (in && last_sign != nullptr) ? last_sign[c] : 0.0f;
        ca[v] = in ? a_src[c] * al : 0.0f;
        cd[v] = in ? a_dst[c] * al : 0.0f;
        sum_a += ca[v];
        sum_d += cd[v];
        last_a = fmaf(ca[v], lb, last_a);
        last_d = fmaf(cd[v], lb, last_d);
    }
    // per-head constants bias * sum_c a[c] alpha[c] and sum_c a[c] alpha[c] b_c: this lane's own
    // head (butterfly) or all heads
    float const_s[H], const_t[H], fold_s[H], fold_t[H];
    if (butterfly) {
        for (int off = 1; off < lanes_per_head; off <<= 1) {
            sum_a += __shfl_xor(sum_a, off, kWave);
            sum_d += __shfl_xor(sum_d, off, kWave);
            last_a += __shfl_xor(last_a, off, kWave);
            last_d += __shfl_xor(last_d, off, kWave);
        }
#pragma unroll
        for (int h = 0; h < H; ++h) {
            const_s[h] = bias * sum_a;
            const_t[h] = bias * sum_d;
            fold_s[h] = last_a;
            fold_t[h] = last_d;
        }
    } else {
#pragma unroll
        for (int h = 0; h < H; ++h) {
            const_s[h] = bias * wave_sum(live && my_head == h ? sum_a : 0.0f);
            const_t[h] = bias * wave_sum(live && my_head == h ? sum_d : 0.0f);
            fold_s[h] = wave_sum(live && my_head == h ? last_a : 0.0f);
            fold_t[h] = wave_sum(live && my_head == h ? last_d : 0.0f);
        }
    }
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * kWavesPerBlock + wave_in_block();
    const int64_t n_waves = static_cast<int64_t>(gridDim.x) * kWavesPerBlock;
    // kAhead steps' rows are requested before the first is used (a wavefront's step is 512 bytes
    // or less; with one in flight the launch reads at a third of the rate)
    constexpr int kAhead = 4;
    const int64_t step_nodes = n_waves * nodes_per_step;
    for (int64_t i0 = wave * nodes_per_step; i0 < n; i0 += step_nodes * kAhead) {
        GatSegment<T> segs[kAhead];
        float bs[kAhead];
#pragma unroll
        for (int q = 0; q < kAhead; ++q) {
            const int64_t i = i0 + q * step_nodes + (butterfly ? slot : 0);
            bs[q] = 0.0f;
            if (live && i < n) {
                segs[q].load(rows + static_cast<uint64_t>(i) * row_bytes + g * V * sizeof(T));
                bs[q] = beta[i];
            }
        }
#pragma unroll
        for (int q = 0; q < kAhead; ++q) {
            if (i0 + q * step_nodes >= n) break;                    // wave-uniform
            const int64_t i = i0 + q * step_nodes + (butterfly ? slot : 0);
            const bool mine = live && i < n;
            GatSegment<T> &seg = segs[q];
            const float b = bs[q];
            float ps = 0.0f, pt = 0.0f;
            if (mine) {
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    const float x = seg.get(v);
                    ps = fmaf(ca[v], x, ps);
                    pt = fmaf(cd[v], x, pt);
                }
            }
            if (butterfly) {
                for (int off = 1; off < lanes_per_head; off <<= 1) {
                    ps += __shfl_xor(ps, off, kWave);
                    pt += __shfl_xor(pt, off, kWave);
                }
                const float ab = fabsf(b);
                const float t_mine = fmaf(b, fold_t[0], ab * fmaf(mul, pt, const_t[0]));
                if (mine && g == my_head * lanes_per_head) {        // first lane of the head's group
                    s[i * H + my_head] = fmaf(b, fold_s[0], ab * fmaf(mul, ps, const_s[0]));
                    if (!embed) {
                        record[i * gat_record_floats<H>() + 1 + my_head] = t_mine;
                        if (g == 0) record[i * gat_record_floats<H>()] = b;
                    }
                }
                if constexpr (gat_embeds<T, G, H>()) {
                    if (embed) {                                    // wave-uniform; every lane is live here
                        const float t2 = t_mine * kLog2e;
                        const float other = H == 2 ? __shfl_xor(t2, 16, kWave) : t2;
                        const uint32_t t0 = __builtin_bit_cast(uint32_t, my_head == 0 ? t2 : other);
                        const uint32_t t1 = __builtin_bit_cast(uint32_t, my_head == 0 ? other : t2);
                        const uint32_t bb = __builtin_bit_cast(uint32_t, b);
                        if (mine) {
                            uint2 raw = seg.raw;
                            raw.x = (raw.x & 0x7fffffffu) | (((bb >> g) & 1u) << 31);
                            raw.y = (raw.y & 0x7fffffffu) | (((t0 >> g) & 1u) << 31);
                            if (H == 2) raw.x = (raw.x & 0xff7fffffu) | (((t1 >> g) & 1u) << 23);
                            *reinterpret_cast<uint2 *>(rows + static_cast<uint64_t>(i) * row_bytes + g * V) = raw;
                        }
                    }
                }
            } else {
                const float b0 = __shfl(b, 0, kWave);
                const float ab0 = fabsf(b0);
#pragma unroll
                for (int h = 0; h < H; ++h) {
                    const float ss = wave_sum(mine && my_head == h ? ps : 0.0f);
                    const float tt = wave_sum(mine && my_head == h ? pt : 0.0f);
                    if (lane == 0) {
                        s[i * H + h] = fmaf(b0, fold_s[h], ab0 * fmaf(mul, ss, const_s[h]));
                        record[i * gat_record_floats<H>() + 1 + h] = fmaf(b0, fold_t[h], ab0 * fmaf(mul, tt, const_t[h]));
                    }
                }
                if (lane == 0) record[i * gat_record_floats<H>()] = b0;
            }
        }
    }
}

// Softmax state of one node and head set while its neighbours stream by.
template <int H>
struct GatState {
    float m[H];       // running maximum of e_ij (wave-uniform)
    float l[H];       // sum of exp(e_ij - m), per-lane partial until reduced
    float sw[H];      // sum of exp(e_ij - m) |beta_j|, per-lane partial until reduced
    float sf[H];      // sum of exp(e_ij - m) beta_j with its sign (layers with a folded last bit)
    float acc[8];     // sum of exp(e_ij - m) |beta_j| q_j over this lane's columns and slot
};

// Neighbours p0..p1-1 of node `row`.  wbuf: this wavefront's H x 64 floats of LDS.
// kFold: the stored scale carries the sign of the neighbour's last input bit (see gat_scores_kernel).
template <typename T, int G, int H, bool kFold>
__device__ __forceinline__ void gat_accumulate(const int32_t *__restrict__ col_idx, const char *__restrict__ lane_base,
                                               uint32_t row_bytes, const float *__restrict__ record,
                                               const float (&si)[H], float slope, int my_head, int64_t p0,
                                               int64_t p1, int lane, float *wbuf, GatState<H> &st)
{
    constexpr int V = 8, S = kWave / G, U = 4;
    const int slot = lane / G;
#pragma unroll
    for (int h = 0; h < H; ++h) { st.m[h] = -INFINITY; st.l[h] = 0.0f; st.sw[h] = 0.0f; st.sf[h] = 0.0f; }
#pragma unroll
    for (int v = 0; v < V; ++v) st.acc[v] = 0.0f;

    for (int64_t pb = p0; pb < p1; pb += kWave) {
        const int cnt = static_cast<int>(p1 - pb < kWave ? p1 - pb : kWave);     // wave-uniform, >= 1
        int k = 0;
        float bk = 0.0f;
        float e[H];
#pragma unroll
        for (int h = 0; h < H; ++h) e[h] = -INFINITY;
        if (lane < cnt) {
            k = col_idx[pb + lane];
            constexpr int kVecs = gat_record_floats<H>() / 4;
            const float4 *src = reinterpret_cast<const float4 *>(record) + static_cast<int64_t>(k) * kVecs;
            float rec[4 * kVecs];
#pragma unroll
            for (int q = 0; q < kVecs; ++q) {
                const float4 part = src[q];
                rec[4 * q] = part.x;
                rec[4 * q + 1] = part.y;
                rec[4 * q + 2] = part.z;
                rec[4 * q + 3] = part.w;
            }
            bk = rec[0];
#pragma unroll
            for (int h = 0; h < H; ++h) e[h] = leaky(si[h] + rec[1 + h], slope);
        }
        float rescale[H], w[H];
#pragma unroll
        for (int h = 0; h < H; ++h) {
            const float mn = fmaxf(st.m[h], wave_max(e[h]));
            rescale[h] = expf(st.m[h] - mn);                 // 0 on the first batch (m = -inf)
            st.m[h] = mn;
            const float pe = lane < cnt ? expf(e[h] - mn) : 0.0f;
            w[h] = pe * (kFold ? fabsf(bk) : bk);
            st.l[h] = fmaf(st.l[h], rescale[h], pe);
            st.sw[h] = fmaf(st.sw[h], rescale[h], w[h]);
            if constexpr (kFold) st.sf[h] = fmaf(st.sf[h], rescale[h], pe * bk);
        }
        const float my_rescale = pick<H>(rescale, my_head);
#pragma unroll
        for (int v = 0; v < V; ++v) st.acc[v] *= my_rescale;
        if constexpr (H > 1) {
            // the weights of this batch, [head][neighbour], for the lanes that load the rows
#pragma unroll
            for (int h = 0; h < H; ++h) wbuf[h * kWave + lane] = w[h];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
        for (int t = 0; t < cnt; t += S * U) {
            GatSegment<T> seg[U];
            float wgt[U];
            bool present[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int src = t + u * S + slot;
                present[u] = src < cnt;
                const int from = present[u] ? src : 0;
                const int kk = __shfl(k, from, kWave);
                if constexpr (H > 1) wgt[u] = wbuf[my_head * kWave + from];
                else wgt[u] = __shfl(w[0], from, kWave);
                if (present[u]) seg[u].load(lane_base + static_cast<uint64_t>(static_cast<uint32_t>(kk)) * row_bytes);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (present[u]) {
#pragma unroll
                    for (int v = 0; v < V; ++v) st.acc[v] = fmaf(wgt[u], seg[u].get(v), st.acc[v]);
                }
            }
        }
        if constexpr (H > 1) {
            // the next batch overwrites wbuf: every lane has read its weights
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
    }
    // totals over the lanes (l, sw) and over the slots (acc)
#pragma unroll
    for (int h = 0; h < H; ++h) {
        st.l[h] = wave_sum(st.l[h]);
        st.sw[h] = wave_sum(st.sw[h]);
        if constexpr (kFold) st.sf[h] = wave_sum(st.sf[h]);
    }
#pragma unroll
    for (int off = G; off < kWave; off <<= 1)
#pragma unroll
        for (int v = 0; v < V; ++v) st.acc[v] += __shfl_xor(st.acc[v], off, kWave);
}

// out_i[c] = alpha[c] (mul * acc[c] + bias * sw[h] + last_sign[c] * sf[h]) / l[h] (the last term
// with kFold only); an empty row gives zeros.
template <int G, int H, bool kFold>
__device__ __forceinline__ void gat_finish(const GatState<H> &st, int64_t row, int lane, int my_head, int d_out,
                                           float mul, float bias, const float *__restrict__ alpha,
                                           const float *__restrict__ last_sign,
                                           float *__restrict__ out, int64_t ld_out, int vector_store)
{
    constexpr int V = 8;
    if (lane >= G) return;
    const float l = pick<H>(st.l, my_head);
    const float inv = l > 0.0f ? 1.0f / l : 0.0f;
    const float base = bias * pick<H>(st.sw, my_head);
    const float folded = kFold ? pick<H>(st.sf, my_head) : 0.0f;
    float r[V];
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const int c = lane * V + v;
        float sum = fmaf(mul, st.acc[v], base);
        if constexpr (kFold) sum = c < d_out ? fmaf(last_sign[c], folded, sum) : sum;
        r[v] = c < d_out ? alpha[c] * sum * inv : 0.0f;
    }
    float *dst = out + row * ld_out + lane * V;
    if (vector_store && lane * V + V <= d_out) {
        reinterpret_cast<float4 *>(dst)[0] = make_float4(r[0], r[1], r[2], r[3]);
        reinterpret_cast<float4 *>(dst)[1] = make_float4(r[4], r[5], r[6], r[7]);
    } else {
#pragma unroll
        for (int v = 0; v < V; ++v)
            if (lane * V + v < d_out) dst[v] = r[v];
    }
}

// Nodes in plan order: workgroup b < n_block_rows owns one long row (four wavefronts, contiguous
// quarters of the neighbour list); every later workgroup owns four nodes, one per wavefront.
// One-byte rows with one or two heads fit 64 registers: ask for 8 wavefronts per SIMD (the
// gather hides its latency with resident wavefronts; measured 6 % faster than 7).
template <typename T, int H>
constexpr int gat_min_waves()
{
    return (sizeof(T) == 1 && H <= 2) ? 8 : 1;
}

template <typename T, int G, int H, bool kFold>
__global__ __launch_bounds__(kBlock, (gat_min_waves<T, H>())) void gat_aggregate_kernel(
    const bigcn_plan_entry *__restrict__ entries, int64_t n, int64_t n_block_rows,
    const int32_t *__restrict__ col_idx, const char *__restrict__ rows, uint32_t row_bytes,
    const float *__restrict__ s, const float *__restrict__ record, const float *__restrict__ alpha, int d_out,
    int d_head, float mul, float bias, float slope, const float *__restrict__ last_sign,
    const int *__restrict__ gate, float *__restrict__ out, int64_t ld_out, int vector_store)
{
    constexpr int V = 8;
    // gate (nullable): a device flag; while it is 0 the rows carry their records themselves and
    // gat_aggregate_embedded_kernel does the work: this launch returns at once
    if (gate != nullptr && *gate == 0) return;
    __shared__ float wbuf_all[kWavesPerBlock][H > 1 ? H * kWave : 1];
    __shared__ float merge[kWavesPerBlock - 1][V + (kFold ? 4 : 3) * H][kWave];
    const int lane = lane_id();
    const int wave = wave_in_block();
    const int g = lane & (G - 1);
    const int my_head = (g * V) / d_head < H ? (g * V) / d_head : H - 1;   // lanes past d_out: any valid head
    const char *lane_base = rows + static_cast<int64_t>(g) * V * sizeof(T);
    float *wbuf = wbuf_all[wave];
    GatState<H> st;
    float si[H];

    if (static_cast<int64_t>(blockIdx.x) < n_block_rows) {
        const bigcn_plan_entry e = entries[blockIdx.x];       // the row and its extent in one load
        const int64_t row = e.row;
        const int64_t p0 = e.first, p1 = e.first + e.count;
        int64_t chunk = (p1 - p0 + kWavesPerBlock - 1) / kWavesPerBlock;
        chunk = (chunk + kWave - 1) / kWave * kWave;
        int64_t q0 = p0 + wave * chunk, q1 = q0 + chunk;
        if (q0 > p1) q0 = p1;
        if (q1 > p1) q1 = p1;
#pragma unroll
        for (int h = 0; h < H; ++h) si[h] = s[row * H + h];
        gat_accumulate<T, G, H, kFold>(col_idx, lane_base, row_bytes, record, si, slope, my_head, q0, q1, lane, wbuf, st);
        if (wave > 0) {
#pragma unroll
            for (int v = 0; v < V; ++v) merge[wave - 1][v][lane] = st.acc[v];
#pragma unroll
            for (int h = 0; h < H; ++h) {
                merge[wave - 1][V + h][lane] = st.m[h];
                merge[wave - 1][V + H + h][lane] = st.l[h];
                merge[wave - 1][V + 2 * H + h][lane] = st.sw[h];
                if constexpr (kFold) merge[wave - 1][V + 3 * H + h][lane] = st.sf[h];
            }
        }
        __syncthreads();
        if (wave == 0) {
            // bring the four partial states to the common maximum and add them
            float top[H];
#pragma unroll
            for (int h = 0; h < H; ++h) {
                top[h] = st.m[h];
#pragma unroll
                for (int w = 0; w < kWavesPerBlock - 1; ++w) top[h] = fmaxf(top[h], merge[w][V + h][lane]);
            }
            float f0[H];
#pragma unroll
            for (int h = 0; h < H; ++h) {
                f0[h] = st.m[h] == -INFINITY ? 0.0f : expf(st.m[h] - top[h]);
                st.l[h] *= f0[h];
                st.sw[h] *= f0[h];
                if constexpr (kFold) st.sf[h] *= f0[h];
            }
            const float mine0 = pick<H>(f0, my_head);
#pragma unroll
            for (int v = 0; v < V; ++v) st.acc[v] *= mine0;
#pragma unroll
            for (int w = 0; w < kWavesPerBlock - 1; ++w) {
                float f[H];
#pragma unroll
                for (int h = 0; h < H; ++h) {
                    const float mw = merge[w][V + h][lane];
                    f[h] = mw == -INFINITY ? 0.0f : expf(mw - top[h]);
                    st.l[h] = fmaf(f[h], merge[w][V + H + h][lane], st.l[h]);
                    st.sw[h] = fmaf(f[h], merge[w][V + 2 * H + h][lane], st.sw[h]);
                    if constexpr (kFold) st.sf[h] = fmaf(f[h], merge[w][V + 3 * H + h][lane], st.sf[h]);
                }
                const float mine = pick<H>(f, my_head);
#pragma unroll
                for (int v = 0; v < V; ++v) st.acc[v] = fmaf(mine, merge[w][v][lane], st.acc[v]);
            }
            gat_finish<G, H, kFold>(st, row, lane, my_head, d_out, mul, bias, alpha, last_sign, out, ld_out, vector_store);
        }
        return;
    }
    const int64_t entry = n_block_rows + (static_cast<int64_t>(blockIdx.x) - n_block_rows) * kWavesPerBlock + wave;
    if (entry >= n) return;                                    // wave-uniform
    const bigcn_plan_entry e = entries[entry];
    const int64_t row = e.row;
#pragma unroll
    for (int h = 0; h < H; ++h) si[h] = s[row * H + h];
    gat_accumulate<T, G, H, kFold>(col_idx, lane_base, row_bytes, record, si, slope, my_head, e.first, e.first + e.count,
                            lane, wbuf, st);
    gat_finish<G, H, kFold>(st, row, lane, my_head, d_out, mul, bias, alpha, last_sign, out, ld_out, vector_store);
}

// ---- compact path, record inside the row ---------------------------------------------------
// One-byte rows of 256 columns whose values fit 7 bits (always so up to 127 input bits, tested by
// gat_fit_kernel beyond) have a spare top bit in every byte, and gat_scores_kernel stores beta_j
// and t_j there: a neighbour costs its two row lines and nothing else.  A load instruction fetches two neighbours (lanes 0..31 one,
// lanes 32..63 the other), and three ballots over the carrier bits give their record words as
// scalar values.  These are written into lanes 0..15, which form the scores, the running maximum
// (raised per eight neighbours, the rescaling skipped while no head's maximum moves) and the
// weights once per neighbour and head; the row lanes fetch the weight of their neighbour and head
// from there and accumulate the weighted values.  Scores are kept in base 2 (t_j and s_i times
// log2 e; LeakyReLU commutes with a positive factor), so a weight is one v_exp_f32.  The kernel
// is bound by its vector instructions, so the inner loop is written for their count.
//
// State of a node at the end of its row (and between the wavefronts that share a long row), per
// row lane:
struct GatLaneState {
    float m;          // maximum of e_ij log2(e) over the lane's head
    float ref;        // m, or 0 while m is -inf (so that exp2(x - ref) is never inf - inf)
    float l;          // sum of 2^(e_ij - m)
    float sw;         // sum of 2^(e_ij - m) |beta_j|
    float sf;         // sum of 2^(e_ij - m) beta_j with its sign (layers with a folded last bit, else unused)
    float acc[8];     // sum of 2^(e_ij - m) |beta_j| q_j over this lane's columns
};

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }

// values 0..7 of a lane's segment; bytes 2, 3 and 7 carry a foreign top bit
__device__ __forceinline__ float embedded_value(const uint2 raw, int v)
{
    const uint32_t word = v < 4 ? raw.x : raw.y;
    const int e = v & 3;
    if (v == 2 || v == 3 || v == 7) return static_cast<float>(static_cast<int>(word << (25 - 8 * e)) >> 25);
    return static_cast<float>(static_cast<int>(word << (24 - 8 * e)) >> 24);
}

constexpr int kGatEmbeddedLoads = 4;   // row loads in flight per wavefront (6 and 8 measured 2-3 % slower)

// Per-lane constants of the embedded kernels.
struct GatLaneMasks {
    uint32_t lane_offset;  // byte offset of this lane's segment in a row
    int half;              // lane / 32: which of a load's two neighbours this lane reads
    int position;          // lane mod 8: the neighbour of a group that this lane scores
    int head_lane;         // 4 x the first softmax lane of this row lane's head (a ds_bpermute address)
    int weight_lane;       // 4 x the softmax lane of this row lane's head and of the first load's neighbour
};

// U row loads: neighbour `from` + 2 u of the batch of `cnt` (from = t + lane / 32) for
// u = 0..U-1, whose column indices sit in the lanes of k.  A lane number past 63 wraps to some
// lane's k, which is then not loaded from; an absent neighbour reads as zeros.
template <int U>
__device__ __forceinline__ void gat_fetch_group(const char *__restrict__ rows, const GatLaneMasks &lm, int k, int from,
                                                int cnt, uint2 (&raw)[U])
{
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t kk = static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute((from + 2 * u) << 2, k));
        raw[u] = make_uint2(0u, 0u);
        if (from < cnt - 2 * u) raw[u] = *reinterpret_cast<const uint2 *>(rows + ((kk << 8) + lm.lane_offset));
    }
}

// Softmax state while the neighbours of a node stream by, kept once per head instead of once per
// lane: lane 8 h + j (h < H, j < 8) works on head h and on the j-th neighbour of each group of
// eight; m and ref are the same in the eight lanes of a head, l and sw are partial sums over j.
struct GatGroupState {
    float m;          // running maximum of e_ij log2(e)
    float ref;        // m, or 0 while m is -inf (so that exp2(x - ref) is never inf - inf)
    float l;          // sum of 2^(e_ij - m)
    float sw;         // sum of 2^(e_ij - m) |beta_j|
    float sf;         // sum of 2^(e_ij - m) beta_j with its sign (kFold)
};

template <int kCtrl>
__device__ __forceinline__ float dpp_move(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), kCtrl, 0xf, 0xf, true));
}

// maximum / sum over the eight lanes 8 q .. 8 q + 7, in all of them
// (the median of a, b and +inf is max(a, b) in one instruction: fmaxf adds one to quieten NaNs)
__device__ __forceinline__ float max_plain(float a, float b) { return __builtin_amdgcn_fmed3f(a, b, INFINITY); }
__device__ __forceinline__ float max_of_eight(float v)
{
    v = max_plain(v, dpp_move<0xb1>(v));       // quad_perm [1, 0, 3, 2]
    v = max_plain(v, dpp_move<0x4e>(v));       // quad_perm [2, 3, 0, 1]
    return max_plain(v, dpp_move<0x141>(v));   // row_half_mirror
}
__device__ __forceinline__ float sum_of_eight(float v)
{
    v += dpp_move<0xb1>(v);
    v += dpp_move<0x4e>(v);
    return v + dpp_move<0x141>(v);
}

// v[kLane] = value, a wave-uniform word.  The compiler's own v_writelane (not inline assembly):
// an SGPR written by a vector compare needs two wait states before a vector instruction reads
// it, which the compiler inserts only around instructions it can see.
__device__ int amdgcn_writelane(int value, int lane, int old) __asm("llvm.amdgcn.writelane.i32");
template <int kLane>
__device__ __forceinline__ void write_lane(int &v, uint32_t value)
{
    v = amdgcn_writelane(static_cast<int>(value), kLane, v);
}

// The record words of the two neighbours of load kLoad (ballots over their carrier bits) into
// the softmax lanes: beta_j into lane j of bw, t_j[h] into lane 8 h + j of tw, j = 2 kLoad + half.
template <int H, int kLoad>
__device__ __forceinline__ void gat_record_to_lanes(const uint2 raw, int &tw, int &bw)
{
    const uint64_t ballot_b = __ballot(static_cast<int>(raw.x) < 0);
    const uint64_t ballot_0 = __ballot(static_cast<int>(raw.y) < 0);
    write_lane<2 * kLoad>(bw, static_cast<uint32_t>(ballot_b));
    write_lane<2 * kLoad + 1>(bw, static_cast<uint32_t>(ballot_b >> 32));
    write_lane<2 * kLoad>(tw, static_cast<uint32_t>(ballot_0));
    write_lane<2 * kLoad + 1>(tw, static_cast<uint32_t>(ballot_0 >> 32));
    if constexpr (H == 2) {
        const uint64_t ballot_1 = __ballot((raw.x & 0x00800000u) != 0u);
        write_lane<8 + 2 * kLoad>(tw, static_cast<uint32_t>(ballot_1));
        write_lane<8 + 2 * kLoad + 1>(tw, static_cast<uint32_t>(ballot_1 >> 32));
    }
}

__device__ __forceinline__ float from_lane(int byte_address, float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(byte_address, __builtin_bit_cast(int, v)));
}

// The loaded neighbours (t .. t + 7 of the batch of cnt) into the state.  The ballots over the
// carrier bits are scalar values; they are written into lanes 0..15 (t_j[h] of neighbour j into
// lane 8 h + j, beta_j into lane j and lane 8 + j), where the scores, the running maximum and the
// weights are formed once per neighbour and head, and every row lane fetches the weight of its
// neighbour and head through the LDS crossbar.  kUnitSlope: 0 <= slope <= 1, where
// LeakyReLU(x) = max(x, slope x).
template <int H, bool kUnitSlope, int U, bool kFold>
__device__ __forceinline__ void gat_consume_group(const uint2 (&raw)[U], const GatLaneMasks &lm, int t, int cnt,
                                                  float s_lane, float slope, GatGroupState &st, float (&acc)[8])
{
    static_assert(U == 4, "a group is eight neighbours: four loads of two");
    constexpr int V = 8;
    int tw = 0, bw = 0;
    gat_record_to_lanes<H, 0>(raw[0], tw, bw);
    gat_record_to_lanes<H, 1>(raw[1], tw, bw);
    gat_record_to_lanes<H, 2>(raw[2], tw, bw);
    gat_record_to_lanes<H, 3>(raw[3], tw, bw);
    // lanes 8..15 take beta_j from lanes 0..7 (row_shr:8 into the upper two banks of a row)
    if constexpr (H == 2) bw = __builtin_amdgcn_update_dpp(bw, bw, 0x118, 0xf, 0xc, false);
    const bool present = (lm.position) < cnt - t;
    const float x = s_lane + __builtin_bit_cast(float, tw);
    const float act = kUnitSlope ? fmaxf(x, slope * x) : leaky(x, slope);
    const float e = present ? act : -INFINITY;
    const float top = max_of_eight(e);
    if ((__ballot(top > st.m) & 0xffffull) != 0ull) {          // a head's maximum moves: rescale
        const float mn = fmaxf(st.m, top);
        const float ref = mn == -INFINITY ? 0.0f : mn;
        const float f = exp2_fast(st.m - ref);                // 0 while m is -inf
        st.m = mn;
        st.ref = ref;
        st.l *= f;
        st.sw *= f;
        if constexpr (kFold) st.sf *= f;
        const float mine = from_lane(lm.head_lane, f);
#pragma unroll
        for (int v = 0; v < V; ++v) acc[v] *= mine;
    }
    const float pe = exp2_fast(e - st.ref);                   // 0 for an absent neighbour
    const float bj = __builtin_bit_cast(float, bw);
    const float w = pe * (kFold ? fabsf(bj) : bj);
    st.l += pe;
    st.sw += w;
    if constexpr (kFold) st.sf = fmaf(pe, bj, st.sf);
    float mine[U];
#pragma unroll
    for (int u = 0; u < U; ++u) mine[u] = from_lane(lm.weight_lane + 8 * u, w);
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
        for (int v = 0; v < V; ++v) acc[v] = fmaf(mine[u], embedded_value(raw[u], v), acc[v]);
    }
}

// Neighbours p0..p1-1 of one node; k_first: their first 64 column indices, one per lane (0 in
// the lanes past the list); s_lane: s_i log2(e) of the head this lane works on in the softmax
// lanes.  The column indices of a batch of 64 are fetched one batch ahead.  (Issuing a group's
// loads before the group in front of it is used was measured and is 4 % slower: the kernel
// waits for issue slots and for the memory system's rate, not for latency.)  At the end every
// lane holds the state of its own head and columns, the two halves of the wavefront added.
template <int H, bool kUnitSlope, bool kFold>
__device__ __forceinline__ void gat_accumulate_embedded(const int32_t *__restrict__ col_idx,
                                                        const char *__restrict__ rows, const GatLaneMasks &lm,
                                                        float s_lane, float slope, int64_t p0, int64_t p1, int k_first,
                                                        int lane, GatLaneState &out)
{
    constexpr int V = 8, U = kGatEmbeddedLoads;
    GatGroupState st;
    st.m = -INFINITY;
    st.ref = 0.0f;
    st.l = 0.0f;
    st.sw = 0.0f;
    st.sf = 0.0f;
#pragma unroll
    for (int v = 0; v < V; ++v) out.acc[v] = 0.0f;

    int k_ahead = k_first;
    for (int64_t pb = p0; pb < p1; pb += kWave) {
        const int cnt = static_cast<int>(p1 - pb < kWave ? p1 - pb : kWave);     // wave-uniform, >= 1
        const int k = k_ahead;
        if (pb + kWave < p1) k_ahead = pb + kWave + lane < p1 ? col_idx[pb + kWave + lane] : 0;
        int from = lm.half;
        for (int t = 0; t < cnt; t += 2 * U) {
            uint2 raw[U];
            gat_fetch_group<U>(rows, lm, k, from, cnt, raw);
            gat_consume_group<H, kUnitSlope, U, kFold>(raw, lm, t, cnt, s_lane, slope, st, out.acc);
            from += 2 * U;
        }
    }
    // totals of the head's eight lanes, handed to the row lanes of that head; the halves added
    const float l = sum_of_eight(st.l), sw = sum_of_eight(st.sw);
    out.m = from_lane(lm.head_lane, st.m);
    out.ref = out.m == -INFINITY ? 0.0f : out.m;
    out.l = from_lane(lm.head_lane, l);
    out.sw = from_lane(lm.head_lane, sw);
    out.sf = 0.0f;
    if constexpr (kFold) out.sf = from_lane(lm.head_lane, sum_of_eight(st.sf));
#pragma unroll
    for (int v = 0; v < V; ++v) out.acc[v] += __shfl_xor(out.acc[v], 32, kWave);
}

__device__ __forceinline__ GatLaneMasks gat_lane_masks(int lane, bool second_head)
{
    GatLaneMasks lm;
    lm.lane_offset = static_cast<uint32_t>(lane & 31) * 8u;
    lm.half = lane >> 5;
    lm.position = lane & 7;
    lm.head_lane = second_head ? 32 : 0;
    lm.weight_lane = lm.head_lane + 4 * lm.half;
    return lm;
}

// Brings `st` and a second state (m2, l2, sw2, sf2, acc2) of the same node, head and columns to
// their common maximum and adds them into `st`.
__device__ __forceinline__ void gat_merge_embedded(GatLaneState &st, float m2, float l2, float sw2, float sf2,
                                                   const float (&acc2)[8])
{
    const float mn = fmaxf(st.m, m2);
    const float ref = mn == -INFINITY ? 0.0f : mn;
    const float f1 = exp2_fast(st.m - ref), f2 = exp2_fast(m2 - ref);
    st.m = mn;
    st.ref = ref;
    st.l = fmaf(f2, l2, st.l * f1);
    st.sw = fmaf(f2, sw2, st.sw * f1);
    st.sf = fmaf(f2, sf2, st.sf * f1);
#pragma unroll
    for (int v = 0; v < 8; ++v) st.acc[v] = fmaf(f2, acc2[v], st.acc[v] * f1);
}

template <bool kFold>
__device__ __forceinline__ void gat_finish_embedded(const GatLaneState &st, int64_t row, int lane, float mul,
                                                    float bias, const float *__restrict__ alpha,
                                                    const float *__restrict__ last_sign,
                                                    float *__restrict__ out, int64_t ld_out, int vector_store)
{
    constexpr int V = 8;
    if (lane >= 32) return;
    const float inv = st.l > 0.0f ? 1.0f / st.l : 0.0f;
    const float base = bias * st.sw;
    float r[V];
#pragma unroll
    for (int v = 0; v < V; ++v) {
        float sum = fmaf(mul, st.acc[v], base);
        if constexpr (kFold) sum = fmaf(last_sign[lane * V + v], st.sf, sum);
        r[v] = alpha[lane * V + v] * sum * inv;
    }
    float *dst = out + row * ld_out + lane * V;
    if (vector_store) {
        reinterpret_cast<float4 *>(dst)[0] = make_float4(r[0], r[1], r[2], r[3]);
        reinterpret_cast<float4 *>(dst)[1] = make_float4(r[4], r[5], r[6], r[7]);
    } else {
#pragma unroll
        for (int v = 0; v < V; ++v) dst[v] = r[v];
    }
}

// Same division of the nodes as gat_aggregate_kernel.  256 columns, H heads of 256 / H; the rows
// take less than 4 GiB (offsets into them are 32-bit).
// misfit (nullable): a device flag; when it is set (some product did not fit 7 bits, so the rows
// were not stamped) the launch returns at once and gat_aggregate_kernel does the work instead.
template <int H, bool kUnitSlope, bool kFold>
__global__ __launch_bounds__(kBlock, 8) void gat_aggregate_embedded_kernel(
    const bigcn_plan_entry *__restrict__ entries, int64_t n, int64_t n_block_rows,
    const int32_t *__restrict__ col_idx, const char *__restrict__ rows, const float *__restrict__ s,
    const float *__restrict__ alpha, float mul, float bias, float slope, const float *__restrict__ last_sign,
    const int *__restrict__ misfit, float *__restrict__ out, int64_t ld_out, int vector_store)
{
    constexpr int V = 8;
    __shared__ float merge[kWavesPerBlock - 1][V + 4][32];
    if (misfit != nullptr && *misfit != 0) return;             // the same for every thread of the launch
    const int lane = lane_id();
    const int wave = wave_in_block();
    const bool second_head = H == 2 && (lane & 31) >= 16;
    const int softmax_head = H == 2 ? (lane >> 3) & 1 : 0;     // of the head this lane scores in lanes 0..15
    const GatLaneMasks lm = gat_lane_masks(lane, second_head);
    GatLaneState st;

    if (static_cast<int64_t>(blockIdx.x) < n_block_rows) {
        const bigcn_plan_entry e = entries[blockIdx.x];       // the row and its extent in one load
        const int64_t row = e.row;
        const int64_t p0 = e.first, p1 = e.first + e.count;
        int64_t chunk = (p1 - p0 + kWavesPerBlock - 1) / kWavesPerBlock;
        chunk = (chunk + kWave - 1) / kWave * kWave;
        int64_t q0 = p0 + wave * chunk, q1 = q0 + chunk;
        if (q0 > p1) q0 = p1;
        if (q1 > p1) q1 = p1;
        const float s_lane = s[row * H + softmax_head] * kLog2e;
        const int k_first = q0 + lane < q1 ? col_idx[q0 + lane] : 0;
        gat_accumulate_embedded<H, kUnitSlope, kFold>(col_idx, rows, lm, s_lane, slope, q0, q1, k_first, lane, st);
        if (wave > 0 && lane < 32) {
#pragma unroll
            for (int v = 0; v < V; ++v) merge[wave - 1][v][lane] = st.acc[v];
            merge[wave - 1][V][lane] = st.m;
            merge[wave - 1][V + 1][lane] = st.l;
            merge[wave - 1][V + 2][lane] = st.sw;
            merge[wave - 1][V + 3][lane] = st.sf;
        }
        __syncthreads();
        if (wave == 0 && lane < 32) {
#pragma unroll
            for (int w = 0; w < kWavesPerBlock - 1; ++w) {
                float acc2[V];
#pragma unroll
                for (int v = 0; v < V; ++v) acc2[v] = merge[w][v][lane];
                gat_merge_embedded(st, merge[w][V][lane], merge[w][V + 1][lane], merge[w][V + 2][lane], merge[w][V + 3][lane],
                                   acc2);
            }
            gat_finish_embedded<kFold>(st, row, lane, mul, bias, alpha, last_sign, out, ld_out, vector_store);
        }
        return;
    }
    const int64_t entry = n_block_rows + (static_cast<int64_t>(blockIdx.x) - n_block_rows) * kWavesPerBlock + wave;
    if (entry >= n) return;                                    // wave-uniform
    const bigcn_plan_entry e = entries[entry];
    const int64_t row = e.row;
    const float s_lane = s[row * H + softmax_head] * kLog2e;
    const int64_t p0 = e.first, p1 = e.first + e.count;
    const int k_first = p0 + lane < p1 ? col_idx[p0 + lane] : 0;
    gat_accumulate_embedded<H, kUnitSlope, kFold>(col_idx, rows, lm, s_lane, slope, p0, p1, k_first, lane, st);
    gat_finish_embedded<kFold>(st, row, lane, mul, bias, alpha, last_sign, out, ld_out, vector_store);
}

// *misfit = 1 if any stored byte is outside [-64, 63] (bit 7 differs from bit 6); the flag is
// cleared by gat_clear_flag_kernel before.
__global__ __launch_bounds__(kBlock) void gat_fit_kernel(const uint4 *__restrict__ rows, int64_t n_vec, int *__restrict__ misfit)
{
    uint32_t bad = 0;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; i < n_vec;
         i += static_cast<int64_t>(gridDim.x) * kBlock) {
        const uint4 v = rows[i];
        bad |= (v.x ^ (v.x << 1)) | (v.y ^ (v.y << 1)) | (v.z ^ (v.z << 1)) | (v.w ^ (v.w << 1));
    }
    if (__ballot((bad & 0x80808080u) != 0u) != 0ull && lane_id() == 0) *misfit = 1;   // plain store of the same value
}

__global__ void gat_clear_flag_kernel(int *__restrict__ flag) { *flag = 0; }

// last_sign[c] = +1 / -1: bit k_bits - 1 of column c's packed weights
__global__ void gat_last_sign_kernel(const uint64_t *__restrict__ w_bits, int64_t ld_words, int k_bits, int d_out,
                                     float *__restrict__ last_sign)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= d_out) return;
    const uint64_t word = w_bits[static_cast<int64_t>(c) * ld_words + ((k_bits - 1) >> 6)];
    last_sign[c] = ((word >> ((k_bits - 1) & 63)) & 1ull) ? 1.0f : -1.0f;
}

struct GatMap {
    size_t bits_off, beta_off, z_off, s_off, t_off, total;
    // compact path: z_off holds the product rows, t_off the records {beta, t[0..H-1]}
    bool compact;
    RowKind kind;
    int groups;           // lanes per row (8 values each)
    int64_t row_bytes;
    // one-byte rows of a layer with 256 input bits: the stored values cover the first 255, the last
    // one rides on the sign of the node's scale and on last_sign[c] = +-1, its weight bit
    bool fold;
    size_t sign_off, flag_off;
    const float *last_sign;   // DEVICE, set by the entry point (nullptr unless fold)
    int *misfit;              // DEVICE flag of gat_fit_kernel, set by the entry point
};

static bool gat_shape_ok(int64_t d_in, int64_t d_out, int heads)
{
    return d_in > 0 && d_in <= BIGCN_MAX_K_BITS && d_out > 0 && d_out <= kWave * kGatMaxV &&
           (heads == 1 || heads == 2 || heads == 4 || heads == 8) && d_out % heads == 0;
}

static GatMap map_gat(int64_t n, int64_t d_in, int64_t d_out, int heads)
{
    auto up = [](size_t v) { return (v + 255) & ~static_cast<size_t>(255); };
    GatMap m;
    m.compact = (d_out / heads) % 8 == 0;
    m.fold = m.compact && d_in == 256;
    m.kind = (d_in <= 255 || m.fold) ? kI8 : (d_in <= 2048 ? kF16 : kF32);
    m.last_sign = nullptr;
    m.groups = 2;
    while (m.groups < kWave && m.groups * 8 < d_out) m.groups <<= 1;
    m.row_bytes = static_cast<int64_t>(m.groups) * 8 * (m.kind == kI8 ? 1 : (m.kind == kF16 ? 2 : 4));
    size_t off = 0;
    m.bits_off = off; off = up(off + static_cast<size_t>(n) * ((d_in + 63) / 64) * 8);
    m.beta_off = off; off = up(off + static_cast<size_t>(n) * 4);
    m.z_off = off;    off = up(off + static_cast<size_t>(n) * (m.compact ? m.row_bytes : d_out * 4));
    m.s_off = off;    off = up(off + static_cast<size_t>(n) * heads * 4);
    // compact path: records of (heads + 1) floats padded to whole 16-byte vectors
    m.t_off = off;    off = up(off + static_cast<size_t>(n) * (m.compact ? (heads + 1 + 3) / 4 * 4 : heads) * 4);
    m.sign_off = off; off = up(off + (m.fold ? static_cast<size_t>(d_out) * 4 : 0));
    m.flag_off = off; off = up(off + 4);
    m.misfit = nullptr;
    m.total = off;
    return m;
}

template <typename T, int G, int H>
static int launch_gat_compact(const bigcn_plan *plan, const int64_t *row_ptr, const int32_t *col_idx, int64_t n,
                              const GatMap &map, char *rows, const float *beta, const float *alpha,
                              const float *a_src, const float *a_dst, float *s, float *record, int64_t d_in,
                              int64_t d_out, float slope, float *out, int64_t ld_out, hipStream_t st)
{
    // The record rides in the rows' spare top bits when every product fits 7 bits: always so up to
    // 127 input bits; up to 256 the rows are tested first (a product over K' bits has standard
    // deviation sqrt(K') / 2, so 7 bits hold 8 sigma at K' = 255) and a device flag picks, inside
    // the launches, between the kernels that read stamped rows and those that read records.
    const int64_t k_stored = map.fold ? d_in - 1 : d_in;
    const bool shape_embeds = gat_embeds<T, G, H>() && d_out == 256 && k_stored <= 255 && n < (int64_t{1} << 24);
    const int embed_mode = !shape_embeds ? 0 : (k_stored <= 127 ? 1 : 2);
    const float mul = sizeof(T) == 1 ? 2.0f : 1.0f;
    const float bias = sizeof(T) == 1 ? static_cast<float>(k_stored & 1) : 0.0f;
    const int d_head = static_cast<int>(d_out / H);
    if (embed_mode == 2) {
        hipLaunchKernelGGL(gat_clear_flag_kernel, dim3(1), dim3(1), 0, st, map.misfit);
        if (hipGetLastError() != hipSuccess) return BIGCN_EHIP;
        const int64_t n_vec = n * map.row_bytes / 16;
        hipLaunchKernelGGL(gat_fit_kernel, dim3(static_cast<unsigned>(compute_units() * 16)), dim3(kBlock), 0, st,
                           reinterpret_cast<const uint4 *>(rows), n_vec, map.misfit);
        if (hipGetLastError() != hipSuccess) return BIGCN_EHIP;
    }
    const int64_t node_blocks = (n + kWavesPerBlock - 1) / kWavesPerBlock;
    const int64_t score_blocks = node_blocks > compute_units() * 8 ? compute_units() * 8 : node_blocks;
    hipLaunchKernelGGL((gat_scores_kernel<T, G, H>), dim3(static_cast<unsigned>(score_blocks)), dim3(kBlock), 0, st,
                       rows, static_cast<uint32_t>(map.row_bytes), n, static_cast<int>(d_out), d_head, mul, bias, beta,
                       alpha, a_src, a_dst, s, record, embed_mode, map.misfit, map.last_sign);
    if (hipGetLastError() != hipSuccess) return BIGCN_EHIP;
    const int64_t wave_rows = n - plan->n_block_rows;
    const int64_t blocks = plan->n_block_rows + (wave_rows + kWavesPerBlock - 1) / kWavesPerBlock;
    const dim3 grid(static_cast<unsigned>(blocks));
    const int vector_store = (ld_out % 4 == 0 && reinterpret_cast<uintptr_t>(out) % 16 == 0) ? 1 : 0;
    const int *flag = embed_mode == 2 ? map.misfit : nullptr;
    if constexpr (gat_embeds<T, G, H>()) {
        if (embed_mode != 0) {
            const bool unit = slope >= 0.0f && slope <= 1.0f;
#define BIGCN_GAT_EMBEDDED(UNIT, FOLD)                                                                              \
    hipLaunchKernelGGL((gat_aggregate_embedded_kernel<H, UNIT, FOLD>), grid, dim3(kBlock), 0, st, plan->entries, n,  \
                       plan->n_block_rows, col_idx, rows, s, alpha, mul, bias, slope, map.last_sign, flag, out,     \
                       ld_out, vector_store)
            if (map.fold) {
                if (unit) BIGCN_GAT_EMBEDDED(true, true);
                else BIGCN_GAT_EMBEDDED(false, true);
            } else {
                if (unit) BIGCN_GAT_EMBEDDED(true, false);
                else BIGCN_GAT_EMBEDDED(false, false);
            }
#undef BIGCN_GAT_EMBEDDED
            if (embed_mode == 1) return check_launch();
            if (hipGetLastError() != hipSuccess) return BIGCN_EHIP;
        }
    }
    if constexpr (sizeof(T) == 1) {
        if (map.fold) {
            hipLaunchKernelGGL((gat_aggregate_kernel<T, G, H, true>), grid, dim3(kBlock), 0, st, plan->entries, n,
                               plan->n_block_rows, col_idx, rows, static_cast<uint32_t>(map.row_bytes), s, record, alpha,
                               static_cast<int>(d_out), d_head, mul, bias, slope, map.last_sign, flag, out, ld_out,
                               vector_store);
            return check_launch();
        }
    }
    hipLaunchKernelGGL((gat_aggregate_kernel<T, G, H, false>), grid, dim3(kBlock), 0, st, plan->entries, n,
                       plan->n_block_rows, col_idx, rows, static_cast<uint32_t>(map.row_bytes), s, record, alpha,
                       static_cast<int>(d_out), d_head, mul, bias, slope, nullptr, flag, out, ld_out, vector_store);
    return check_launch();
}

template <typename T, int H>
static int launch_gat_compact_groups(int groups, const bigcn_plan *plan, const int64_t *row_ptr,
                                     const int32_t *col_idx, int64_t n, const GatMap &map, char *rows,
                                     const float *beta, const float *alpha, const float *a_src, const float *a_dst,
                                     float *s, float *record, int64_t d_in, int64_t d_out, float slope, float *out,
                                     int64_t ld_out, hipStream_t st)
{
#define BIGCN_GAT_GROUPS(GG)                                                                                        \
    case GG:                                                                                                        \
        return launch_gat_compact<T, GG, H>(plan, row_ptr, col_idx, n, map, rows, beta, alpha, a_src, a_dst, s,    \
                                            record, d_in, d_out, slope, out, ld_out, st)
    switch (groups) {
        BIGCN_GAT_GROUPS(2);
        BIGCN_GAT_GROUPS(4);
        BIGCN_GAT_GROUPS(8);
        BIGCN_GAT_GROUPS(16);
        BIGCN_GAT_GROUPS(32);
        BIGCN_GAT_GROUPS(64);
    default:
        return BIGCN_EINVAL;
    }
#undef BIGCN_GAT_GROUPS
}

template <typename T>
static int launch_gat_compact_heads(int heads, int groups, const bigcn_plan *plan, const int64_t *row_ptr,
                                    const int32_t *col_idx, int64_t n, const GatMap &map, char *rows,
                                    const float *beta, const float *alpha, const float *a_src, const float *a_dst,
                                    float *s, float *record, int64_t d_in, int64_t d_out, float slope, float *out,
                                    int64_t ld_out, hipStream_t st)
{
#define BIGCN_GAT_HEADS(HH)                                                                                         \
    case HH:                                                                                                        \
        return launch_gat_compact_groups<T, HH>(groups, plan, row_ptr, col_idx, n, map, rows, beta, alpha, a_src,  \
                                                a_dst, s, record, d_in, d_out, slope, out, ld_out, st)
    switch (heads) {
        BIGCN_GAT_HEADS(1);
        BIGCN_GAT_HEADS(2);
        BIGCN_GAT_HEADS(4);
        BIGCN_GAT_HEADS(8);
    default:
        return BIGCN_ESHAPE;
    }
#undef BIGCN_GAT_HEADS
}

}  // namespace bigcn

using namespace bigcn;

extern "C" size_t bigcn_gat_layer_workspace_bytes(int64_t n, int64_t d_in, int64_t d_out, int heads)
{
    if (n <= 0 || !gat_shape_ok(d_in, d_out, heads)) return 0;
    return map_gat(n, d_in, d_out, heads).total;
}

extern "C" int bigcn_gat_layer(const bigcn_plan *plan, const int64_t *row_ptr, const int32_t *col_idx, int64_t n,
                               const float *x, int64_t ld_x, const float *bn_shift, const float *bn_mul,
                               const uint64_t *w_bits, const float *alpha, int64_t ld_words, int64_t d_in,
                               int64_t d_out, int heads, const float *a_src, const float *a_dst,
                               float negative_slope, float *out, int64_t ld_out, void *workspace,
                               size_t workspace_bytes, void *stream)
{
    if (plan == nullptr || row_ptr == nullptr || col_idx == nullptr || x == nullptr || w_bits == nullptr ||
        alpha == nullptr || a_src == nullptr || a_dst == nullptr || out == nullptr)
        return BIGCN_ENULL;
    if (n != plan->n || d_in <= 0 || d_out <= 0 || ld_x < d_in || ld_out < d_out || ld_words < (d_in + 63) / 64 ||
        heads <= 0 || (heads > 0 && d_out % heads != 0))
        return BIGCN_EINVAL;
    if (!gat_shape_ok(d_in, d_out, heads)) return BIGCN_ESHAPE;
    if (n == 0) return BIGCN_OK;
    GatMap map = map_gat(n, d_in, d_out, heads);
    if (workspace == nullptr || workspace_bytes < map.total || reinterpret_cast<uintptr_t>(workspace) % 256 != 0)
        return BIGCN_EWORKSPACE;
    hipStream_t st = as_stream(stream);
    char *ws = static_cast<char *>(workspace);
    uint64_t *bits = reinterpret_cast<uint64_t *>(ws + map.bits_off);
    float *beta = reinterpret_cast<float *>(ws + map.beta_off);
    float *s = reinterpret_cast<float *>(ws + map.s_off);
    float *t = reinterpret_cast<float *>(ws + map.t_off);
    const int64_t words = (d_in + 63) / 64;

    // fold: the scale carries the sign of the node's last input bit
    int rc = launch_pack(x, n, d_in, ld_x, 1, bn_shift, bn_mul, nullptr, map.fold ? 1 : 0, bits, words, beta, st);
    if (rc != BIGCN_OK) return rc;

    if (map.compact) {
        char *rows = ws + map.z_off;
        const int64_t k_stored = map.fold ? d_in - 1 : d_in;          // bits covered by the stored values
        if (map.fold) {
            float *last_sign = reinterpret_cast<float *>(ws + map.sign_off);
            hipLaunchKernelGGL(gat_last_sign_kernel, dim3(static_cast<unsigned>((d_out + 255) / 256)), dim3(256), 0, st,
                               w_bits, ld_words, static_cast<int>(d_in), static_cast<int>(d_out), last_sign);
            if (hipGetLastError() != hipSuccess) return BIGCN_EHIP;
            map.last_sign = last_sign;
        }
        map.misfit = reinterpret_cast<int *>(ws + map.flag_off);
        // large layers of one-byte rows on the matrix cores, everything else by XOR and bit counts
        if (map.kind == kI8 && fp4_natural_covers(n, k_stored, map.groups * 8))
            rc = launch_bitgemm_fp4_natural(bits, n, words, w_bits, d_out, ld_words, k_stored, rows, map.groups * 8, st);
        else
            rc = launch_bitgemm_natural(bits, n, words, w_bits, d_out, ld_words, k_stored, rows, map.groups * 8, map.kind, st,
                                        map.fold ? 0x7fffffffu : 0xffffffffu);
        if (rc != BIGCN_OK) return rc;
        if (map.kind == kI8)
            return launch_gat_compact_heads<int8_t>(heads, map.groups, plan, row_ptr, col_idx, n, map, rows, beta,
                                                    alpha, a_src, a_dst, s, t, d_in, d_out, negative_slope, out,
                                                    ld_out, st);
        if (map.kind == kF16)
            return launch_gat_compact_heads<__half>(heads, map.groups, plan, row_ptr, col_idx, n, map, rows, beta,
                                                    alpha, a_src, a_dst, s, t, d_in, d_out, negative_slope, out,
                                                    ld_out, st);
        return launch_gat_compact_heads<float>(heads, map.groups, plan, row_ptr, col_idx, n, map, rows, beta, alpha,
                                               a_src, a_dst, s, t, d_in, d_out, negative_slope, out, ld_out, st);
    }

    float *z = reinterpret_cast<float *>(ws + map.z_off);
    rc = bigcn_binary_gemm(bits, beta, n, words, w_bits, alpha, d_out, ld_words, d_in, nullptr, 0, z, d_out, stream);
    if (rc != BIGCN_OK) return rc;

    const int d_head = static_cast<int>(d_out / heads);
    int64_t blocks = (n + kWavesPerBlock - 1) / kWavesPerBlock;
    const int64_t score_blocks = blocks > compute_units() * 32 ? compute_units() * 32 : blocks;
#define BIGCN_GAT_CASE(HH)                                                                                          \
    case HH:                                                                                                        \
        hipLaunchKernelGGL(gat_scores_plain_kernel<HH>, dim3(static_cast<unsigned>(score_blocks)), dim3(kBlock), 0, st, z, n, \
                           static_cast<int>(d_out), d_head, a_src, a_dst, s, t);                                    \
        if (hipGetLastError() != hipSuccess) return BIGCN_EHIP;                                                     \
        hipLaunchKernelGGL(gat_aggregate_plain_kernel<HH>, dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0, st,      \
                           plan->row_order, n, row_ptr, col_idx, z, static_cast<int>(d_out), d_head, s, t,          \
                           negative_slope, out, ld_out);                                                            \
        break
    switch (heads) {
        BIGCN_GAT_CASE(1);
        BIGCN_GAT_CASE(2);
        BIGCN_GAT_CASE(4);
        BIGCN_GAT_CASE(8);
    default:
        return BIGCN_ESHAPE;
    }
#undef BIGCN_GAT_CASE
    return check_launch();
}
