// One Bi-GAT layer (Sec. 4.4.1): z_j = W~ (*) h~_j by the binarise+pack and bit-GEMM kernels
// (Sec. 4.2), then, per head,
//   e_ij = LeakyReLU(a_src . z_i + a_dst . z_j),  a_ij = softmax_{j in N_i} e_ij,
//   out_i = sum_{j in N_i} a_ij z_j.
// The attention vectors are not binarised.  Two kernels follow the GEMM: the per-node scores
// s_i = a_src . z_i and t_i = a_dst . z_i, and the aggregation, which owns a node per wavefront,
// takes the row maximum of e_ij first and then accumulates exp(e_ij - max) z_j and its sum in a
// fixed order (run-to-run identical).  A first version: z is kept in fp32 rows.
#include "bigcn_internal.h"

namespace bigcn {

constexpr int kGatMaxV = 8;              // columns per lane: d_out <= 512

// s[i][h], t[i][h]: one wavefront per node, lane l takes columns l, l + 64, ...
template <int H>
__global__ __launch_bounds__(kBlock) void gat_scores_kernel(const float *__restrict__ z, int64_t n, int d_out, int d_head,
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
__global__ __launch_bounds__(kBlock) void gat_aggregate_kernel(const int32_t *__restrict__ row_order, int64_t n,
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

struct GatMap {
    size_t bits_off, beta_off, z_off, s_off, t_off, total;
};

static GatMap map_gat(int64_t n, int64_t d_in, int64_t d_out, int heads)
{
    auto up = [](size_t v) { return (v + 255) & ~static_cast<size_t>(255); };
    GatMap m;
    size_t off = 0;
    m.bits_off = off; off = up(off + static_cast<size_t>(n) * ((d_in + 63) / 64) * 8);
    m.beta_off = off; off = up(off + static_cast<size_t>(n) * 4);
    m.z_off = off;    off = up(off + static_cast<size_t>(n) * d_out * 4);
    m.s_off = off;    off = up(off + static_cast<size_t>(n) * heads * 4);
    m.t_off = off;    off = up(off + static_cast<size_t>(n) * heads * 4);
    m.total = off;
    return m;
}

static bool gat_shape_ok(int64_t d_in, int64_t d_out, int heads)
{
    return d_in > 0 && d_in <= BIGCN_MAX_K_BITS && d_out > 0 && d_out <= kWave * kGatMaxV &&
           (heads == 1 || heads == 2 || heads == 4 || heads == 8) && d_out % heads == 0;
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
    const GatMap map = map_gat(n, d_in, d_out, heads);
    if (workspace == nullptr || workspace_bytes < map.total || reinterpret_cast<uintptr_t>(workspace) % 256 != 0)
        return BIGCN_EWORKSPACE;
    hipStream_t st = as_stream(stream);
    char *ws = static_cast<char *>(workspace);
    uint64_t *bits = reinterpret_cast<uint64_t *>(ws + map.bits_off);
    float *beta = reinterpret_cast<float *>(ws + map.beta_off);
    float *z = reinterpret_cast<float *>(ws + map.z_off);
    float *s = reinterpret_cast<float *>(ws + map.s_off);
    float *t = reinterpret_cast<float *>(ws + map.t_off);
    const int64_t words = (d_in + 63) / 64;

    int rc = launch_pack(x, n, d_in, ld_x, 1, bn_shift, bn_mul, nullptr, 0, bits, words, beta, st);
    if (rc != BIGCN_OK) return rc;
    rc = bigcn_binary_gemm(bits, beta, n, words, w_bits, alpha, d_out, ld_words, d_in, nullptr, 0, z, d_out, stream);
    if (rc != BIGCN_OK) return rc;

    const int d_head = static_cast<int>(d_out / heads);
    int64_t blocks = (n + kWavesPerBlock - 1) / kWavesPerBlock;
    const int64_t score_blocks = blocks > 256 * 32 ? 256 * 32 : blocks;
#define BIGCN_GAT_CASE(HH)                                                                                          \
    case HH:                                                                                                        \
        hipLaunchKernelGGL(gat_scores_kernel<HH>, dim3(static_cast<unsigned>(score_blocks)), dim3(kBlock), 0, st, z, n, \
                           static_cast<int>(d_out), d_head, a_src, a_dst, s, t);                                    \
        if (hipGetLastError() != hipSuccess) return BIGCN_EHIP;                                                     \
        hipLaunchKernelGGL(gat_aggregate_kernel<HH>, dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0, st,      \
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
