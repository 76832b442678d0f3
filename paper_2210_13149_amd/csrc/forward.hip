// Fused L-layer driver (Eq. (1) with H^(0) = X, Sec. 4.2.3 per layer) and library metadata.
//
// Per layer l the stream carries two steps: the bit-GEMM, which turns the packed signs of
// the layer input into the integer products C (one compact row per node), and the fused
// aggregation, which gathers those rows over the graph, applies beta_k / alpha_j / degree
// scaling and emits either the next layer's packed signs and scales or the final logits.
// Only the first layer needs a separate binarise+pack pass over the fp32 features.
// The Bi-GraphSAGE driver (Sec. 4.4.2) is the same sequence with two bit-GEMMs per layer (one
// product array per weight matrix) and an aggregation that adds the node's own row.
#include <algorithm>
#include <mutex>
#include <new>

#include "bigcn_internal.h"

namespace bigcn {

struct WorkspaceMap {
    size_t bits_off, scale0_off, scale1_off, rows_off, self_rows_off, alt_rows_off, alt_self_rows_off, flags_off, total;
    bool escape;      // some layer keeps an alternate copy (bytes or fp16) of rows that do not fit 7 bits
};

static size_t align_up(size_t v) { return (v + 255) & ~static_cast<size_t>(255); }

// One layer as both drivers see it; w_self_bits == nullptr for Bi-GCN.
struct LayerView {
    const uint64_t *w_bits;
    const float *alpha;
    const uint64_t *w_self_bits;
    const float *alpha_self;
    int64_t d_in, d_out, ld_words;
    const float *bn_shift, *bn_mul;
};

constexpr int kMaxLayers = BIGCN_MAX_LAYERS;

static bool layers_ok(int64_t n, const LayerView *layers, int n_layers, bool own_term, int *status)
{
    *status = BIGCN_OK;
    if (n < 0 || n_layers <= 0 || n_layers > kMaxLayers) { *status = BIGCN_EINVAL; return false; }
    for (int l = 0; l < n_layers; ++l) {
        const LayerView &L = layers[l];
        if (L.w_bits == nullptr || L.alpha == nullptr) { *status = BIGCN_ENULL; return false; }
        if (own_term && (L.w_self_bits == nullptr || L.alpha_self == nullptr)) { *status = BIGCN_ENULL; return false; }
        if (L.d_in <= 0 || L.d_out <= 0 || L.ld_words < (L.d_in + 63) / 64) { *status = BIGCN_EINVAL; return false; }
        if (l > 0 && L.d_in != layers[l - 1].d_out) { *status = BIGCN_EINVAL; return false; }
        if (L.d_in > BIGCN_MAX_K_BITS || L.d_out > BIGCN_MAX_FORWARD_D_OUT) { *status = BIGCN_ESHAPE; return false; }
    }
    return true;
}

static int view_gcn(const bigcn_layer *layers, int n_layers, LayerView *out)
{
    if (layers == nullptr) return BIGCN_ENULL;
    if (n_layers <= 0 || n_layers > kMaxLayers) return BIGCN_EINVAL;
    for (int l = 0; l < n_layers; ++l)
        out[l] = LayerView{layers[l].w_bits, layers[l].alpha, nullptr, nullptr, layers[l].d_in,
                           layers[l].d_out, layers[l].ld_words, layers[l].bn_shift, layers[l].bn_mul};
    return BIGCN_OK;
}

static int view_sage(const bigcn_sage_layer *layers, int n_layers, LayerView *out)
{
    if (layers == nullptr) return BIGCN_ENULL;
    if (n_layers <= 0 || n_layers > kMaxLayers) return BIGCN_EINVAL;
    for (int l = 0; l < n_layers; ++l)
        out[l] = LayerView{layers[l].w_nbr_bits, layers[l].alpha_nbr, layers[l].w_self_bits,
                           layers[l].alpha_self, layers[l].d_in, layers[l].d_out, layers[l].ld_words,
                           layers[l].bn_shift, layers[l].bn_mul};
    return BIGCN_OK;
}

static WorkspaceMap map_workspace(int64_t n, const LayerView *layers, int n_layers, bool own_term)
{
    int64_t max_words = 0, max_row_bytes = 0, max_alt_bytes = 0;
    for (int l = 0; l < n_layers; ++l) {
        const RowLayout layout = choose_layout(layers[l].d_in, layers[l].d_out);
        max_words = std::max<int64_t>(max_words, (layers[l].d_in + 63) / 64);
        max_row_bytes = std::max<int64_t>(max_row_bytes, layout.row_bytes());
        if (layout.escape) max_alt_bytes = std::max<int64_t>(max_alt_bytes, layout.alt_row_bytes());
    }
    WorkspaceMap m;
    m.escape = max_alt_bytes > 0;
    size_t off = 0;
    m.bits_off = off;   off = align_up(off + static_cast<size_t>(n) * max_words * sizeof(uint64_t));
    m.scale0_off = off; off = align_up(off + static_cast<size_t>(n) * sizeof(float));
    m.scale1_off = off; off = align_up(off + static_cast<size_t>(n) * sizeof(float));
    m.rows_off = off;   off = align_up(off + static_cast<size_t>(n) * max_row_bytes);
    m.self_rows_off = off;
    if (own_term) off = align_up(off + static_cast<size_t>(n) * max_row_bytes);
    m.alt_rows_off = off;
    if (m.escape) off = align_up(off + static_cast<size_t>(n) * max_alt_bytes);
    m.alt_self_rows_off = off;
    if (m.escape && own_term) off = align_up(off + static_cast<size_t>(n) * max_alt_bytes);
    // one int per layer: "some product row of this layer went to the alternate array"
    m.flags_off = off;
    if (m.escape) off = align_up(off + kMaxLayers * sizeof(int));
    m.total = off;
    return m;
}

}  // namespace bigcn

// Workspace of bigcn_forward_static, for callers that cannot allocate: one copy per GPU that
// loads the library, held until the process ends.  The name is only a host-side handle of the
// symbol; host code uses the device address looked up once per device (static_workspace()).
static __device__ __align__(256) unsigned char scratch[BIGCN_STATIC_WORKSPACE_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void *scratch_ptr[kMaxDevices];   // device address of `scratch` on GPU d, nullptr until first use

// Address of the current device's copy of `scratch`.
int static_workspace(void **out)
{
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return BIGCN_EHIP;
    std::lock_guard<std::mutex> guard(scratch_mutex);
    if (scratch_ptr[device] == nullptr) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return BIGCN_EHIP;
        scratch_ptr[device] = p;
    }
    *out = scratch_ptr[device];
    return BIGCN_OK;
}

}  // namespace

// Per-launch timing of forward passes: (1 + 2 L) launches per call bracketed by (2 + 2 L)
// events, for up to max_calls calls between two reads.
struct bigcn_profile {
    int n_layers;
    int max_calls;
    int calls;
    hipEvent_t *events;      // max_calls * (2 + 2 * n_layers)
    int per_call() const { return 2 + 2 * n_layers; }
};

using namespace bigcn;

extern "C" const char *bigcn_status_string(int status)
{
    switch (status) {
    case BIGCN_OK: return "ok";
    case BIGCN_EINVAL: return "invalid size, stride or flag";
    case BIGCN_ENULL: return "required pointer is NULL";
    case BIGCN_ESHAPE: return "shape exceeds a documented limit";
    case BIGCN_EWORKSPACE: return "workspace missing, too small or misaligned";
    case BIGCN_EGRAPH: return "CSR pattern failed validation";
    case BIGCN_EHIP: return "HIP runtime call or kernel launch failed";
    default: return "unknown status";
    }
}

extern "C" int bigcn_version(void) { return 0 * 10000 + 1 * 100 + 0; }

extern "C" int64_t bigcn_forward_row_bytes(int64_t d_in, int64_t d_out, int *scale_embedded)
{
    if (d_in <= 0 || d_out <= 0 || d_in > BIGCN_MAX_K_BITS || d_out > BIGCN_MAX_FORWARD_D_OUT) return 0;
    const RowLayout l = choose_layout(d_in, d_out);
    if (scale_embedded != nullptr) *scale_embedded = l.embed_scale != kScaleSeparate ? 1 : 0;
    return l.row_bytes();
}

extern "C" int bigcn_forward_row_layout(int64_t d_in, int64_t d_out, int32_t *fields)
{
    if (fields == nullptr) return BIGCN_ENULL;
    if (d_in <= 0 || d_out <= 0 || d_in > BIGCN_MAX_K_BITS || d_out > BIGCN_MAX_FORWARD_D_OUT) return BIGCN_EINVAL;
    const RowLayout l = choose_layout(d_in, d_out);
    const int32_t v[8] = {l.groups, l.vec, l.kind, l.k_eff, l.fold_last, l.embed_scale, l.escape, l.alt_kind};
    for (int i = 0; i < 8; ++i) fields[i] = v[i];
    return BIGCN_OK;
}

extern "C" int bigcn_forward_workspace_map(int64_t n, const bigcn_layer *layers, int n_layers, size_t *offsets)
{
    if (offsets == nullptr) return BIGCN_ENULL;
    LayerView view[kMaxLayers];
    int status = view_gcn(layers, n_layers, view);
    if (status != BIGCN_OK) return status;
    if (!layers_ok(n, view, n_layers, false, &status)) return status;
    const WorkspaceMap m = map_workspace(n, view, n_layers, false);
    const size_t v[6] = {m.bits_off, m.scale0_off, m.scale1_off, m.rows_off, m.alt_rows_off, m.total};
    for (int i = 0; i < 6; ++i) offsets[i] = v[i];
    return BIGCN_OK;
}

extern "C" int bigcn_forward_gemm_path(int64_t n, int64_t d_in, int64_t d_out)
{
    if (n < 0 || d_in <= 0 || d_out <= 0 || d_in > BIGCN_MAX_K_BITS || d_out > BIGCN_MAX_FORWARD_D_OUT) return BIGCN_EINVAL;
    return fp4_rows_covers(n, d_in, choose_layout(d_in, d_out)) ? BIGCN_GEMM_FP4 : BIGCN_GEMM_VALU;
}

extern "C" size_t bigcn_forward_workspace_bytes(int64_t n, const bigcn_layer *layers, int n_layers)
{
    LayerView view[kMaxLayers];
    int status;
    if (view_gcn(layers, n_layers, view) != BIGCN_OK || !layers_ok(n, view, n_layers, false, &status)) return 0;
    return map_workspace(n, view, n_layers, false).total;
}

extern "C" size_t bigcn_sage_forward_workspace_bytes(int64_t n, const bigcn_sage_layer *layers, int n_layers)
{
    LayerView view[kMaxLayers];
    int status;
    if (view_sage(layers, n_layers, view) != BIGCN_OK || !layers_ok(n, view, n_layers, true, &status)) return 0;
    return map_workspace(n, view, n_layers, true).total;
}

// dst_mul: factor of node i's neighbour sum; src_row_mul: factor folded into every stored source
// scale (nullptr = 1).  Bi-GCN passes D^-1/2 for both; Bi-GraphSAGE passes 1/|N_i| and nullptr.
// The input is either fp32 features (x, ld_x) or their packed signs and row scales
// (in.bits, in.ld_words, in.beta) with x == nullptr.
struct PackedInput {
    const uint64_t *bits;
    int64_t ld_words;
    const float *beta;
};

static int forward_impl(const bigcn_plan *plan, const int64_t *row_ptr, const int32_t *col_idx,
                        const float *dst_mul, const float *src_row_mul, bool own_term, int64_t n,
                        const float *x, int64_t ld_x, PackedInput in, const LayerView *layers, int n_layers,
                        float *logits, int64_t ld_logits, void *workspace, size_t workspace_bytes,
                        void *stream, bigcn_profile *prof)
{
    const bool packed = x == nullptr;
    if (plan == nullptr || row_ptr == nullptr || col_idx == nullptr || dst_mul == nullptr || logits == nullptr)
        return BIGCN_ENULL;
    if (packed && (in.bits == nullptr || in.beta == nullptr)) return BIGCN_ENULL;
    int status;
    if (!layers_ok(n, layers, n_layers, own_term, &status)) return status;
    if (n != plan->n || ld_logits < layers[n_layers - 1].d_out) return BIGCN_EINVAL;
    if (!packed && ld_x < layers[0].d_in) return BIGCN_EINVAL;
    // a packed input was standardised (if at all) when it was packed
    if (packed && (in.ld_words < (layers[0].d_in + 63) / 64 || layers[0].bn_shift != nullptr ||
                   layers[0].bn_mul != nullptr))
        return BIGCN_EINVAL;
    const WorkspaceMap map = map_workspace(n, layers, n_layers, own_term);
    if (n == 0) return BIGCN_OK;
    if (workspace == nullptr || workspace_bytes < map.total || reinterpret_cast<uintptr_t>(workspace) % 256 != 0)
        return BIGCN_EWORKSPACE;
    hipEvent_t *ev = nullptr;
    if (prof != nullptr) {
        if (prof->n_layers != n_layers) return BIGCN_EINVAL;
        if (prof->calls >= prof->max_calls) return BIGCN_ESHAPE;
        ev = prof->events + static_cast<size_t>(prof->calls) * prof->per_call();
    }

    hipStream_t s = as_stream(stream);
#define BIGCN_MARK() do { if (ev != nullptr && hipEventRecord(*ev++, s) != hipSuccess) return BIGCN_EHIP; } while (0)
    char *ws = static_cast<char *>(workspace);
    uint64_t *bits = reinterpret_cast<uint64_t *>(ws + map.bits_off);
    float *scale[2] = {reinterpret_cast<float *>(ws + map.scale0_off), reinterpret_cast<float *>(ws + map.scale1_off)};
    void *c_rows = ws + map.rows_off;
    void *self_rows = own_term ? ws + map.self_rows_off : nullptr;
    void *alt_rows = map.escape ? ws + map.alt_rows_off : nullptr;
    void *alt_self_rows = (map.escape && own_term) ? ws + map.alt_self_rows_off : nullptr;
    // Flag of a layer whose layout has one-byte alternates: cleared by the kernel that runs before
    // the layer's bit-GEMMs (the aggregation of the layer before; for layer 0 the binarisation of X
    // or the source-scale kernel), set by the bit-GEMMs when a row goes to the alternate array, and
    // the gate of the layer's two aggregation launches (without the per-row test when it is 0, with
    // it otherwise).  When the binarisation is folded into the first bit-GEMM no kernel runs ahead
    // of it, and layer 0 keeps the single launch with the test.
    int *flags = map.escape ? reinterpret_cast<int *>(ws + map.flags_off) : nullptr;

    // layer 0 input: binarise X (or take it binarised); the stored scale is src_row_mul[i] * beta_i
    int64_t words = (layers[0].d_in + 63) / 64;
    const uint64_t *in_bits = bits;
    const RowLayout layout0 = choose_layout(layers[0].d_in, layers[0].d_out);
    const int fold0 = layout0.fold_last;
    // small graphs: the binarisation of X is folded into the first bit-GEMM (one launch fewer, no
    // packed input written); not with an own-row term, whose two products share the packed input
    const bool fuse0 = !packed && !own_term && pack_bitgemm_covers(n, layers[0].d_in, layout0);
    BIGCN_MARK();
    int rc = BIGCN_OK;
    if (fuse0) {
        // nothing to launch here
    } else if (packed) {
        in_bits = in.bits;
        words = in.ld_words;
        rc = launch_source_scale(in.beta, src_row_mul, in.bits, in.ld_words, layers[0].d_in, fold0, scale[0], n, s,
                                 (layout0.escape && layout0.alt_kind == kI8) ? flags : nullptr);
    } else {
        rc = launch_pack(x, n, layers[0].d_in, ld_x, 1, layers[0].bn_shift, layers[0].bn_mul, src_row_mul, fold0,
                         bits, words, scale[0], s, (layout0.escape && layout0.alt_kind == kI8) ? flags : nullptr);
    }
    if (rc != BIGCN_OK) return rc;
    BIGCN_MARK();

    for (int l = 0; l < n_layers; ++l) {
        const LayerView &L = layers[l];
        const RowLayout layout = choose_layout(L.d_in, L.d_out);
        // (with fp16 alternates the kernel with the test measured no slower than the plain one: no flag)
        int *flag = (flags != nullptr && layout.escape && layout.alt_kind == kI8 && !(l == 0 && fuse0)) ? flags + l : nullptr;
        if (l == 0 && fuse0)
            rc = launch_pack_bitgemm_layout(x, n, ld_x, L.bn_shift, L.bn_mul, src_row_mul, scale[0], L.w_bits, L.d_out,
                                            L.ld_words, L.d_in, c_rows, alt_rows, layout, s);
        else if (fp4_rows_covers(n, L.d_in, layout))
            rc = launch_bitgemm_fp4_rows(in_bits, n, words, L.w_bits, L.d_out, L.ld_words, L.d_in, scale[l & 1], c_rows,
                                         alt_rows, layout, s, flag);
        else
            rc = launch_bitgemm_layout(in_bits, n, words, L.w_bits, L.d_out, L.ld_words, L.d_in, scale[l & 1], c_rows,
                                       alt_rows, layout, s, flag);
        if (rc != BIGCN_OK) return rc;
        if (own_term) {
            if (fp4_rows_covers(n, L.d_in, layout))
                rc = launch_bitgemm_fp4_rows(in_bits, n, words, L.w_self_bits, L.d_out, L.ld_words, L.d_in, scale[l & 1],
                                             self_rows, alt_self_rows, layout, s, flag);
            else
                rc = launch_bitgemm_layout(in_bits, n, words, L.w_self_bits, L.d_out, L.ld_words, L.d_in, scale[l & 1],
                                           self_rows, alt_self_rows, layout, s, flag);
            if (rc != BIGCN_OK) return rc;
        }
        BIGCN_MARK();

        FusedSpmmArgs a{};
        a.plan = plan;
        a.row_ptr = row_ptr;
        a.col_idx = col_idx;
        a.dst_mul = dst_mul;
        a.src_scale = scale[l & 1];
        a.c_rows = c_rows;
        a.alt_rows = alt_rows;
        a.alt_self_rows = alt_self_rows;
        a.escape_flag = flag;
        if (flags != nullptr && l + 1 < n_layers) {
            const RowLayout next = choose_layout(layers[l + 1].d_in, layers[l + 1].d_out);
            if (next.escape && next.alt_kind == kI8) a.clear_flag = flags + l + 1;
        }
        a.layout = layout;
        a.alpha = L.alpha;
        a.d_out = L.d_out;
        a.w_bits = L.w_bits;
        a.w_ld_words = L.ld_words;
        a.d_in = L.d_in;
        if (own_term) {
            a.self_rows = self_rows;
            a.self_alpha = L.alpha_self;
            a.self_w_bits = L.w_self_bits;
        }
        if (l == n_layers - 1) {
            a.logits = logits;
            a.ld_logits = ld_logits;
        } else {
            words = (L.d_out + 63) / 64;
            in_bits = bits;
            a.next_shift = layers[l + 1].bn_shift;
            a.next_mul = layers[l + 1].bn_mul;
            a.next_bits = bits;
            a.next_ld_words = words;
            a.next_scale = scale[(l + 1) & 1];
            a.next_row_mul = src_row_mul;
            a.next_fold_last_sign = choose_layout(layers[l + 1].d_in, layers[l + 1].d_out).fold_last;
        }
        rc = launch_fused_spmm(a, s);
        if (rc != BIGCN_OK) return rc;
        BIGCN_MARK();
    }
#undef BIGCN_MARK
    // the call counts only once every one of its events was recorded: a launch that failed half
    // way leaves no slot whose events bigcn_profile_read would wait for in vain
    if (prof != nullptr) prof->calls++;
    return BIGCN_OK;
}

static int gcn_forward(const bigcn_plan *plan, const int64_t *row_ptr, const int32_t *col_idx,
                       const float *dinv_sqrt, int64_t n, const float *x, int64_t ld_x,
                       const bigcn_layer *layers, int n_layers, float *logits, int64_t ld_logits,
                       void *workspace, size_t workspace_bytes, void *stream, bigcn_profile *prof)
{
    LayerView view[kMaxLayers];
    const int rc = view_gcn(layers, n_layers, view);
    if (rc != BIGCN_OK) return rc;
    return forward_impl(plan, row_ptr, col_idx, dinv_sqrt, dinv_sqrt, false, n, x, ld_x, PackedInput{}, view,
                        n_layers, logits, ld_logits, workspace, workspace_bytes, stream, prof);
}

static int sage_forward(const bigcn_plan *plan, const int64_t *row_ptr, const int32_t *col_idx,
                        const float *inv_deg, int64_t n, const float *x, int64_t ld_x,
                        const bigcn_sage_layer *layers, int n_layers, float *out, int64_t ld_out,
                        void *workspace, size_t workspace_bytes, void *stream, bigcn_profile *prof)
{
    LayerView view[kMaxLayers];
    const int rc = view_sage(layers, n_layers, view);
    if (rc != BIGCN_OK) return rc;
    return forward_impl(plan, row_ptr, col_idx, inv_deg, nullptr, true, n, x, ld_x, PackedInput{}, view, n_layers,
                        out, ld_out, workspace, workspace_bytes, stream, prof);
}

extern "C" int bigcn_forward(const bigcn_plan *plan, const int64_t *row_ptr, const int32_t *col_idx,
                             const float *dinv_sqrt, int64_t n, const float *x, int64_t ld_x,
                             const bigcn_layer *layers, int n_layers, float *logits,
                             int64_t ld_logits, void *workspace, size_t workspace_bytes, void *stream)
{
    return gcn_forward(plan, row_ptr, col_idx, dinv_sqrt, n, x, ld_x, layers, n_layers, logits,
                       ld_logits, workspace, workspace_bytes, stream, nullptr);
}

extern "C" int bigcn_forward_static(const bigcn_plan *plan, const int64_t *row_ptr, const int32_t *col_idx,
                                    const float *dinv_sqrt, int64_t n, const float *x, int64_t ld_x,
                                    const bigcn_layer *layers, int n_layers, float *logits,
                                    int64_t ld_logits, void *stream)
{
    LayerView view[kMaxLayers];
    int status = view_gcn(layers, n_layers, view);
    if (status != BIGCN_OK) return status;
    if (!layers_ok(n, view, n_layers, false, &status)) return status;
    if (map_workspace(n, view, n_layers, false).total > BIGCN_STATIC_WORKSPACE_BYTES) return BIGCN_ESHAPE;
    void *workspace = nullptr;
    status = static_workspace(&workspace);
    if (status != BIGCN_OK) return status;
    return forward_impl(plan, row_ptr, col_idx, dinv_sqrt, dinv_sqrt, false, n, x, ld_x, PackedInput{}, view,
                        n_layers, logits, ld_logits, workspace, BIGCN_STATIC_WORKSPACE_BYTES, stream, nullptr);
}

extern "C" int bigcn_forward_packed(const bigcn_plan *plan, const int64_t *row_ptr, const int32_t *col_idx,
                                    const float *dinv_sqrt, int64_t n, const uint64_t *x_bits,
                                    int64_t ld_x_words, const float *x_beta, const bigcn_layer *layers,
                                    int n_layers, float *logits, int64_t ld_logits, void *workspace,
                                    size_t workspace_bytes, void *stream)
{
    if (x_bits == nullptr || x_beta == nullptr) return BIGCN_ENULL;
    LayerView view[kMaxLayers];
    const int rc = view_gcn(layers, n_layers, view);
    if (rc != BIGCN_OK) return rc;
    return forward_impl(plan, row_ptr, col_idx, dinv_sqrt, dinv_sqrt, false, n, nullptr, 0,
                        PackedInput{x_bits, ld_x_words, x_beta}, view, n_layers, logits, ld_logits, workspace,
                        workspace_bytes, stream, nullptr);
}

extern "C" int bigcn_forward_profiled(const bigcn_plan *plan, const int64_t *row_ptr,
                                      const int32_t *col_idx, const float *dinv_sqrt, int64_t n,
                                      const float *x, int64_t ld_x, const bigcn_layer *layers,
                                      int n_layers, float *logits, int64_t ld_logits, void *workspace,
                                      size_t workspace_bytes, void *stream, bigcn_profile *profile)
{
    if (profile == nullptr) return BIGCN_ENULL;
    return gcn_forward(plan, row_ptr, col_idx, dinv_sqrt, n, x, ld_x, layers, n_layers, logits,
                       ld_logits, workspace, workspace_bytes, stream, profile);
}

extern "C" int bigcn_sage_forward(const bigcn_plan *plan, const int64_t *row_ptr, const int32_t *col_idx,
                                  const float *inv_deg, int64_t n, const float *x, int64_t ld_x,
                                  const bigcn_sage_layer *layers, int n_layers, float *out,
                                  int64_t ld_out, void *workspace, size_t workspace_bytes, void *stream)
{
    return sage_forward(plan, row_ptr, col_idx, inv_deg, n, x, ld_x, layers, n_layers, out, ld_out,
                        workspace, workspace_bytes, stream, nullptr);
}

extern "C" int bigcn_sage_forward_profiled(const bigcn_plan *plan, const int64_t *row_ptr,
                                           const int32_t *col_idx, const float *inv_deg, int64_t n,
                                           const float *x, int64_t ld_x, const bigcn_sage_layer *layers,
                                           int n_layers, float *out, int64_t ld_out, void *workspace,
                                           size_t workspace_bytes, void *stream, bigcn_profile *profile)
{
    if (profile == nullptr) return BIGCN_ENULL;
    return sage_forward(plan, row_ptr, col_idx, inv_deg, n, x, ld_x, layers, n_layers, out, ld_out,
                        workspace, workspace_bytes, stream, profile);
}

extern "C" int bigcn_profile_create(int n_layers, int max_calls, bigcn_profile **out)
{
    if (out == nullptr) return BIGCN_ENULL;
    if (n_layers <= 0 || max_calls <= 0 || max_calls > 4096) return BIGCN_EINVAL;
    bigcn_profile *p = new (std::nothrow) bigcn_profile();
    if (p == nullptr) return BIGCN_EHIP;
    p->n_layers = n_layers;
    p->max_calls = max_calls;
    p->calls = 0;
    const size_t count = static_cast<size_t>(max_calls) * p->per_call();
    p->events = new (std::nothrow) hipEvent_t[count];
    if (p->events == nullptr) { delete p; return BIGCN_EHIP; }
    for (size_t i = 0; i < count; ++i) {
        if (hipEventCreate(&p->events[i]) != hipSuccess) {
            for (size_t j = 0; j < i; ++j) (void)hipEventDestroy(p->events[j]);
            delete[] p->events;
            delete p;
            return BIGCN_EHIP;
        }
    }
    *out = p;
    return BIGCN_OK;
}

extern "C" void bigcn_profile_destroy(bigcn_profile *profile)
{
    if (profile == nullptr) return;
    const size_t count = static_cast<size_t>(profile->max_calls) * profile->per_call();
    for (size_t i = 0; i < count; ++i) (void)hipEventDestroy(profile->events[i]);
    delete[] profile->events;
    delete profile;
}

extern "C" int bigcn_profile_read(bigcn_profile *profile, float *launch_ms, int *calls)
{
    if (profile == nullptr || launch_ms == nullptr) return BIGCN_ENULL;
    const int slots = 1 + 2 * profile->n_layers;
    for (int k = 0; k < slots; ++k) launch_ms[k] = 0.0f;
    const int recorded = profile->calls;
    profile->calls = 0;                      // also on the error returns below: the profile stays usable
    for (int c = 0; c < recorded; ++c) {
        hipEvent_t *ev = profile->events + static_cast<size_t>(c) * profile->per_call();
        if (hipEventSynchronize(ev[slots]) != hipSuccess) return BIGCN_EHIP;
        for (int k = 0; k < slots; ++k) {
            float ms = 0.0f;
            if (hipEventElapsedTime(&ms, ev[k], ev[k + 1]) != hipSuccess) return BIGCN_EHIP;
            launch_ms[k] += ms;
        }
    }
    if (recorded > 0)
        for (int k = 0; k < slots; ++k) launch_ms[k] /= static_cast<float>(recorded);
    if (calls != nullptr) *calls = recorded;
    return BIGCN_OK;
}
