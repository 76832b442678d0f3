// Graph-side helpers: the coefficients of A~ = D^-1/2 (A+I) D^-1/2 (Sec. 3.1, Eq. (1)) and of
// the mean aggregator 1/|N_i| (Sec. 4.4.2), validation of the CSR pattern, and the aggregation
// plan (row order by decreasing length for the power-law degree distributions of the paper's
// graphs).
#include <algorithm>
#include <new>
#include <vector>

#include "bigcn_internal.h"

namespace bigcn {

__global__ __launch_bounds__(kBlock) void dinv_sqrt_kernel(const int64_t *__restrict__ row_ptr,
                                                           int64_t n, float *__restrict__ dinv)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i < n) {
        const float deg = static_cast<float>(row_ptr[i + 1] - row_ptr[i]);
        dinv[i] = 1.0f / sqrtf(deg);
    }
}

__global__ __launch_bounds__(kBlock) void inv_degree_kernel(const int64_t *__restrict__ row_ptr,
                                                            int64_t n, float *__restrict__ inv_deg)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i < n) {
        const int64_t deg = row_ptr[i + 1] - row_ptr[i];
        inv_deg[i] = deg > 0 ? 1.0f / static_cast<float>(deg) : 0.0f;
    }
}

// one wavefront per row: vals[p] = dinv[i] * dinv[col[p]]
__global__ __launch_bounds__(kBlock) void edge_norm_kernel(const int64_t *__restrict__ row_ptr,
                                                           const int32_t *__restrict__ col_idx,
                                                           int64_t n, const float *__restrict__ dinv,
                                                           float *__restrict__ vals)
{
    const int lane = lane_id();
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * kWavesPerBlock + wave_in_block();
    const int64_t n_waves = static_cast<int64_t>(gridDim.x) * kWavesPerBlock;
    for (int64_t i = wave; i < n; i += n_waves) {
        const float di = dinv[i];
        const int64_t p1 = row_ptr[i + 1];
        for (int64_t p = row_ptr[i] + lane; p < p1; p += kWave) vals[p] = di * dinv[col_idx[p]];
    }
}

// Pattern checks; any violation sets *flag (plain store of a non-zero value: races are benign).
// full_pattern: also require the self-loop and the symmetry of A + I.
__global__ __launch_bounds__(kBlock) void validate_kernel(const int64_t *__restrict__ row_ptr,
                                                          const int32_t *__restrict__ col_idx,
                                                          int64_t n, int full_pattern,
                                                          int *__restrict__ flag)
{
    const int lane = lane_id();
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * kWavesPerBlock + wave_in_block();
    const int64_t n_waves = static_cast<int64_t>(gridDim.x) * kWavesPerBlock;
    for (int64_t i = wave; i < n; i += n_waves) {
        const int64_t p0 = row_ptr[i], p1 = row_ptr[i + 1];
        bool has_loop = false;
        for (int64_t p = p0 + lane; p < p1; p += kWave) {
            const int64_t k = col_idx[p];
            if (k < 0 || k >= n) { *flag = 1; continue; }
            if (p > p0 && col_idx[p - 1] >= k) *flag = 2;          // not strictly increasing
            if (!full_pattern) continue;
            if (k == i) { has_loop = true; continue; }
            // symmetry: binary search for i in row k
            int64_t lo = row_ptr[k], hi = row_ptr[k + 1];
            bool found = false;
            while (lo < hi) {
                const int64_t mid = (lo + hi) >> 1;
                const int64_t c = col_idx[mid];
                if (c == i) { found = true; break; }
                if (c < i) lo = mid + 1; else hi = mid;
            }
            if (!found) *flag = 3;
        }
        if (full_pattern && __ballot(has_loop) == 0ull && lane == 0) *flag = 4;    // self-loop missing
    }
}

}  // namespace bigcn

using namespace bigcn;

extern "C" int bigcn_gcn_norm(const int64_t *row_ptr, const int32_t *col_idx, int64_t n,
                              float *dinv_sqrt, float *vals, void *stream)
{
    if (row_ptr == nullptr || dinv_sqrt == nullptr) return BIGCN_ENULL;
    if (vals != nullptr && col_idx == nullptr) return BIGCN_ENULL;
    if (n < 0) return BIGCN_EINVAL;
    if (n == 0) return BIGCN_OK;
    hipStream_t s = as_stream(stream);
    hipLaunchKernelGGL(dinv_sqrt_kernel, dim3(static_cast<unsigned>((n + kBlock - 1) / kBlock)),
                       dim3(kBlock), 0, s, row_ptr, n, dinv_sqrt);
    if (vals != nullptr) {
        int64_t blocks = (n + kWavesPerBlock - 1) / kWavesPerBlock;
        if (blocks > 256 * 32) blocks = 256 * 32;
        hipLaunchKernelGGL(edge_norm_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0, s,
                           row_ptr, col_idx, n, dinv_sqrt, vals);
    }
    return check_launch();
}

extern "C" int bigcn_mean_norm(const int64_t *row_ptr, int64_t n, float *inv_deg, void *stream)
{
    if (row_ptr == nullptr || inv_deg == nullptr) return BIGCN_ENULL;
    if (n < 0) return BIGCN_EINVAL;
    if (n == 0) return BIGCN_OK;
    hipLaunchKernelGGL(inv_degree_kernel, dim3(static_cast<unsigned>((n + kBlock - 1) / kBlock)),
                       dim3(kBlock), 0, as_stream(stream), row_ptr, n, inv_deg);
    return check_launch();
}

extern "C" int bigcn_plan_create(const int64_t *row_ptr, const int32_t *col_idx, int64_t n,
                                 int validate, bigcn_plan **out, void *stream)
{
    if (row_ptr == nullptr || col_idx == nullptr || out == nullptr) return BIGCN_ENULL;
    if (n < 0 || n >= (static_cast<int64_t>(1) << 31)) return BIGCN_EINVAL;
    if (validate != BIGCN_VALIDATE_NONE && validate != BIGCN_VALIDATE_GCN && validate != BIGCN_VALIDATE_NEIGHBOURS)
        return BIGCN_EINVAL;
    hipStream_t s = as_stream(stream);

    std::vector<int64_t> rp;
    try {
        rp.resize(static_cast<size_t>(n) + 1);
    } catch (const std::bad_alloc &) {
        return BIGCN_EHIP;
    }
    if (hipMemcpyAsync(rp.data(), row_ptr, sizeof(int64_t) * (n + 1), hipMemcpyDeviceToHost, s) != hipSuccess)
        return BIGCN_EHIP;
    if (hipStreamSynchronize(s) != hipSuccess) return BIGCN_EHIP;
    if (rp[0] != 0) return BIGCN_EINVAL;
    int64_t max_degree = 0;
    for (int64_t i = 0; i < n; ++i) {
        const int64_t d = rp[i + 1] - rp[i];
        if (d < 0) return BIGCN_EINVAL;
        max_degree = std::max(max_degree, d);
    }
    const int64_t nnz = rp[n];

    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) return BIGCN_EHIP;

    if (validate != 0 && n > 0) {
        int *flag = nullptr;
        if (hipMalloc(&flag, sizeof(int)) != hipSuccess) return BIGCN_EHIP;
        int host_flag = 0;
        bool ok = hipMemsetAsync(flag, 0, sizeof(int), s) == hipSuccess;
        if (ok) {
            int64_t blocks = (n + kWavesPerBlock - 1) / kWavesPerBlock;
            if (blocks > 256 * 32) blocks = 256 * 32;
            hipLaunchKernelGGL(validate_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0, s,
                               row_ptr, col_idx, n, validate == BIGCN_VALIDATE_GCN ? 1 : 0, flag);
            ok = hipGetLastError() == hipSuccess &&
                 hipMemcpyAsync(&host_flag, flag, sizeof(int), hipMemcpyDeviceToHost, s) == hipSuccess &&
                 hipStreamSynchronize(s) == hipSuccess;
        }
        (void)hipFree(flag);
        if (!ok) return BIGCN_EHIP;
        if (host_flag != 0) return BIGCN_EGRAPH;
    }

    // counting sort of the rows by decreasing degree (stable: ties keep increasing row id)
    std::vector<int32_t> order;
    std::vector<int64_t> start;
    try {
        order.resize(static_cast<size_t>(n));
        start.assign(static_cast<size_t>(max_degree) + 2, 0);
    } catch (const std::bad_alloc &) {
        return BIGCN_EHIP;
    }
    for (int64_t i = 0; i < n; ++i) start[static_cast<size_t>(max_degree - (rp[i + 1] - rp[i])) + 1]++;
    for (size_t d = 1; d < start.size(); ++d) start[d] += start[d - 1];
    int64_t n_block_rows = 0, n_split_rows = 0;
    for (int64_t i = 0; i < n; ++i) {
        const int64_t deg = rp[i + 1] - rp[i];
        order[static_cast<size_t>(start[static_cast<size_t>(max_degree - deg)]++)] = static_cast<int32_t>(i);
        if (deg >= kBlockRowDegree) ++n_block_rows;
        if (deg >= kSplitRowDegree) ++n_split_rows;
    }

    bigcn_plan *plan = new (std::nothrow) bigcn_plan();
    if (plan == nullptr) return BIGCN_EHIP;
    plan->n = n;
    plan->nnz = nnz;
    plan->device = device;
    if (hipDeviceGetAttribute(&plan->compute_units, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess ||
        plan->compute_units <= 0) {
        (void)hipGetLastError();
        plan->compute_units = 256;                       // MI355X
    }
    plan->row_order = nullptr;
    plan->entries = nullptr;
    plan->n_block_rows = n_block_rows;
    plan->n_split_rows = n_split_rows;
    plan->max_degree = max_degree;
    if (n > 0) {
        std::vector<bigcn_plan_entry> entries;
        try {
            entries.resize(static_cast<size_t>(n));
        } catch (const std::bad_alloc &) {
            delete plan;
            return BIGCN_EHIP;
        }
        for (int64_t e = 0; e < n; ++e) {
            const int32_t row = order[static_cast<size_t>(e)];
            entries[static_cast<size_t>(e)] = bigcn_plan_entry{rp[static_cast<size_t>(row)], row,
                                                        static_cast<int32_t>(rp[static_cast<size_t>(row) + 1] - rp[static_cast<size_t>(row)])};
        }
        if (hipMalloc(&plan->row_order, sizeof(int32_t) * n) != hipSuccess ||
            hipMalloc(&plan->entries, sizeof(bigcn_plan_entry) * n) != hipSuccess) {
            (void)hipGetLastError();
            if (plan->row_order != nullptr) (void)hipFree(plan->row_order);
            if (plan->entries != nullptr) (void)hipFree(plan->entries);
            delete plan;
            return BIGCN_EHIP;
        }
        if (hipMemcpyAsync(plan->row_order, order.data(), sizeof(int32_t) * n, hipMemcpyHostToDevice, s) != hipSuccess ||
            hipMemcpyAsync(plan->entries, entries.data(), sizeof(bigcn_plan_entry) * n, hipMemcpyHostToDevice, s) != hipSuccess ||
            hipStreamSynchronize(s) != hipSuccess) {
            (void)hipFree(plan->row_order);
            (void)hipFree(plan->entries);
            delete plan;
            return BIGCN_EHIP;
        }
    }
    *out = plan;
    return BIGCN_OK;
}

extern "C" void bigcn_plan_destroy(bigcn_plan *plan)
{
    if (plan == nullptr) return;
    if (plan->row_order != nullptr) (void)hipFree(plan->row_order);
    delete plan;
}

extern "C" int64_t bigcn_plan_rows(const bigcn_plan *plan) { return plan ? plan->n : -1; }
extern "C" int64_t bigcn_plan_nnz(const bigcn_plan *plan) { return plan ? plan->nnz : -1; }
