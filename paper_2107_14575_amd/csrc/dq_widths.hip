// Per-tensor bit-widths: the table that tells the kernels each tensor's level bits and where its
// level fields start in the message, the bit rule that fills it, and the cost accounting.
//
// Rule.  The paper's program (the one Eq. (17) solves, appendix "Proof of Eq. (17)") with one
// level count s_l per tensor: Lemma 1's variance bound of an iteration becomes
// sum_l d_l Nbar_l^2 / (4 s_l^2) with Nbar_l^2 = (1/M) sum_i N_{i,l}^2, the cost sum_l d_l b_l; the
// same Lagrangian steps give s_l proportional to alpha^((T-1-t)/2) Nbar_l (d_l cancels) and the
// constraint fixes the factor: s*_{t,l} = sqrt(T/eps_hat) alpha^((T-1-t)/2) Nbar_{t,l}.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <new>

#include "dq_internal.h"

namespace {

int64_t padded_len(int64_t len) { return (len + DQ_GRANULE - 1) / DQ_GRANULE * DQ_GRANULE; }

} // namespace

extern "C" int dq_select_bits_per_tensor(const float* norms_host, int M, int n_seg, int64_t t, int64_t T,
                                         double eps_hat_q, double alpha, int b_min, int b_max,
                                         int32_t* b_out_host, double* nbar_out_host)
{
    if (!norms_host || !b_out_host || M < 1 || n_seg < 1) return DQ_ERR_INVALID_ARG;
    if (T < 1 || t < 0 || t >= T) return DQ_ERR_INVALID_ARG;
    if (!(eps_hat_q > 0.0) || !(alpha > 0.0) || !(alpha <= 1.0)) return DQ_ERR_INVALID_ARG;
    if (b_min < 1 || b_max > 8 || b_min > b_max) return DQ_ERR_INVALID_ARG;
    const double factor = sqrt(static_cast<double>(T) / eps_hat_q) * pow(alpha, static_cast<double>(T - 1 - t) / 2.0);
    for (int l = 0; l < n_seg; ++l) {
        double sum_sq = 0.0;
        for (int i = 0; i < M; ++i) {
            const double n = static_cast<double>(norms_host[static_cast<int64_t>(i) * n_seg + l]);
            sum_sq += n * n;
        }
        const double nbar = sqrt(sum_sq / static_cast<double>(M));
        const double s_star = factor * nbar;
        int b = b_max;
        for (int cand = b_min; cand <= b_max; ++cand) {
            if (static_cast<double>((1 << cand) - 1) >= s_star) {
                b = cand;
                break;
            }
        }
        b_out_host[l] = b;
        if (nbar_out_host) nbar_out_host[l] = nbar;
    }
    return DQ_OK;
}

extern "C" int64_t dq_comm_cost_bits_per_tensor(int W, const int64_t* seg_len_host, const int32_t* b_host,
                                                int32_t n_seg, int B_pre)
{
    if (W < 1 || !seg_len_host || !b_host || n_seg < 1 || B_pre < 0) return -1;
    int64_t bits = 0;
    for (int32_t l = 0; l < n_seg; ++l) {
        if (seg_len_host[l] < 0 || b_host[l] < 1 || b_host[l] > 8) return -1;
        bits += seg_len_host[l] * static_cast<int64_t>(b_host[l] + 1) + B_pre;
    }
    return static_cast<int64_t>(W) * bits;
}

extern "C" int64_t dq_packed_bytes_v(const dq_plan_t* plan, const int32_t* b_host)
{
    if (!plan || !b_host) return -1;
    int64_t bytes = plan->padded_elems / 8;
    for (int32_t l = 0; l < plan->n_seg; ++l) {
        if (b_host[l] < 1 || b_host[l] > 8) return -1;
        bytes += padded_len(plan->seg_len[l]) / 8 * b_host[l];
    }
    return bytes;
}

extern "C" int dq_widths_create(const dq_plan_t* plan, dq_widths_t** widths_out)
{
    if (!widths_out) return DQ_ERR_INVALID_ARG;
    *widths_out = nullptr;
    if (!plan) return DQ_ERR_INVALID_ARG;
    const int rc = dq_plan_check_device(plan);
    if (rc != DQ_OK) return rc;
    dq_widths* w = new (std::nothrow) dq_widths();
    if (!w) return DQ_ERR_ALLOC;
    memset(w, 0, sizeof(*w));
    w->plan = plan;
    w->packed_bytes = -1;
    const size_t bytes = sizeof(dq_cseg_width) * static_cast<size_t>(plan->n_cseg > 0 ? plan->n_cseg : 1);
    w->b_host = static_cast<int32_t*>(malloc(sizeof(int32_t) * plan->n_seg));
    bool ok = w->b_host != nullptr;
    ok = ok && hipMalloc(reinterpret_cast<void**>(&w->d_table), bytes) == hipSuccess;
    ok = ok && hipHostMalloc(reinterpret_cast<void**>(&w->h_stage), bytes, hipHostMallocDefault) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&w->uploaded, hipEventDisableTiming) == hipSuccess;
    if (!ok) {
        (void)hipGetLastError();
        dq_widths_destroy(w);
        return DQ_ERR_ALLOC;
    }
    *widths_out = w;
    return DQ_OK;
}

extern "C" void dq_widths_destroy(dq_widths_t* w)
{
    if (!w) return;
    int cur = 0;
    const bool have_cur = hipGetDevice(&cur) == hipSuccess;
    if (w->plan && w->plan->device >= 0 && hipSetDevice(w->plan->device) == hipSuccess) {
        if (w->uploaded) {
            (void)hipEventSynchronize(w->uploaded);
            (void)hipEventDestroy(w->uploaded);
        }
        if (w->d_table) (void)hipFree(w->d_table);
        if (w->h_stage) (void)hipHostFree(w->h_stage);
    }
    if (have_cur) (void)hipSetDevice(cur);
    free(w->b_host);
    delete w;
}

extern "C" int dq_widths_set(dq_widths_t* w, const int32_t* b_host, void* hip_stream)
{
    if (!w || !b_host) return DQ_ERR_INVALID_ARG;
    const dq_plan* plan = w->plan;
    for (int32_t l = 0; l < plan->n_seg; ++l)
        if (b_host[l] < 1 || b_host[l] > 8) return DQ_ERR_INVALID_ARG;
    const int rc = dq_plan_check_device(plan);
    if (rc != DQ_OK) return rc;
    // the previous upload must have left the staging buffer before it is overwritten
    if (w->packed_bytes >= 0 && hipEventSynchronize(w->uploaded) != hipSuccess) return DQ_ERR_HIP;
    int64_t level_bytes = 0;
    int32_t c = 0;
    for (int32_t l = 0; l < plan->n_seg; ++l) {
        if (plan->seg_len[l] == 0) continue;
        dq_cseg_width& e = w->h_stage[c++];
        e.level_start = level_bytes;
        e.seg_start = plan->seg_start[l];
        e.b = b_host[l];
        e.reserved = 0;
        level_bytes += padded_len(plan->seg_len[l]) / 8 * b_host[l];
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (c > 0 && hipMemcpyAsync(w->d_table, w->h_stage, sizeof(dq_cseg_width) * static_cast<size_t>(c),
                                hipMemcpyHostToDevice, stream) != hipSuccess)
        return DQ_ERR_HIP;
    if (hipEventRecord(w->uploaded, stream) != hipSuccess) return DQ_ERR_HIP;
    memcpy(w->b_host, b_host, sizeof(int32_t) * plan->n_seg);
    w->packed_bytes = plan->padded_elems / 8 + level_bytes;
    return DQ_OK;
}

extern "C" int64_t dq_widths_packed_bytes(const dq_widths_t* w) { return w ? w->packed_bytes : -1; }
