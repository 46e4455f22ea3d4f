// Plan (layout tables), host-side size queries, the bit rule and status strings.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <new>
#include <vector>

#include "dq_internal.h"

namespace {

int64_t padded_len(int64_t len) { return (len + DQ_GRANULE - 1) / DQ_GRANULE * DQ_GRANULE; }

template <typename T>
bool upload(T** dst, const std::vector<T>& src)
{
    *dst = nullptr;
    const size_t bytes = (src.empty() ? 1 : src.size()) * sizeof(T);
    if (hipMalloc(reinterpret_cast<void**>(dst), bytes) != hipSuccess) return false;
    if (!src.empty() &&
        hipMemcpy(*dst, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice) != hipSuccess)
        return false;
    return true;
}

void free_device_tables(dq_plan* p)
{
    if (p->d_granule_cseg) (void)hipFree(p->d_granule_cseg);
    if (p->d_cseg_seg) (void)hipFree(p->d_cseg_seg);
    if (p->d_cseg_valid_end) (void)hipFree(p->d_cseg_valid_end);
    if (p->d_cseg_start) (void)hipFree(p->d_cseg_start);
    if (p->d_span_cseg) (void)hipFree(p->d_span_cseg);
    if (p->d_items) (void)hipFree(p->d_items);
    if (p->d_seg_item_begin) (void)hipFree(p->d_seg_item_begin);
    if (p->d_finish_seg) (void)hipFree(p->d_finish_seg);
    p->d_finish_seg = nullptr;
    p->d_granule_cseg = nullptr;
    p->d_cseg_seg = nullptr;
    p->d_cseg_valid_end = nullptr;
    p->d_cseg_start = nullptr;
    p->d_span_cseg = nullptr;
    p->d_items = nullptr;
    p->d_seg_item_begin = nullptr;
}

} // namespace

extern "C" int dq_plan_create(const int64_t* seg_len_host, int32_t n_seg, dq_plan_t** plan_out)
{
    if (!plan_out) return DQ_ERR_INVALID_ARG;
    *plan_out = nullptr;
    if (!seg_len_host || n_seg < 1 || n_seg == INT32_MAX) return DQ_ERR_INVALID_ARG; // tables hold n_seg + 1 entries
    int64_t total = 0;
    for (int32_t l = 0; l < n_seg; ++l) {
        if (seg_len_host[l] < 0 || seg_len_host[l] > (INT64_C(1) << 40)) return DQ_ERR_INVALID_ARG;
        total += padded_len(seg_len_host[l]);
        if (total > (INT64_C(1) << 40)) return DQ_ERR_INVALID_ARG;
    }

    dq_plan* p = new (std::nothrow) dq_plan();
    if (!p) return DQ_ERR_ALLOC;
    memset(p, 0, sizeof(*p));
    p->n_seg = n_seg;
    p->padded_elems = total;
    p->device = -1;
    p->seg_len = static_cast<int64_t*>(malloc(sizeof(int64_t) * n_seg));
    p->seg_start = static_cast<int64_t*>(malloc(sizeof(int64_t) * (n_seg + 1)));
    if (!p->seg_len || !p->seg_start) {
        dq_plan_destroy(p);
        return DQ_ERR_ALLOC;
    }
    int64_t n_items = 0;
    p->seg_start[0] = 0;
    p->chunk_local = true;
    for (int32_t l = 0; l < n_seg; ++l) {
        p->seg_len[l] = seg_len_host[l];
        p->seg_start[l + 1] = p->seg_start[l] + padded_len(seg_len_host[l]);
        if (seg_len_host[l] > 0 && p->seg_start[l] / 4096 != (p->seg_start[l + 1] - 1) / 4096) p->chunk_local = false;
        n_items += (seg_len_host[l] + DQ_NORM_CHUNK - 1) / DQ_NORM_CHUNK;
    }
    if (n_items > INT32_MAX) {
        dq_plan_destroy(p);
        return DQ_ERR_INVALID_ARG;
    }
    p->n_items = static_cast<int32_t>(n_items);

    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) != hipSuccess || n_dev < 1) {
        (void)hipGetLastError(); // host-only plan: size queries work, launches return DQ_ERR_HIP
        *plan_out = p;
        return DQ_OK;
    }
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        dq_plan_destroy(p);
        return DQ_ERR_HIP;
    }

    std::vector<int64_t> cseg_valid_end;
    std::vector<int64_t> cseg_start;
    std::vector<int32_t> span_cseg;
    std::vector<int32_t> cseg_seg;
    std::vector<int32_t> granule_cseg;
    std::vector<dq_norm_item> items;
    std::vector<int32_t> item_begin;
    std::vector<int32_t> finish_seg;
    try {
        // every allocation of the host tables happens in here: std::bad_alloc never leaves the call
        granule_cseg.resize(static_cast<size_t>(total / DQ_GRANULE));
        item_begin.resize(static_cast<size_t>(n_seg) + 1);
        items.reserve(static_cast<size_t>(n_items));
        for (int32_t l = 0; l < n_seg; ++l) {
            if (p->seg_len[l] > 0) {
                const int32_t c = static_cast<int32_t>(cseg_seg.size());
                cseg_seg.push_back(l);
                cseg_valid_end.push_back(p->seg_start[l] + p->seg_len[l]);
                cseg_start.push_back(p->seg_start[l]);
                if (p->seg_start[l] / 4096 != (p->seg_start[l] + p->seg_len[l] - 1) / 4096) span_cseg.push_back(c);
                for (int64_t g = p->seg_start[l] / DQ_GRANULE; g < p->seg_start[l + 1] / DQ_GRANULE; ++g)
                    granule_cseg[static_cast<size_t>(g)] = c;
            }
            item_begin[l] = static_cast<int32_t>(items.size());
            for (int64_t off = 0; off < p->seg_len[l]; off += DQ_NORM_CHUNK) {
                dq_norm_item it;
                it.start = p->seg_start[l] + off;
                const int64_t left = p->seg_len[l] - off;
                it.count = static_cast<int32_t>(left < DQ_NORM_CHUNK ? left : DQ_NORM_CHUNK);
                it.seg = l;
                items.push_back(it);
            }
        }
        item_begin[n_seg] = static_cast<int32_t>(items.size());
        for (int32_t l = 0; l < n_seg; ++l)
            if (item_begin[l + 1] - item_begin[l] != 1) finish_seg.push_back(l);
    } catch (const std::bad_alloc&) {
        dq_plan_destroy(p);
        return DQ_ERR_ALLOC;
    }

    const bool ok = upload(&p->d_granule_cseg, granule_cseg) && upload(&p->d_cseg_seg, cseg_seg) &&
                    upload(&p->d_cseg_valid_end, cseg_valid_end) && upload(&p->d_cseg_start, cseg_start) && upload(&p->d_span_cseg, span_cseg) &&
                    upload(&p->d_items, items) && upload(&p->d_seg_item_begin, item_begin) &&
                    upload(&p->d_finish_seg, finish_seg);
    if (!ok) {
        (void)hipGetLastError();
        free_device_tables(p);
        dq_plan_destroy(p);
        return DQ_ERR_ALLOC;
    }
    p->device = dev;
    dq_norm_static_scratch_prepare(dev); // set-up time: the allocation-free entry point then only launches
    p->n_cseg = static_cast<int32_t>(cseg_seg.size());
    p->n_finish = static_cast<int32_t>(finish_seg.size());
    p->n_span = static_cast<int32_t>(span_cseg.size());
    *plan_out = p;
    return DQ_OK;
}

extern "C" void dq_plan_destroy(dq_plan_t* plan)
{
    if (!plan) return;
    if (plan->device >= 0) {
        int cur = 0;
        const bool have_cur = hipGetDevice(&cur) == hipSuccess;
        if (hipSetDevice(plan->device) == hipSuccess) free_device_tables(plan);
        if (have_cur) (void)hipSetDevice(cur);
    }
    free(plan->seg_len);
    free(plan->seg_start);
    delete plan;
}

extern "C" int32_t dq_plan_num_segments(const dq_plan_t* plan) { return plan ? plan->n_seg : -1; }

extern "C" int64_t dq_plan_padded_elems(const dq_plan_t* plan) { return plan ? plan->padded_elems : -1; }

extern "C" int64_t dq_plan_segment_start(const dq_plan_t* plan, int32_t l)
{
    if (!plan || l < 0 || l >= plan->n_seg) return -1;
    return plan->seg_start[l];
}

extern "C" int64_t dq_packed_bytes(const dq_plan_t* plan, int b)
{
    if (!plan || b < 1 || b > 8) return -1;
    return plan->padded_elems / 8 + plan->padded_elems * b / 8;
}

extern "C" int64_t dq_workspace_bytes(const dq_plan_t* plan, int M)
{
    if (!plan || M < 1 || M > DQ_MAX_WORKERS) return -1;
    const int64_t partials = static_cast<int64_t>(M) * plan->n_items * static_cast<int64_t>(sizeof(double));
    return partials < 16 ? 16 : (partials + 15) / 16 * 16;
}

extern "C" int dq_plan_is_chunk_local(const dq_plan_t* plan) { return plan && plan->chunk_local ? 1 : 0; }

extern "C" int dq_plan_has_device(const dq_plan_t* plan) { return plan && plan->device >= 0 ? 1 : 0; }

int dq_plan_check_device(const dq_plan* plan)
{
    if (!plan) return DQ_ERR_INVALID_ARG;
    if (plan->device < 0) return DQ_ERR_HIP;
    int cur = -1;
    if (hipGetDevice(&cur) != hipSuccess) return DQ_ERR_HIP;
    if (cur != plan->device && hipSetDevice(plan->device) != hipSuccess) return DQ_ERR_HIP;
    return DQ_OK;
}

// Eq. (17) with b = b_paper - 1, rounded up: the smallest b whose 2^b - 1 levels reach s*.
// G-bar^2 is the mean over workers of the squared whole-gradient norm: the sum of the squared
// segment norms for p = 2, the square of the largest segment norm for p = infinity.
static int select_bits(bool linf, const float* norms_host, int M, int n_seg, int64_t t, int64_t T,
                       double eps_hat_q, double alpha, int b_min, int b_max, int* b_out, double* gbar_out)
{
    if (!norms_host || !b_out || M < 1 || n_seg < 1) return DQ_ERR_INVALID_ARG;
    if (T < 1 || t < 0 || t >= T) return DQ_ERR_INVALID_ARG;
    if (!(eps_hat_q > 0.0) || !(alpha > 0.0) || !(alpha <= 1.0)) return DQ_ERR_INVALID_ARG;
    if (b_min < 1 || b_max > 8 || b_min > b_max) return DQ_ERR_INVALID_ARG;
    double sum_sq = 0.0;
    for (int i = 0; i < M; ++i) {
        const float* row = norms_host + static_cast<int64_t>(i) * n_seg;
        double worker_sq = 0.0;
        if (linf) {
            for (int l = 0; l < n_seg; ++l) {
                const double sq = static_cast<double>(row[l]) * static_cast<double>(row[l]);
                worker_sq = sq > worker_sq ? sq : worker_sq;
            }
        } else {
            worker_sq = dq_worker_squared_norm(row, n_seg);
        }
        sum_sq += worker_sq;
    }
    const double gbar = sqrt(sum_sq / static_cast<double>(M));
    const double weight = pow(alpha, static_cast<double>(T - 1 - t) / 2.0);
    const double s_star = sqrt(static_cast<double>(T) / eps_hat_q) * weight * gbar;
    int b = b_max;
    for (int cand = b_min; cand <= b_max; ++cand) {
        if (static_cast<double>((1 << cand) - 1) >= s_star) {
            b = cand;
            break;
        }
    }
    *b_out = b;
    if (gbar_out) *gbar_out = gbar;
    return DQ_OK;
}

extern "C" int dq_select_bits(const float* norms_host, int M, int n_seg, int64_t t, int64_t T,
                              double eps_hat_q, double alpha, int b_min, int b_max, int* b_out,
                              double* gbar_out)
{
    return select_bits(false, norms_host, M, n_seg, t, T, eps_hat_q, alpha, b_min, b_max, b_out, gbar_out);
}

extern "C" int dq_select_bits_linf(const float* norms_host, int M, int n_seg, int64_t t, int64_t T,
                                   double eps_hat_q, double alpha, int b_min, int b_max, int* b_out,
                                   double* gbar_out)
{
    return select_bits(true, norms_host, M, n_seg, t, T, eps_hat_q, alpha, b_min, b_max, b_out, gbar_out);
}

// Eq. (24): alpha_est = (F(x_t) / F(x_0))^(1/t).
extern "C" double dq_alpha_est(double F_t, double F_0, int64_t t)
{
    if (t < 1 || !(F_t > 0.0) || !(F_0 > 0.0)) return -1.0;
    return pow(F_t / F_0, 1.0 / static_cast<double>(t));
}

// Eq. (7), one iteration: W * (d * b_paper + n_norms * B_pre) with b_paper = b + 1.
extern "C" int64_t dq_comm_cost_bits(int W, int64_t d, int b, int32_t n_norms, int B_pre)
{
    if (W < 1 || d < 0 || b < 0 || b > 31 || n_norms < 0 || B_pre < 0) return -1;
    return static_cast<int64_t>(W) * (d * (b + 1) + static_cast<int64_t>(n_norms) * B_pre);
}

extern "C" const char* dq_status_string(int status)
{
    switch (status) {
    case DQ_OK: return "ok";
    case DQ_ERR_INVALID_ARG: return "invalid argument";
    case DQ_ERR_HIP: return "HIP runtime error or no GPU bound to the plan";
    case DQ_ERR_ALLOC: return "allocation failed";
    default: return "unknown status";
    }
}
