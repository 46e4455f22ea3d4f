// Per-tensor bit-widths: the table that tells the kernels each tensor's level bits and where its
// level fields start in the message (one row shared by the workers, or one row per worker), the
// bit rules that fill it -- on the host, or on the GPU without a round trip -- and the cost
// accounting.
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

constexpr int SB_THREADS = 256;

__device__ __forceinline__ int smallest_width(double s_star, int b_min, int b_max)
{
    int b = b_max;
    for (int cand = b_max; cand >= b_min; --cand) // same result as the ascending search: the levels grow with cand
        if (static_cast<double>((1 << cand) - 1) >= s_star) b = cand;
    return b;
}

// The bit rules on the device, in the arithmetic of the host functions (binary64, a worker's or a
// tensor's squares added in index order; products of binary32 norms are exact), so that a step
// needs no round trip to the host: one workgroup reads the M x n_seg norms, decides the widths,
// and fills the widths table (b and, by a scan over the tensors, where each tensor's level bytes
// start).  rule: 0 = Eq. (17) with the l2 norms, 1 = with max norms, 2 = one width per tensor.
__global__ __launch_bounds__(SB_THREADS) void k_select_bits(
    const float* __restrict__ norms, int M, int32_t n_seg, int32_t n_cseg, const int32_t* __restrict__ cseg_seg,
    const int64_t* __restrict__ cseg_valid_end, dq_cseg_width* __restrict__ table, int rule, double root_T_eps,
    double weight, int b_min, int b_max, int64_t sign_bytes, int32_t* __restrict__ b_out,
    double* __restrict__ gbar_out, int64_t* __restrict__ packed_bytes_out)
{
    __shared__ double worker_sq[DQ_MAX_WORKERS];
    __shared__ int b_all;
    __shared__ int64_t scan[SB_THREADS];
    __shared__ int64_t carry;
    const int tid = threadIdx.x;
    const double factor = root_T_eps * weight;

    if (rule != 2) {
        if (tid < M) {
            const float* row = norms + static_cast<int64_t>(tid) * n_seg;
            double acc = 0.0;
            for (int32_t l = 0; l < n_seg; ++l) {
                const double sq = static_cast<double>(row[l]) * static_cast<double>(row[l]);
                if (rule == 1)
                    acc = sq > acc ? sq : acc;
                else
                    acc += sq;
            }
            worker_sq[tid] = acc;
        }
        __syncthreads();
        if (tid == 0) {
            double sum_sq = 0.0;
            for (int i = 0; i < M; ++i) sum_sq += worker_sq[i];
            const double gbar = sqrt(sum_sq / static_cast<double>(M));
            b_all = smallest_width(factor * gbar, b_min, b_max);
            if (gbar_out) gbar_out[0] = gbar;
        }
        __syncthreads();
        const int b = b_all;
        if (b_out)
            for (int32_t l = tid; l < n_seg; l += SB_THREADS) b_out[l] = b;
        for (int32_t c = tid; c < n_cseg; c += SB_THREADS) table[c].b = b;
    } else {
        auto tensor_width = [&](int32_t l, double* nbar_out) {
            double acc = 0.0;
            for (int i = 0; i < M; ++i) {
                const double n = static_cast<double>(norms[static_cast<int64_t>(i) * n_seg + l]);
                acc += n * n;
            }
            const double nbar = sqrt(acc / static_cast<double>(M));
            if (nbar_out) *nbar_out = nbar;
            return smallest_width(factor * nbar, b_min, b_max);
        };
        if (b_out || gbar_out)
            for (int32_t l = tid; l < n_seg; l += SB_THREADS) {
                const int b = tensor_width(l, gbar_out ? gbar_out + l : nullptr);
                if (b_out) b_out[l] = b;
            }
        for (int32_t c = tid; c < n_cseg; c += SB_THREADS) table[c].b = tensor_width(cseg_seg[c], nullptr);
    }
    if (tid == 0) carry = 0;
    __syncthreads();

    // exclusive scan of the tensors' level bytes, 256 tensors per round; thread tid reads back the
    // width it wrote itself
    for (int32_t base = 0; base < n_cseg; base += SB_THREADS) {
        const int32_t c = base + tid;
        int64_t mine = 0;
        if (c < n_cseg) {
            const int64_t len = cseg_valid_end[c] - table[c].seg_start;
            mine = (len + DQ_GRANULE - 1) / DQ_GRANULE * (DQ_GRANULE / 8) * table[c].b;
        }
        scan[tid] = mine;
        __syncthreads();
        for (int off = 1; off < SB_THREADS; off <<= 1) {
            const int64_t add = tid >= off ? scan[tid - off] : 0;
            __syncthreads();
            scan[tid] += add;
            __syncthreads();
        }
        if (c < n_cseg) table[c].level_start = carry + scan[tid] - mine;
        __syncthreads();
        if (tid == 0) carry += scan[SB_THREADS - 1];
        __syncthreads();
    }
    if (tid == 0 && packed_bytes_out) *packed_bytes_out = sign_bytes + carry;
}

// ---------------------------------------------------------------------------------------------
// The same rules for plans with many tensors (a bucketed gradient has tens of thousands), split
// over several launches so that no single workgroup walks the whole table.  Every sum keeps the
// order of the one-workgroup kernel, so the widths are the same.
// ---------------------------------------------------------------------------------------------
// grid = M: worker i's squared whole-gradient norm (or squared max norm).  Lane j adds blocks j,
// j + 256, ... of DQ_SUM_BLOCK tensors, each in index order; lane 0 then adds the block sums in
// index order -- the order of dq_worker_squared_norm.  (A maximum needs no order.)
__global__ __launch_bounds__(SB_THREADS) void k_rule_worker_sums(const float* __restrict__ norms, int32_t n_seg,
                                                                 int linf, double* __restrict__ worker_sq,
                                                                 double* __restrict__ block_sums)
{
    const int tid = threadIdx.x;
    const float* row = norms + static_cast<int64_t>(blockIdx.x) * n_seg;
    const int32_t n_blocks = (n_seg - 1) / DQ_SUM_BLOCK + 1;
    double* mine = block_sums + static_cast<int64_t>(blockIdx.x) * n_blocks;
    for (int32_t blk = tid; blk < n_blocks; blk += SB_THREADS) {
        const int32_t begin = blk * DQ_SUM_BLOCK;
        const int32_t end = begin + DQ_SUM_BLOCK < n_seg ? begin + DQ_SUM_BLOCK : n_seg;
        double acc = 0.0;
        int32_t l = begin;
        for (; l + 16 <= end; l += 16) { // sixteen loads in flight, then the adds in index order
            double sq[16];
#pragma unroll
            for (int j = 0; j < 16; ++j) sq[j] = static_cast<double>(row[l + j]) * static_cast<double>(row[l + j]);
#pragma unroll
            for (int j = 0; j < 16; ++j) acc = linf ? (sq[j] > acc ? sq[j] : acc) : acc + sq[j];
        }
        for (; l < end; ++l) {
            const double sq = static_cast<double>(row[l]) * static_cast<double>(row[l]);
            acc = linf ? (sq > acc ? sq : acc) : acc + sq;
        }
        mine[blk] = acc;
    }
    __syncthreads(); // the block sums written above are read below by lane 0 of the same workgroup
    if (tid == 0) {
        double total = 0.0;
        for (int32_t blk = 0; blk < n_blocks; ++blk) total = linf ? (mine[blk] > total ? mine[blk] : total) : total + mine[blk];
        worker_sq[blockIdx.x] = total;
    }
}

// grid over max(n_seg, n_cseg): rules 0/1 -- every lane repeats the short sum over the M workers
// and the search for b, then writes its tensor's and its table entry's width.
__global__ __launch_bounds__(SB_THREADS) void k_rule_apply_single(
    const double* __restrict__ worker_sq, int M, int32_t n_seg, int32_t n_cseg, dq_cseg_width* __restrict__ table,
    double factor, int b_min, int b_max, int32_t* __restrict__ b_out, double* __restrict__ gbar_out)
{
    double sum_sq = 0.0;
    for (int i = 0; i < M; ++i) sum_sq += worker_sq[i];
    const double gbar = sqrt(sum_sq / static_cast<double>(M));
    const int b = smallest_width(factor * gbar, b_min, b_max);
    const int64_t t = static_cast<int64_t>(blockIdx.x) * SB_THREADS + threadIdx.x;
    if (t == 0 && gbar_out) gbar_out[0] = gbar;
    if (b_out && t < n_seg) b_out[t] = b;
    if (t < n_cseg) table[t].b = b;
}

// grid over max(n_seg, n_cseg): rule 2 -- lane t decides tensor t's width for the outputs and
// table entry t's width for the kernels.
__global__ __launch_bounds__(SB_THREADS) void k_rule_tensor_widths(
    const float* __restrict__ norms, int M, int32_t n_seg, int32_t n_cseg, const int32_t* __restrict__ cseg_seg,
    dq_cseg_width* __restrict__ table, double factor, int b_min, int b_max, int32_t* __restrict__ b_out,
    double* __restrict__ nbar_out)
{
    auto tensor_width = [&](int32_t l, double* nbar_dst) {
        double acc = 0.0;
        for (int i = 0; i < M; ++i) {
            const double n = static_cast<double>(norms[static_cast<int64_t>(i) * n_seg + l]);
            acc += n * n;
        }
        const double nbar = sqrt(acc / static_cast<double>(M));
        if (nbar_dst) *nbar_dst = nbar;
        return smallest_width(factor * nbar, b_min, b_max);
    };
    const int64_t t = static_cast<int64_t>(blockIdx.x) * SB_THREADS + threadIdx.x;
    if ((b_out || nbar_out) && t < n_seg) {
        const int b = tensor_width(static_cast<int32_t>(t), nbar_out ? nbar_out + t : nullptr);
        if (b_out) b_out[t] = b;
    }
    if (t < n_cseg) table[t].b = tensor_width(cseg_seg[t], nullptr);
}

// one workgroup of 1024 lanes: exclusive scan of the tensors' level bytes; every lane owns a
// contiguous run of table entries.
constexpr int SCAN_THREADS = 1024;

__global__ __launch_bounds__(SCAN_THREADS) void k_rule_scan(int32_t n_cseg, const int64_t* __restrict__ cseg_valid_end,
                                                            dq_cseg_width* __restrict__ table, int64_t sign_bytes,
                                                            int64_t* __restrict__ packed_bytes_out)
{
    __shared__ int64_t part[SCAN_THREADS];
    const int tid = threadIdx.x;
    const int32_t per = (n_cseg + SCAN_THREADS - 1) / SCAN_THREADS;
    const int32_t begin = tid * per < n_cseg ? tid * per : n_cseg;
    const int32_t end = begin + per < n_cseg ? begin + per : n_cseg;
    auto level_bytes = [&](int32_t c) {
        const int64_t len = cseg_valid_end[c] - table[c].seg_start;
        return (len + DQ_GRANULE - 1) / DQ_GRANULE * (DQ_GRANULE / 8) * table[c].b;
    };
    int64_t mine = 0;
    for (int32_t c = begin; c < end; ++c) mine += level_bytes(c);
    part[tid] = mine;
    __syncthreads();
    for (int off = 1; off < SCAN_THREADS; off <<= 1) {
        const int64_t add = tid >= off ? part[tid - off] : 0;
        __syncthreads();
        part[tid] += add;
        __syncthreads();
    }
    int64_t run = part[tid] - mine;
    for (int32_t c = begin; c < end; ++c) {
        const int64_t bytes = level_bytes(c);
        table[c].level_start = run;
        run += bytes;
    }
    if (tid == SCAN_THREADS - 1 && packed_bytes_out) *packed_bytes_out = sign_bytes + part[tid];
}

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

namespace {

int widths_create(const dq_plan_t* plan, int n_workers, dq_widths_t** widths_out)
{
    if (!widths_out) return DQ_ERR_INVALID_ARG;
    *widths_out = nullptr;
    if (!plan || n_workers < 1 || n_workers > DQ_MAX_WORKERS) return DQ_ERR_INVALID_ARG;
    const int rc = dq_plan_check_device(plan);
    if (rc != DQ_OK) return rc;
    dq_widths* w = new (std::nothrow) dq_widths();
    if (!w) return DQ_ERR_ALLOC;
    memset(w, 0, sizeof(*w));
    w->plan = plan;
    w->n_workers = n_workers;
    w->packed_bytes = -1;
    const size_t rows = static_cast<size_t>(n_workers);
    const size_t bytes = sizeof(dq_cseg_width) * rows * static_cast<size_t>(plan->n_cseg > 0 ? plan->n_cseg : 1);
    w->b_host = static_cast<int32_t*>(malloc(sizeof(int32_t) * rows * plan->n_seg));
    w->worker_bytes = static_cast<int64_t*>(malloc(sizeof(int64_t) * rows));
    bool ok = w->b_host != nullptr && w->worker_bytes != nullptr;
    ok = ok && hipMalloc(reinterpret_cast<void**>(&w->d_table), bytes) == hipSuccess;
    ok = ok && hipHostMalloc(reinterpret_cast<void**>(&w->h_stage), bytes, hipHostMallocDefault) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&w->uploaded, hipEventDisableTiming) == hipSuccess;
    // per-worker squared norms, followed by the block sums they are made of (multi-launch rules)
    const size_t n_sum_blocks = static_cast<size_t>((static_cast<int64_t>(plan->n_seg) + DQ_SUM_BLOCK - 1) / DQ_SUM_BLOCK);
    ok = ok && hipMalloc(reinterpret_cast<void**>(&w->d_worker_sq),
                         sizeof(double) * DQ_MAX_WORKERS * (1 + n_sum_blocks)) == hipSuccess;
    if (ok) {
        // the fixed part of the table (where each tensor starts); widths come later
        size_t k = 0;
        for (int r = 0; r < n_workers; ++r)
            for (int32_t l = 0; l < plan->n_seg; ++l) {
                if (plan->seg_len[l] == 0) continue;
                w->h_stage[k].level_start = 0;
                w->h_stage[k].seg_start = plan->seg_start[l];
                w->h_stage[k].b = 0;
                w->h_stage[k].reserved = 0;
                ++k;
            }
        ok = k == 0 || hipMemcpy(w->d_table, w->h_stage, sizeof(dq_cseg_width) * k, hipMemcpyHostToDevice) == hipSuccess;
    }
    if (!ok) {
        (void)hipGetLastError();
        dq_widths_destroy(w);
        return DQ_ERR_ALLOC;
    }
    *widths_out = w;
    return DQ_OK;
}

} // namespace

extern "C" int dq_widths_create(const dq_plan_t* plan, dq_widths_t** widths_out)
{
    return widths_create(plan, 1, widths_out);
}

extern "C" int dq_widths_create_per_worker(const dq_plan_t* plan, int M, dq_widths_t** widths_out)
{
    return widths_create(plan, M, widths_out);
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
        if (w->d_worker_sq) (void)hipFree(w->d_worker_sq);
        if (w->h_stage) (void)hipHostFree(w->h_stage);
    }
    if (have_cur) (void)hipSetDevice(cur);
    free(w->b_host);
    free(w->worker_bytes);
    delete w;
}

extern "C" int dq_widths_set(dq_widths_t* w, const int32_t* b_host, void* hip_stream)
{
    if (!w || !b_host) return DQ_ERR_INVALID_ARG;
    const dq_plan* plan = w->plan;
    const int64_t n_widths = static_cast<int64_t>(w->n_workers) * plan->n_seg;
    for (int64_t k = 0; k < n_widths; ++k)
        if (b_host[k] < 1 || b_host[k] > 8) return DQ_ERR_INVALID_ARG;
    const int rc = dq_plan_check_device(plan);
    if (rc != DQ_OK) return rc;
    // the previous upload must have left the staging buffer before it is overwritten
    if (w->packed_bytes >= 0 && hipEventSynchronize(w->uploaded) != hipSuccess) return DQ_ERR_HIP;
    size_t k = 0;
    int64_t longest = 0;
    for (int r = 0; r < w->n_workers; ++r) {
        const int32_t* row = b_host + static_cast<int64_t>(r) * plan->n_seg;
        int64_t level_bytes = 0;
        for (int32_t l = 0; l < plan->n_seg; ++l) {
            if (plan->seg_len[l] == 0) continue;
            dq_cseg_width& e = w->h_stage[k++];
            e.level_start = level_bytes;
            e.seg_start = plan->seg_start[l];
            e.b = row[l];
            e.reserved = 0;
            level_bytes += padded_len(plan->seg_len[l]) / 8 * row[l];
        }
        w->worker_bytes[r] = plan->padded_elems / 8 + level_bytes;
        longest = w->worker_bytes[r] > longest ? w->worker_bytes[r] : longest;
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (k > 0 && hipMemcpyAsync(w->d_table, w->h_stage, sizeof(dq_cseg_width) * k, hipMemcpyHostToDevice, stream) !=
                     hipSuccess)
        return DQ_ERR_HIP;
    if (hipEventRecord(w->uploaded, stream) != hipSuccess) return DQ_ERR_HIP;
    memcpy(w->b_host, b_host, sizeof(int32_t) * static_cast<size_t>(n_widths));
    w->packed_bytes = longest;
    return DQ_OK;
}

extern "C" int64_t dq_widths_worker_packed_bytes(const dq_widths_t* w, int worker)
{
    if (!w || w->packed_bytes < 0 || worker < 0) return -1;
    if (w->n_workers == 1) return w->worker_bytes[0];
    return worker < w->n_workers ? w->worker_bytes[worker] : -1;
}

extern "C" int64_t dq_widths_packed_bytes(const dq_widths_t* w) { return w ? w->packed_bytes : -1; }

extern "C" int dq_select_bits_device(const dq_plan_t* plan, dq_widths_t* widths, const float* norms_dev, int M,
                                     int64_t t, int64_t T, double eps_hat_q, double alpha, int b_min, int b_max,
                                     int rule, int32_t* b_out_dev, double* gbar_out_dev,
                                     int64_t* packed_bytes_out_dev, void* hip_stream)
{
    if (!plan || !widths || !norms_dev || widths->plan != plan) return DQ_ERR_INVALID_ARG;
    if (widths->n_workers != 1) return DQ_ERR_INVALID_ARG; // the device rules decide widths the workers share
    if (M < 1 || M > DQ_MAX_WORKERS || T < 1 || t < 0 || t >= T) return DQ_ERR_INVALID_ARG;
    if (!(eps_hat_q > 0.0) || !(alpha > 0.0) || !(alpha <= 1.0)) return DQ_ERR_INVALID_ARG;
    if (b_min < 1 || b_max > 8 || b_min > b_max || rule < 0 || rule > 2) return DQ_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(norms_dev) & 3u) || (reinterpret_cast<uintptr_t>(b_out_dev) & 3u) ||
        (reinterpret_cast<uintptr_t>(gbar_out_dev) & 7u) || (reinterpret_cast<uintptr_t>(packed_bytes_out_dev) & 7u))
        return DQ_ERR_INVALID_ARG;
    const int rc = dq_plan_check_device(plan);
    if (rc != DQ_OK) return rc;
    const double root_T_eps = sqrt(static_cast<double>(T) / eps_hat_q);
    const double weight = pow(alpha, static_cast<double>(T - 1 - t) / 2.0);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (plan->n_seg <= 1024) {
        hipLaunchKernelGGL(k_select_bits, dim3(1), dim3(SB_THREADS), 0, stream, norms_dev, M, plan->n_seg, plan->n_cseg,
                           plan->d_cseg_seg, plan->d_cseg_valid_end, widths->d_table, rule, root_T_eps, weight, b_min,
                           b_max, plan->padded_elems / 8, b_out_dev, gbar_out_dev, packed_bytes_out_dev);
    } else {
        const double factor = root_T_eps * weight;
        const int32_t widest = plan->n_seg > plan->n_cseg ? plan->n_seg : plan->n_cseg;
        const dim3 grid((widest + SB_THREADS - 1) / SB_THREADS), block(SB_THREADS);
        if (rule == 2) {
            hipLaunchKernelGGL(k_rule_tensor_widths, grid, block, 0, stream, norms_dev, M, plan->n_seg, plan->n_cseg,
                               plan->d_cseg_seg, widths->d_table, factor, b_min, b_max, b_out_dev, gbar_out_dev);
        } else {
            hipLaunchKernelGGL(k_rule_worker_sums, dim3(M), block, 0, stream, norms_dev, plan->n_seg, rule == 1 ? 1 : 0,
                               widths->d_worker_sq, widths->d_worker_sq + DQ_MAX_WORKERS);
            hipLaunchKernelGGL(k_rule_apply_single, grid, block, 0, stream, widths->d_worker_sq, M, plan->n_seg,
                               plan->n_cseg, widths->d_table, factor, b_min, b_max, b_out_dev, gbar_out_dev);
        }
        hipLaunchKernelGGL(k_rule_scan, dim3(1), dim3(SCAN_THREADS), 0, stream, plan->n_cseg, plan->d_cseg_valid_end,
                           widths->d_table, plan->padded_elems / 8, packed_bytes_out_dev);
    }
    if (hipGetLastError() != hipSuccess) return DQ_ERR_HIP;
    // the host no longer knows the widths: messages must have room for b_max everywhere
    int64_t level_bytes = 0;
    for (int32_t l = 0; l < plan->n_seg; ++l) {
        widths->b_host[l] = 0;
        level_bytes += padded_len(plan->seg_len[l]) / 8 * b_max;
    }
    widths->packed_bytes = plan->padded_elems / 8 + level_bytes;
    widths->worker_bytes[0] = widths->packed_bytes;
    return DQ_OK;
}

// Eq. (17) with each worker's own norm (or each worker's tensor norms): see the header.
extern "C" int dq_select_bits_per_worker(const float* norms_host, int M, int n_seg, int64_t t, int64_t T,
                                         double eps_hat_q, double alpha, int b_min, int b_max, int per_tensor,
                                         int32_t* b_out_host)
{
    if (!norms_host || !b_out_host || M < 1 || n_seg < 1) return DQ_ERR_INVALID_ARG;
    if (T < 1 || t < 0 || t >= T) return DQ_ERR_INVALID_ARG;
    if (!(eps_hat_q > 0.0) || !(alpha > 0.0) || !(alpha <= 1.0)) return DQ_ERR_INVALID_ARG;
    if (b_min < 1 || b_max > 8 || b_min > b_max) return DQ_ERR_INVALID_ARG;
    const double factor = sqrt(static_cast<double>(T) / eps_hat_q) * pow(alpha, static_cast<double>(T - 1 - t) / 2.0);
    for (int i = 0; i < M; ++i) {
        const float* row = norms_host + static_cast<int64_t>(i) * n_seg;
        const double worker_norm = sqrt(dq_worker_squared_norm(row, n_seg));
        for (int l = 0; l < n_seg; ++l) {
            const double s_star = factor * (per_tensor ? static_cast<double>(row[l]) : worker_norm);
            int b = b_max;
            for (int cand = b_min; cand <= b_max; ++cand) {
                if (static_cast<double>((1 << cand) - 1) >= s_star) {
                    b = cand;
                    break;
                }
            }
            b_out_host[static_cast<int64_t>(i) * n_seg + l] = b;
        }
    }
    return DQ_OK;
}
