// dq_norm / dq_norm_linf: l2 or max norm per (worker, segment) -- the ||g||_p of Eq. (5) with
// p = 2 or p = infinity.
//
// Two passes, both deterministic.  Pass 1: one workgroup per (norm item, worker) sums the squares
// of up to 4096 valid elements in binary64 (squares of binary32 values are exact there): per-lane
// partial, wavefront shuffle tree, then the four wave sums through LDS in wave order.  Pass 2: one
// workgroup per (segment, worker) adds that segment's item partials in a fixed order and takes
// the square root.  A segment of a single item (at most 4096 elements) is finished by pass 1
// itself -- the same value, since its sum has one term -- so a gradient cut into many small
// tensors costs no second-pass workgroups.  HBM traffic: 4 bytes read per element, plus 8 bytes
// per 4096 elements.
// The max norm takes the same two passes with binary32 maxima in place of the binary64 sums (a
// maximum does not depend on the order; a NaN element never wins a comparison).
//
// Plans in which no tensor crosses a multiple of 4096 padded elements take k_norm_chunk instead:
// one workgroup per chunk finishes the norms of all the tensors inside it, one pass.
#include <atomic>

#include "dq_chunk_norm.h"
#include "dq_internal.h"

// Scratch of dq_norm_static_scratch: the per-(item, worker) partial sums that dq_norm keeps in the
// caller's workspace.  Every GPU the library runs on holds its own copy of this array until the
// process ends.  In host code the name is only a stand-in: the device address of a GPU's copy
// comes from hipGetSymbolAddress (static_scratch_of below) and that pointer is what kernels get.
static __device__ __align__(256) unsigned char scratch[DQ_NORM_STATIC_SCRATCH_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
std::atomic<void*> g_scratch_ptr[MAX_DEVICES]; // device address of `scratch` on each GPU, null until asked for

// The current device's copy of `scratch`; `device` must be the current device.  Looked up once per
// device (two threads that both find it missing look up the same address).
void* static_scratch_of(int device)
{
    if (device < 0 || device >= MAX_DEVICES) return nullptr;
    void* ptr = g_scratch_ptr[device].load(std::memory_order_acquire);
    if (ptr) return ptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
        (void)hipGetLastError();
        return nullptr;
    }
    g_scratch_ptr[device].store(ptr, std::memory_order_release);
    return ptr;
}

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_down(v, off, 64);
    return v; // lane 0 holds the sum
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float o = __shfl_down(v, off, 64);
        v = o > v ? o : v;
    }
    return v; // lane 0 holds the maximum
}

__device__ __forceinline__ float larger(float m, float x)
{
    const float a = fabsf(x);
    return a > m ? a : m;
}

template <bool LINF>
__global__ __launch_bounds__(256) void k_norm_partial(const float* __restrict__ grads,
                                                      int64_t worker_stride,
                                                      const dq_norm_item* __restrict__ items,
                                                      int32_t n_items, void* __restrict__ partial_out,
                                                      const int32_t* __restrict__ seg_item_begin, int32_t n_seg,
                                                      float* __restrict__ norms)
{
    __shared__ double wave_part[4];
    const int item_id = blockIdx.x;
    const int w = blockIdx.y;
    const dq_norm_item item = items[item_id];
    const float* g = grads + static_cast<int64_t>(w) * worker_stride + item.start;
    const int tid = threadIdx.x;

    float4 v[DQ_NORM_CHUNK / 1024];
#pragma unroll
    for (int k = 0; k < DQ_NORM_CHUNK / 1024; ++k) {
        const int e = (k * 256 + tid) * 4;
        // the padded allocation is a multiple of 128 elements, so a float4 that starts inside the
        // item's valid range never leaves the worker's buffer
        // read once here (non-temporal): measured 2.69 -> 2.57 ms at D = 2^28, M = 16
        v[k] = e < item.count ? dq_load_stream(reinterpret_cast<const float4*>(g + e)) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    if constexpr (LINF) {
        float m = 0.f;
#pragma unroll
        for (int k = 0; k < DQ_NORM_CHUNK / 1024; ++k) {
            const int e = (k * 256 + tid) * 4;
            m = larger(m, e + 0 < item.count ? v[k].x : 0.f);
            m = larger(m, e + 1 < item.count ? v[k].y : 0.f);
            m = larger(m, e + 2 < item.count ? v[k].z : 0.f);
            m = larger(m, e + 3 < item.count ? v[k].w : 0.f);
        }
        m = wave_max(m);
        float* wave_m = reinterpret_cast<float*>(wave_part);
        if ((tid & 63) == 0) wave_m[tid >> 6] = m;
        __syncthreads();
        if (tid == 0) {
            float top = wave_m[0];
#pragma unroll
            for (int k = 1; k < 4; ++k) top = wave_m[k] > top ? wave_m[k] : top;
            if (seg_item_begin[item.seg + 1] - seg_item_begin[item.seg] == 1)
                norms[static_cast<int64_t>(w) * n_seg + item.seg] = top;
            else
                static_cast<float*>(partial_out)[static_cast<int64_t>(w) * n_items + item_id] = top;
        }
        return;
    }
    double* partial = static_cast<double*>(partial_out);
    double acc = 0.0;
    // masked in binary32 before the conversion (measured faster than a separate unmasked path for full items)
#pragma unroll
    for (int k = 0; k < DQ_NORM_CHUNK / 1024; ++k) {
        const int e = (k * 256 + tid) * 4;
        const double x0 = static_cast<double>(e + 0 < item.count ? v[k].x : 0.0f);
        const double x1 = static_cast<double>(e + 1 < item.count ? v[k].y : 0.0f);
        const double x2 = static_cast<double>(e + 2 < item.count ? v[k].z : 0.0f);
        const double x3 = static_cast<double>(e + 3 < item.count ? v[k].w : 0.0f);
        acc = __builtin_fma(x0, x0, acc);
        acc = __builtin_fma(x1, x1, acc);
        acc = __builtin_fma(x2, x2, acc);
        acc = __builtin_fma(x3, x3, acc);
    }
    acc = wave_sum(acc);
    if ((tid & 63) == 0) wave_part[tid >> 6] = acc;
    __syncthreads();
    if (tid == 0) {
        const double total = ((wave_part[0] + wave_part[1]) + wave_part[2]) + wave_part[3];
        if (seg_item_begin[item.seg + 1] - seg_item_begin[item.seg] == 1)
            norms[static_cast<int64_t>(w) * n_seg + item.seg] = static_cast<float>(sqrt(total));
        else
            partial[static_cast<int64_t>(w) * n_items + item_id] = total;
    }
}

constexpr int FINISH_THREADS = 1024;

__global__ __launch_bounds__(FINISH_THREADS) void k_norm_finish(const double* __restrict__ partial, int32_t n_items,
                                                                const int32_t* __restrict__ seg_item_begin,
                                                                const int32_t* __restrict__ finish_seg,
                                                                int32_t n_seg, float* __restrict__ norms)
{
    __shared__ double wave_part[FINISH_THREADS / 64];
    const int seg = finish_seg[blockIdx.x];
    const int w = blockIdx.y;
    const int tid = threadIdx.x;
    const int begin = seg_item_begin[seg], end = seg_item_begin[seg + 1];
    const double* p = partial + static_cast<int64_t>(w) * n_items;
    // lane-strided, in a fixed order; eight independent loads in flight per lane
    double acc = 0.0;
    int i = begin + tid;
    for (; i + 7 * FINISH_THREADS < end; i += 8 * FINISH_THREADS) {
        double v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = p[i + k * FINISH_THREADS];
#pragma unroll
        for (int k = 0; k < 8; ++k) acc += v[k];
    }
    for (; i < end; i += FINISH_THREADS) acc += p[i];
    acc = wave_sum(acc);
    if ((tid & 63) == 0) wave_part[tid >> 6] = acc;
    __syncthreads();
    if (tid == 0) {
        double total = 0.0;
#pragma unroll
        for (int k = 0; k < FINISH_THREADS / 64; ++k) total += wave_part[k];
        norms[static_cast<int64_t>(w) * n_seg + seg] = static_cast<float>(sqrt(total));
    }
}

__global__ __launch_bounds__(FINISH_THREADS) void k_norm_linf_finish(const float* __restrict__ partial, int32_t n_items,
                                                                     const int32_t* __restrict__ seg_item_begin,
                                                                     const int32_t* __restrict__ finish_seg,
                                                                     int32_t n_seg, float* __restrict__ norms)
{
    __shared__ float wave_m[FINISH_THREADS / 64];
    const int seg = finish_seg[blockIdx.x];
    const int w = blockIdx.y;
    const int tid = threadIdx.x;
    const int begin = seg_item_begin[seg], end = seg_item_begin[seg + 1];
    const float* p = partial + static_cast<int64_t>(w) * n_items;
    float m = 0.f;
    int i = begin + tid;
    for (; i + 7 * FINISH_THREADS < end; i += 8 * FINISH_THREADS) {
        float v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = p[i + k * FINISH_THREADS];
#pragma unroll
        for (int k = 0; k < 8; ++k) m = v[k] > m ? v[k] : m;
    }
    for (; i < end; i += FINISH_THREADS) m = p[i] > m ? p[i] : m;
    m = wave_max(m);
    if ((tid & 63) == 0) wave_m[tid >> 6] = m;
    __syncthreads();
    if (tid == 0) {
        float top = 0.f;
#pragma unroll
        for (int k = 0; k < FINISH_THREADS / 64; ++k) top = wave_m[k] > top ? wave_m[k] : top;
        norms[static_cast<int64_t>(w) * n_seg + seg] = top;
    }
}

// Chunk-local plans: one workgroup per 4096-element chunk finishes the norms of all the tensors
// inside it, however small they are; no second pass.
template <bool LINF>
__global__ __launch_bounds__(256) void k_norm_chunk(const float* __restrict__ grads, int64_t worker_stride,
                                                    const int32_t* __restrict__ granule_cseg,
                                                    const int32_t* __restrict__ cseg_seg,
                                                    const int64_t* __restrict__ cseg_valid_end, int64_t padded_elems,
                                                    int32_t n_seg, float* __restrict__ norms)
{
    __shared__ double lds_gsum[DQ_CHUNK_GRANULES];
    __shared__ int32_t lds_glocal[DQ_CHUNK_GRANULES];
    __shared__ int32_t lds_valid_end[DQ_CHUNK_GRANULES];
    const int tid = threadIdx.x;
    const int w = blockIdx.y;
    const int64_t chunk0 = static_cast<int64_t>(blockIdx.x) * DQ_CHUNK;
    const uint32_t n_elems = static_cast<uint32_t>(padded_elems - chunk0 < DQ_CHUNK ? padded_elems - chunk0 : DQ_CHUNK);
    const float* g = grads + static_cast<int64_t>(w) * worker_stride + chunk0;
    const int32_t* gseg = granule_cseg + (chunk0 >> 7);

    float4 x[2][2];
    int32_t seg[2];
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        uint32_t e = it * 2048 + tid * 8;
        e = e < n_elems ? e : n_elems - 8; // clamped: always in bounds, masked out below
        x[it][0] = dq_load_stream(reinterpret_cast<const float4*>(g + e));
        x[it][1] = dq_load_stream(reinterpret_cast<const float4*>(g + e + 4));
        seg[it] = gseg[e >> 7];
    }
    const int32_t seg_first = gseg[0];
    const int n_local = gseg[(n_elems - 1) >> 7] - seg_first + 1;
    if (tid < n_local) {
        const int64_t rel = cseg_valid_end[seg_first + tid] - chunk0;
        lds_valid_end[tid] = rel < DQ_CHUNK ? static_cast<int32_t>(rel) : DQ_CHUNK;
    }
    __syncthreads();
    int valid[2], local[2];
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const uint32_t e = it * 2048 + tid * 8;
        local[it] = seg[it] - seg_first;
        valid[it] = e < n_elems ? lds_valid_end[local[it]] - static_cast<int32_t>(e) : 0;
    }
    const int n_scan = dq_chunk_granule_sums<LINF>(x, valid, local, tid, lds_gsum, lds_glocal, n_local == 1,
                                                   static_cast<int>(n_elems >> 7));
    __syncthreads();
    if (tid < DQ_CHUNK_GRANULES)
        dq_chunk_tensor_norms<LINF>(tid, n_scan, lds_gsum, lds_glocal, [&](int j, float N) {
            norms[static_cast<int64_t>(w) * n_seg + cseg_seg[seg_first + j]] = N;
        });
}

__global__ __launch_bounds__(256) void k_zero_floats(float* __restrict__ dst, int64_t n)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i < n) dst[i] = 0.0f;
}

int norm_entry(bool linf, const dq_plan_t* plan, const float* grads_dev, int64_t worker_stride_elems, int M,
               float* norms_dev, void* workspace_dev, void* hip_stream);

} // namespace

int dq_zero_floats(float* dst_dev, int64_t n, hipStream_t stream)
{
    if (n <= 0) return DQ_OK;
    const int64_t blocks = (n + 255) / 256;
    if (blocks > INT32_MAX) return DQ_ERR_INVALID_ARG;
    hipLaunchKernelGGL(k_zero_floats, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, stream, dst_dev, n);
    return hipGetLastError() == hipSuccess ? DQ_OK : DQ_ERR_HIP;
}

extern "C" int dq_norm(const dq_plan_t* plan, const float* grads_dev, int64_t worker_stride_elems,
                       int M, float* norms_dev, void* workspace_dev, void* hip_stream)
{
    return norm_entry(false, plan, grads_dev, worker_stride_elems, M, norms_dev, workspace_dev, hip_stream);
}

extern "C" int dq_norm_linf(const dq_plan_t* plan, const float* grads_dev, int64_t worker_stride_elems,
                            int M, float* norms_dev, void* workspace_dev, void* hip_stream)
{
    return norm_entry(true, plan, grads_dev, worker_stride_elems, M, norms_dev, workspace_dev, hip_stream);
}

void dq_norm_static_scratch_prepare(int device) { (void)static_scratch_of(device); }

extern "C" int64_t dq_norm_static_scratch_max_bytes(void) { return DQ_NORM_STATIC_SCRATCH_BYTES; }

extern "C" int dq_norm_static_scratch(const dq_plan_t* plan, const float* grads_dev, int64_t worker_stride_elems,
                                      int M, int linf, float* norms_dev, void* hip_stream)
{
    if (!plan) return DQ_ERR_INVALID_ARG;
    const int64_t need = dq_workspace_bytes(plan, M);
    if (need < 0 || need > DQ_NORM_STATIC_SCRATCH_BYTES) return DQ_ERR_INVALID_ARG;
    const int rc = dq_plan_check_device(plan); // makes the plan's GPU current
    if (rc != DQ_OK) return rc;
    void* ptr = static_scratch_of(plan->device);
    if (!ptr) return DQ_ERR_HIP;
    // every partial a launch reads it has written itself: nothing in the scratch has to start at zero
    return norm_entry(linf != 0, plan, grads_dev, worker_stride_elems, M, norms_dev, ptr, hip_stream);
}

namespace {

int norm_entry(bool linf, const dq_plan_t* plan, const float* grads_dev, int64_t worker_stride_elems, int M,
               float* norms_dev, void* workspace_dev, void* hip_stream)
{
    if (!plan || !grads_dev || !norms_dev || !workspace_dev) return DQ_ERR_INVALID_ARG;
    if (M < 1 || M > DQ_MAX_WORKERS) return DQ_ERR_INVALID_ARG;
    if (worker_stride_elems < plan->padded_elems || (worker_stride_elems & 3)) return DQ_ERR_INVALID_ARG;
    if (!dq_aligned16(grads_dev) || !dq_aligned16(workspace_dev) || (reinterpret_cast<uintptr_t>(norms_dev) & 3u))
        return DQ_ERR_INVALID_ARG;
    const int rc = dq_plan_check_device(plan);
    if (rc != DQ_OK) return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (plan->chunk_local) {
        // tensors without elements belong to no chunk: their norm is zero
        if (plan->n_cseg < plan->n_seg) {
            const int zrc = dq_zero_floats(norms_dev, static_cast<int64_t>(M) * plan->n_seg, stream);
            if (zrc != DQ_OK) return zrc;
        }
        const int64_t n_chunks = (plan->padded_elems + DQ_CHUNK - 1) / DQ_CHUNK;
        if (n_chunks > INT32_MAX) return DQ_ERR_INVALID_ARG;
        const dim3 grid(static_cast<unsigned>(n_chunks), M);
        if (n_chunks > 0) {
            if (linf)
                hipLaunchKernelGGL(k_norm_chunk<true>, grid, dim3(256), 0, stream, grads_dev, worker_stride_elems,
                                   plan->d_granule_cseg, plan->d_cseg_seg, plan->d_cseg_valid_end, plan->padded_elems,
                                   plan->n_seg, norms_dev);
            else
                hipLaunchKernelGGL(k_norm_chunk<false>, grid, dim3(256), 0, stream, grads_dev, worker_stride_elems,
                                   plan->d_granule_cseg, plan->d_cseg_seg, plan->d_cseg_valid_end, plan->padded_elems,
                                   plan->n_seg, norms_dev);
        }
        return hipGetLastError() == hipSuccess ? DQ_OK : DQ_ERR_HIP;
    }
    const dim3 grid_items(plan->n_items, M), grid_segs(plan->n_finish, M);
    if (linf) {
        if (plan->n_items > 0)
            hipLaunchKernelGGL(k_norm_partial<true>, grid_items, dim3(256), 0, stream, grads_dev,
                               worker_stride_elems, plan->d_items, plan->n_items, workspace_dev,
                               plan->d_seg_item_begin, plan->n_seg, norms_dev);
        if (plan->n_finish > 0)
            hipLaunchKernelGGL(k_norm_linf_finish, grid_segs, dim3(FINISH_THREADS), 0, stream,
                               static_cast<const float*>(workspace_dev), plan->n_items, plan->d_seg_item_begin,
                               plan->d_finish_seg, plan->n_seg, norms_dev);
    } else {
        if (plan->n_items > 0)
            hipLaunchKernelGGL(k_norm_partial<false>, grid_items, dim3(256), 0, stream, grads_dev,
                               worker_stride_elems, plan->d_items, plan->n_items, workspace_dev,
                               plan->d_seg_item_begin, plan->n_seg, norms_dev);
        if (plan->n_finish > 0)
            hipLaunchKernelGGL(k_norm_finish, grid_segs, dim3(FINISH_THREADS), 0, stream,
                               static_cast<const double*>(workspace_dev), plan->n_items, plan->d_seg_item_begin,
                               plan->d_finish_seg, plan->n_seg, norms_dev);
    }
    return hipGetLastError() == hipSuccess ? DQ_OK : DQ_ERR_HIP;
}

} // namespace
