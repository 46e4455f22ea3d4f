// dq_quantize_pack: the EWU quantizer of Eq. (5)-(6) fused with the packing of the message whose
// size Eq. (7) counts.
//
// Work split.  One workgroup (256 lanes) owns TILES consecutive tiles of 2048 padded elements of
// one worker; a lane owns 8 consecutive elements of each tile (two 16-byte loads, two Philox
// blocks), so its output is exactly one sign byte and B level bytes.  Those bytes are staged in
// LDS and leave the workgroup as 16-byte stores that cover each plane's bytes contiguously.
//
// Per-segment state.  The scale s/N and the end of the valid range of every segment the
// workgroup touches (at most one per 128-element granule) are put in LDS once per workgroup, so
// the one binary32 division per (worker, segment) is never on a lane's critical path.
//
// HBM traffic per element: 4 bytes read, (B+1)/8 bytes written, plus 4 bytes per 128 elements for
// the granule table.
#include "dq_quantize_core.h"

namespace {

template <int B, int TILES, int NORM>
__global__ __launch_bounds__(QP_THREADS) void k_quantize_pack(
    const float* __restrict__ grads, int64_t worker_stride, const float* __restrict__ norms, int32_t n_seg,
    const int32_t* __restrict__ granule_cseg, const int32_t* __restrict__ cseg_seg,
    const int64_t* __restrict__ cseg_valid_end, int64_t padded_elems,
    uint32_t key0, uint32_t key1, uint32_t step, uint32_t worker_base, uint8_t* __restrict__ packed,
    int64_t packed_stride, float* __restrict__ norms_out)
{
    quantize_pack_chunk<B, TILES, NORM>(grads, worker_stride, norms, n_seg, granule_cseg, cseg_seg, cseg_valid_end,
                                        padded_elems, key0, key1, step, worker_base, packed, packed_stride, norms_out,
                                        blockIdx.x);
}

template <int TILES, int NORM> // NORM as in k_quantize_pack
__global__ __launch_bounds__(QP_THREADS) void k_quantize_pack_v(
    const float* __restrict__ grads, int64_t worker_stride, const float* __restrict__ norms, int32_t n_seg,
    const int32_t* __restrict__ granule_cseg, const int32_t* __restrict__ cseg_seg,
    const int64_t* __restrict__ cseg_valid_end, const dq_cseg_width* __restrict__ widths_table,
    int32_t widths_worker_stride, int64_t padded_elems,
    uint32_t key0, uint32_t key1, uint32_t step, uint32_t worker_base, uint8_t* __restrict__ packed,
    int64_t packed_stride, float* __restrict__ norms_out)
{
    quantize_pack_chunk_v<TILES, NORM>(grads, worker_stride, norms, n_seg, granule_cseg, cseg_seg, cseg_valid_end,
                                       widths_table, widths_worker_stride, padded_elems, key0, key1, step, worker_base,
                                       packed, packed_stride, norms_out, blockIdx.x);
}

// ---------------------------------------------------------------------------------------------
// Sign-only messages (the one-bit baseline of the paper's Table 2): the sign plane alone.  Same
// work split with four tiles per workgroup; no random numbers, no norms.
// HBM traffic per element: 4 bytes read, 1/8 byte written.
// ---------------------------------------------------------------------------------------------
constexpr int SP_TILES = 4;

__global__ __launch_bounds__(QP_THREADS) void k_sign_pack(const float* __restrict__ grads, int64_t worker_stride,
                                                          const int32_t* __restrict__ granule_cseg,
                                                          const int64_t* __restrict__ cseg_valid_end,
                                                          int64_t padded_elems, uint8_t* __restrict__ packed,
                                                          int64_t packed_stride)
{
    constexpr int CHUNK = QP_TILE * SP_TILES;
    __shared__ __align__(16) uint8_t lds_sign[SP_TILES * QP_THREADS];

    const uint32_t tid = threadIdx.x;
    const uint32_t w = blockIdx.y;
    const int64_t chunk0 = static_cast<int64_t>(blockIdx.x) * CHUNK;
    const uint32_t n_elems = static_cast<uint32_t>(padded_elems - chunk0 < CHUNK ? padded_elems - chunk0 : CHUNK);
    const float* g = grads + static_cast<int64_t>(w) * worker_stride + chunk0;
    const int32_t* gseg = granule_cseg + (chunk0 >> 7);

    float4 x[SP_TILES][2];
    int64_t valid_end[SP_TILES];
#pragma unroll
    for (int it = 0; it < SP_TILES; ++it) {
        uint32_t e = it * QP_TILE + tid * QP_PER_LANE;
        e = e < n_elems ? e : n_elems - QP_PER_LANE; // clamped: always in bounds, result unused
        x[it][0] = *reinterpret_cast<const float4*>(g + e);
        x[it][1] = *reinterpret_cast<const float4*>(g + e + 4);
        valid_end[it] = cseg_valid_end[gseg[e >> 7]];
    }
#pragma unroll
    for (int it = 0; it < SP_TILES; ++it) {
        const uint32_t e = it * QP_TILE + tid * QP_PER_LANE;
        if (e < n_elems) {
            const float v[8] = { x[it][0].x, x[it][0].y, x[it][0].z, x[it][0].w,
                                 x[it][1].x, x[it][1].y, x[it][1].z, x[it][1].w };
            uint32_t sign = 0;
#pragma unroll
            for (int k = 7; k >= 0; --k) sign = __builtin_amdgcn_alignbit(sign, __float_as_uint(v[k]), 31);
            const int64_t n_valid = valid_end[it] - (chunk0 + e);
            if (n_valid < QP_PER_LANE) sign &= (1u << (n_valid > 0 ? static_cast<int>(n_valid) : 0)) - 1u;
            lds_sign[it * QP_THREADS + tid] = static_cast<uint8_t>(sign);
        }
    }
    __syncthreads();
    uint4* dst = reinterpret_cast<uint4*>(packed + static_cast<int64_t>(w) * packed_stride + (chunk0 >> 3));
    const uint4* src = reinterpret_cast<const uint4*>(lds_sign);
    for (uint32_t i = tid; i < n_elems / 128; i += QP_THREADS) dq_store_stream(dst + i, src[i]);
}

template <int B, int NORM>
int launch(const dq_plan* plan, const float* grads, int64_t worker_stride, int M, const float* norms,
           uint64_t seed, uint32_t step, uint32_t worker_base, uint8_t* packed, int64_t packed_stride,
           float* norms_out, hipStream_t stream)
{
    constexpr int TILES = DQ_QP_TILES;
    constexpr int CHUNK = QP_TILE * TILES;
    const int64_t n_chunks = (plan->padded_elems + CHUNK - 1) / CHUNK;
    if (n_chunks > INT32_MAX) return DQ_ERR_INVALID_ARG;
    hipLaunchKernelGGL((k_quantize_pack<B, TILES, NORM>), dim3(static_cast<unsigned>(n_chunks), M), dim3(QP_THREADS),
                       0, stream, grads, worker_stride, norms, plan->n_seg, plan->d_granule_cseg,
                       plan->d_cseg_seg, plan->d_cseg_valid_end, plan->padded_elems, static_cast<uint32_t>(seed),
                       static_cast<uint32_t>(seed >> 32), step, worker_base, packed, packed_stride, norms_out);
    return hipGetLastError() == hipSuccess ? DQ_OK : DQ_ERR_HIP;
}

template <int NORM>
int launch_width(int b, const dq_plan* plan, const float* grads, int64_t worker_stride, int M, const float* norms,
                 uint64_t seed, uint32_t step, uint32_t worker_base, uint8_t* packed, int64_t packed_stride,
                 float* norms_out, hipStream_t stream)
{
    switch (b) {
    case 1: return launch<1, NORM>(plan, grads, worker_stride, M, norms, seed, step, worker_base, packed, packed_stride, norms_out, stream);
    case 2: return launch<2, NORM>(plan, grads, worker_stride, M, norms, seed, step, worker_base, packed, packed_stride, norms_out, stream);
    case 3: return launch<3, NORM>(plan, grads, worker_stride, M, norms, seed, step, worker_base, packed, packed_stride, norms_out, stream);
    case 4: return launch<4, NORM>(plan, grads, worker_stride, M, norms, seed, step, worker_base, packed, packed_stride, norms_out, stream);
    case 5: return launch<5, NORM>(plan, grads, worker_stride, M, norms, seed, step, worker_base, packed, packed_stride, norms_out, stream);
    case 6: return launch<6, NORM>(plan, grads, worker_stride, M, norms, seed, step, worker_base, packed, packed_stride, norms_out, stream);
    case 7: return launch<7, NORM>(plan, grads, worker_stride, M, norms, seed, step, worker_base, packed, packed_stride, norms_out, stream);
    default: return launch<8, NORM>(plan, grads, worker_stride, M, norms, seed, step, worker_base, packed, packed_stride, norms_out, stream);
    }
}

} // namespace

extern "C" int dq_quantize_pack(const dq_plan_t* plan, const float* grads_dev, int64_t worker_stride_elems,
                                int M, const float* norms_dev, int b, uint64_t seed, uint32_t step,
                                uint32_t worker_base, uint8_t* packed_dev,
                                int64_t packed_worker_stride_bytes, void* hip_stream)
{
    if (!plan || !grads_dev || !norms_dev || !packed_dev) return DQ_ERR_INVALID_ARG;
    if (M < 1 || M > DQ_MAX_WORKERS || b < 1 || b > 8) return DQ_ERR_INVALID_ARG;
    if (worker_stride_elems < plan->padded_elems || (worker_stride_elems & 3)) return DQ_ERR_INVALID_ARG;
    if (packed_worker_stride_bytes < dq_packed_bytes(plan, b) || (packed_worker_stride_bytes & 15))
        return DQ_ERR_INVALID_ARG;
    if (!dq_aligned16(grads_dev) || !dq_aligned16(packed_dev) || (reinterpret_cast<uintptr_t>(norms_dev) & 3u))
        return DQ_ERR_INVALID_ARG;
    const int rc = dq_plan_check_device(plan);
    if (rc != DQ_OK) return rc;
    if (plan->padded_elems == 0) return DQ_OK;
    return launch_width<0>(b, plan, grads_dev, worker_stride_elems, M, norms_dev, seed, step, worker_base, packed_dev,
                           packed_worker_stride_bytes, nullptr, static_cast<hipStream_t>(hip_stream));
}

namespace {

int quantize_v_entry(int norm_mode, const dq_plan_t* plan, const dq_widths_t* widths, const float* grads_dev,
                     int64_t worker_stride_elems, int M, const float* norms_in, float* norms_out, uint64_t seed,
                     uint32_t step, uint32_t worker_base, uint8_t* packed_dev, int64_t packed_worker_stride_bytes,
                     void* hip_stream)
{
    const float* norms_any = norm_mode == 0 ? norms_in : norms_out;
    if (!plan || !widths || !grads_dev || !norms_any || !packed_dev) return DQ_ERR_INVALID_ARG;
    if (widths->plan != plan || widths->packed_bytes < 0) return DQ_ERR_INVALID_ARG;
    if (norm_mode != 0 && !plan->chunk_local) return DQ_ERR_INVALID_ARG;
    if (M < 1 || M > DQ_MAX_WORKERS) return DQ_ERR_INVALID_ARG;
    if (widths->n_workers != 1 && widths->n_workers != M) return DQ_ERR_INVALID_ARG;
    const int32_t row_stride = widths->n_workers == 1 ? 0 : plan->n_cseg;
    if (worker_stride_elems < plan->padded_elems || (worker_stride_elems & 3)) return DQ_ERR_INVALID_ARG;
    if (packed_worker_stride_bytes < widths->packed_bytes || (packed_worker_stride_bytes & 15))
        return DQ_ERR_INVALID_ARG;
    if (!dq_aligned16(grads_dev) || !dq_aligned16(packed_dev) || (reinterpret_cast<uintptr_t>(norms_any) & 3u))
        return DQ_ERR_INVALID_ARG;
    const int rc = dq_plan_check_device(plan);
    if (rc != DQ_OK) return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (norm_mode != 0 && plan->n_cseg < plan->n_seg) { // tensors without elements: norm zero
        const int zrc = dq_zero_floats(norms_out, static_cast<int64_t>(M) * plan->n_seg, stream);
        if (zrc != DQ_OK) return zrc;
    }
    if (plan->padded_elems == 0) return DQ_OK;
    constexpr int TILES = DQ_QP_TILES;
    constexpr int CHUNK = QP_TILE * TILES;
    const int64_t n_chunks = (plan->padded_elems + CHUNK - 1) / CHUNK;
    if (n_chunks > INT32_MAX) return DQ_ERR_INVALID_ARG;
    const dim3 grid(static_cast<unsigned>(n_chunks), M), block(QP_THREADS);
#define DQ_LAUNCH_QV(NORM)                                                                                        \
    hipLaunchKernelGGL((k_quantize_pack_v<TILES, NORM>), grid, block, 0, stream, grads_dev, worker_stride_elems,  \
                       norms_in, plan->n_seg, plan->d_granule_cseg, plan->d_cseg_seg, plan->d_cseg_valid_end,     \
                       widths->d_table, row_stride, plan->padded_elems, static_cast<uint32_t>(seed),              \
                       static_cast<uint32_t>(seed >> 32), step, worker_base, packed_dev, packed_worker_stride_bytes, \
                       norms_out)
    if (norm_mode == 0)
        DQ_LAUNCH_QV(0);
    else if (norm_mode == 1)
        DQ_LAUNCH_QV(1);
    else
        DQ_LAUNCH_QV(2);
#undef DQ_LAUNCH_QV
    return hipGetLastError() == hipSuccess ? DQ_OK : DQ_ERR_HIP;
}

} // namespace

extern "C" int dq_quantize_pack_v(const dq_plan_t* plan, const dq_widths_t* widths, const float* grads_dev,
                                  int64_t worker_stride_elems, int M, const float* norms_dev, uint64_t seed,
                                  uint32_t step, uint32_t worker_base, uint8_t* packed_dev,
                                  int64_t packed_worker_stride_bytes, void* hip_stream)
{
    return quantize_v_entry(0, plan, widths, grads_dev, worker_stride_elems, M, norms_dev, nullptr, seed, step,
                            worker_base, packed_dev, packed_worker_stride_bytes, hip_stream);
}

extern "C" int dq_norm_quantize_pack_v(const dq_plan_t* plan, const dq_widths_t* widths, const float* grads_dev,
                                       int64_t worker_stride_elems, int M, int linf, uint64_t seed, uint32_t step,
                                       uint32_t worker_base, float* norms_dev, uint8_t* packed_dev,
                                       int64_t packed_worker_stride_bytes, void* hip_stream)
{
    return quantize_v_entry(linf ? 2 : 1, plan, widths, grads_dev, worker_stride_elems, M, nullptr, norms_dev, seed,
                            step, worker_base, packed_dev, packed_worker_stride_bytes, hip_stream);
}

extern "C" int dq_sign_pack(const dq_plan_t* plan, const float* grads_dev, int64_t worker_stride_elems, int M,
                            uint8_t* packed_dev, int64_t packed_worker_stride_bytes, void* hip_stream)
{
    if (!plan || !grads_dev || !packed_dev) return DQ_ERR_INVALID_ARG;
    if (M < 1 || M > DQ_MAX_WORKERS) return DQ_ERR_INVALID_ARG;
    if (worker_stride_elems < plan->padded_elems || (worker_stride_elems & 3)) return DQ_ERR_INVALID_ARG;
    if (packed_worker_stride_bytes < plan->padded_elems / 8 || (packed_worker_stride_bytes & 15))
        return DQ_ERR_INVALID_ARG;
    if (!dq_aligned16(grads_dev) || !dq_aligned16(packed_dev)) return DQ_ERR_INVALID_ARG;
    const int rc = dq_plan_check_device(plan);
    if (rc != DQ_OK) return rc;
    if (plan->padded_elems == 0) return DQ_OK;
    constexpr int CHUNK = QP_TILE * SP_TILES;
    const int64_t n_chunks = (plan->padded_elems + CHUNK - 1) / CHUNK;
    if (n_chunks > INT32_MAX) return DQ_ERR_INVALID_ARG;
    hipLaunchKernelGGL(k_sign_pack, dim3(static_cast<unsigned>(n_chunks), M), dim3(QP_THREADS), 0,
                       static_cast<hipStream_t>(hip_stream), grads_dev, worker_stride_elems, plan->d_granule_cseg,
                       plan->d_cseg_valid_end, plan->padded_elems, packed_dev, packed_worker_stride_bytes);
    return hipGetLastError() == hipSuccess ? DQ_OK : DQ_ERR_HIP;
}

extern "C" int dq_norm_quantize_pack(const dq_plan_t* plan, const float* grads_dev, int64_t worker_stride_elems,
                                     int M, int linf, int b, uint64_t seed, uint32_t step, uint32_t worker_base,
                                     float* norms_dev, uint8_t* packed_dev, int64_t packed_worker_stride_bytes,
                                     void* hip_stream)
{
    if (!plan || !grads_dev || !norms_dev || !packed_dev) return DQ_ERR_INVALID_ARG;
    if (!plan->chunk_local) return DQ_ERR_INVALID_ARG;
    if (M < 1 || M > DQ_MAX_WORKERS || b < 1 || b > 8) return DQ_ERR_INVALID_ARG;
    if (worker_stride_elems < plan->padded_elems || (worker_stride_elems & 3)) return DQ_ERR_INVALID_ARG;
    if (packed_worker_stride_bytes < dq_packed_bytes(plan, b) || (packed_worker_stride_bytes & 15))
        return DQ_ERR_INVALID_ARG;
    if (!dq_aligned16(grads_dev) || !dq_aligned16(packed_dev) || (reinterpret_cast<uintptr_t>(norms_dev) & 3u))
        return DQ_ERR_INVALID_ARG;
    const int rc = dq_plan_check_device(plan);
    if (rc != DQ_OK) return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    // tensors without elements belong to no chunk: their norm is zero
    if (plan->n_cseg < plan->n_seg) {
        const int zrc = dq_zero_floats(norms_dev, static_cast<int64_t>(M) * plan->n_seg, stream);
        if (zrc != DQ_OK) return zrc;
    }
    if (plan->padded_elems == 0) return DQ_OK;
    return linf ? launch_width<2>(b, plan, grads_dev, worker_stride_elems, M, nullptr, seed, step, worker_base,
                                  packed_dev, packed_worker_stride_bytes, norms_dev, stream)
                : launch_width<1>(b, plan, grads_dev, worker_stride_elems, M, nullptr, seed, step, worker_base,
                                  packed_dev, packed_worker_stride_bytes, norms_dev, stream);
}
