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
#include "dq_chunk_norm.h"
#include "dq_internal.h"

namespace {

#ifndef DQ_QP_TILES
#define DQ_QP_TILES 2 // tiles of 2048 elements per workgroup
#endif

constexpr int QP_THREADS = 256;
constexpr int QP_PER_LANE = 8;
constexpr int QP_TILE = QP_THREADS * QP_PER_LANE; // 2048 elements

// Writes the low B bytes of v at dst (LDS, byte offset a multiple of B) with naturally aligned
// stores only.
template <int B>
__device__ __forceinline__ void stage_bytes(uint8_t* dst, uint64_t v)
{
    if constexpr (B == 8) {
        *reinterpret_cast<uint64_t*>(dst) = v;
    } else if constexpr (B == 4) {
        *reinterpret_cast<uint32_t*>(dst) = static_cast<uint32_t>(v);
    } else if constexpr (B % 2 == 0) {
#pragma unroll
        for (int k = 0; k < B / 2; ++k) reinterpret_cast<uint16_t*>(dst)[k] = static_cast<uint16_t>(v >> (16 * k));
    } else {
#pragma unroll
        for (int k = 0; k < B; ++k) dst[k] = static_cast<uint8_t>(v >> (8 * k));
    }
}

// Four elements (one Philox block): sign bits into bits 0..3 of `sign` (shifted in from the top
// element down), levels into a 4*B-bit little-endian field.
template <int B>
__device__ __forceinline__ void quantize4(const float4 x, const float scale, const uint32_t (&r)[4],
                                          uint32_t& sign, uint32_t& level)
{
    constexpr float S = static_cast<float>((1 << B) - 1);
    const float v[4] = { x.x, x.y, x.z, x.w };
    level = 0;
#pragma unroll
    for (int k = 3; k >= 0; --k) {
        sign = __builtin_amdgcn_alignbit(sign, __float_as_uint(v[k]), 31); // (sign << 1) | sign bit
        const float a = fminf(fabsf(v[k]) * scale, S);                     // s|g|/N, one rounding, clamped
        const float p = __builtin_amdgcn_fractf(a);                         // a - floor(a), exact
        const float u = static_cast<float>(r[k] >> 8) * 0x1p-24f;           // exact, in [0,1)
        level = (level << B) + static_cast<uint32_t>(a) + (u < p ? 1u : 0u);
    }
}

// NORM = 0: the norms are an input.  NORM = 1 (l2) or 2 (max): chunk-local plans only; the kernel
// computes the norms of its chunk's tensors itself, writes them to norms_out and quantizes from
// the registers it already holds -- one read of the gradient instead of two.
template <int B, int TILES, int NORM>
__device__ __forceinline__ void quantize_pack_chunk(
    const float* __restrict__ grads, int64_t worker_stride, const float* __restrict__ norms, int32_t n_seg,
    const int32_t* __restrict__ granule_cseg, const int32_t* __restrict__ cseg_seg,
    const int64_t* __restrict__ cseg_valid_end, int64_t padded_elems,
    uint32_t key0, uint32_t key1, uint32_t step, uint32_t worker_base, uint8_t* __restrict__ packed,
    int64_t packed_stride, float* __restrict__ norms_out)
{
    constexpr int CHUNK = QP_TILE * TILES;
    constexpr int MAX_LOCAL_SEG = CHUNK / DQ_GRANULE;
    constexpr float S = static_cast<float>((1 << B) - 1);
    static_assert(NORM == 0 || CHUNK == DQ_CHUNK, "the fused norm works on 4096-element chunks");

    __shared__ float lds_scale[MAX_LOCAL_SEG];
    __shared__ int32_t lds_valid_end[MAX_LOCAL_SEG]; // relative to the chunk, clamped to CHUNK
    __shared__ __align__(16) uint8_t lds_sign[TILES * QP_THREADS];
    __shared__ __align__(16) uint8_t lds_level[TILES * QP_THREADS * B];

    const uint32_t tid = threadIdx.x;
    const uint32_t w = blockIdx.y;
    const int64_t chunk0 = static_cast<int64_t>(blockIdx.x) * CHUNK;
    // elements of this chunk that exist (a multiple of 128, at least 128)
    const uint32_t n_elems = static_cast<uint32_t>(padded_elems - chunk0 < CHUNK ? padded_elems - chunk0 : CHUNK);
    const float* g = grads + static_cast<int64_t>(w) * worker_stride + chunk0; // uniform base
    const int32_t* gseg = granule_cseg + (chunk0 >> 7);

    // This lane's inputs first, so the loads are in flight while the segment table is built.
    // Lanes past the end of a ragged last chunk re-read its last eight elements (always in
    // bounds); what they compute is never stored.
    float4 x[TILES][2];
    int32_t seg[TILES];
#pragma unroll
    for (int it = 0; it < TILES; ++it) {
        uint32_t e = it * QP_TILE + tid * QP_PER_LANE;
        e = e < n_elems ? e : n_elems - QP_PER_LANE;
        x[it][0] = *reinterpret_cast<const float4*>(g + e);
        x[it][1] = *reinterpret_cast<const float4*>(g + e + 4);
        seg[it] = gseg[e >> 7];
    }

    // compact segment indices grow by at most one per granule, so the chunk's segments fit the table
    const int32_t seg_first = gseg[0];
    const int32_t seg_last = gseg[(n_elems - 1) >> 7];
    if constexpr (NORM == 0) {
        if (static_cast<int32_t>(tid) <= seg_last - seg_first) {
            const float N = norms[static_cast<int64_t>(w) * n_seg + cseg_seg[seg_first + tid]];
            lds_scale[tid] = N >= DQ_MIN_NORM ? S / N : 0.0f; // zero, tiny or NaN norm: every level 0
            const int64_t rel = cseg_valid_end[seg_first + tid] - chunk0;
            lds_valid_end[tid] = rel < CHUNK ? static_cast<int32_t>(rel) : CHUNK;
        }
        __syncthreads();
    } else {
        __shared__ double lds_gsum[DQ_CHUNK_GRANULES];
        __shared__ int32_t lds_glocal[DQ_CHUNK_GRANULES];
        if (static_cast<int32_t>(tid) <= seg_last - seg_first) {
            const int64_t rel = cseg_valid_end[seg_first + tid] - chunk0;
            lds_valid_end[tid] = rel < CHUNK ? static_cast<int32_t>(rel) : CHUNK;
        }
        __syncthreads();
        int valid[TILES], local[TILES];
#pragma unroll
        for (int it = 0; it < TILES; ++it) {
            const uint32_t e = it * QP_TILE + tid * QP_PER_LANE;
            local[it] = seg[it] - seg_first;
            valid[it] = e < n_elems ? lds_valid_end[local[it]] - static_cast<int32_t>(e) : 0;
        }
        dq_chunk_granule_sums<NORM == 2>(x, valid, local, static_cast<int>(tid), lds_gsum, lds_glocal);
        __syncthreads();
        if (tid < DQ_CHUNK_GRANULES)
            dq_chunk_tensor_norms<NORM == 2>(static_cast<int>(tid), static_cast<int>(n_elems >> 7), lds_gsum, lds_glocal,
                                             [&](int j, float N) {
                                                 norms_out[static_cast<int64_t>(w) * n_seg + cseg_seg[seg_first + j]] = N;
                                                 lds_scale[j] = N >= DQ_MIN_NORM ? S / N : 0.0f;
                                             });
        __syncthreads();
    }

    // Philox counter words: quad index P>>2 (low word varies per lane, high word is uniform because
    // a chunk never straddles a multiple of 2^34 elements), worker, step
    const uint32_t quad_lo0 = static_cast<uint32_t>(static_cast<uint64_t>(chunk0) >> 2);
    const uint32_t quad_hi = static_cast<uint32_t>(static_cast<uint64_t>(chunk0) >> 34);
    const uint32_t worker = worker_base + w;

#pragma unroll
    for (int it = 0; it < TILES; ++it) {
        const uint32_t e = it * QP_TILE + tid * QP_PER_LANE;
        if (e < n_elems) {
            const int local = seg[it] - seg_first;
            const float scale = lds_scale[local];
            const int32_t n_valid = lds_valid_end[local] - static_cast<int32_t>(e); // may be <= 0 or > 8

            const uint32_t quad = quad_lo0 + (e >> 2); // even; quad + 1 cannot carry
            uint32_t r0[4], r1[4];
            dq_philox4x32_10(quad, quad_hi, worker, step, key0, key1, r0);
            dq_philox4x32_10(quad + 1u, quad_hi, worker, step, key0, key1, r1);

            uint32_t sign = 0, lv_lo, lv_hi;
            quantize4<B>(x[it][1], scale, r1, sign, lv_hi); // elements 4..7 first: element 0 ends in bit 0
            quantize4<B>(x[it][0], scale, r0, sign, lv_lo);
            uint64_t level = static_cast<uint64_t>(lv_lo) | (static_cast<uint64_t>(lv_hi) << (4 * B));
            if (n_valid < QP_PER_LANE) { // the tensor ends inside (or before) this lane's eight elements
                const int nv = n_valid > 0 ? n_valid : 0;
                sign &= (1u << nv) - 1u;
                level &= (static_cast<uint64_t>(1) << (nv * B)) - 1u;
            }
            lds_sign[it * QP_THREADS + tid] = static_cast<uint8_t>(sign);
            stage_bytes<B>(&lds_level[(it * QP_THREADS + tid) * B], level);
        }
    }
    __syncthreads();

    // 16-byte stores; every plane of a chunk is a whole number of 16-byte pieces because the
    // chunk holds a multiple of 128 elements
    uint8_t* msg = packed + static_cast<int64_t>(w) * packed_stride;
    {
        uint4* dst = reinterpret_cast<uint4*>(msg + (chunk0 >> 3));
        const uint4* src = reinterpret_cast<const uint4*>(lds_sign);
        for (uint32_t i = tid; i < n_elems / 128; i += QP_THREADS) dst[i] = src[i];
    }
    {
        uint4* dst = reinterpret_cast<uint4*>(msg + (padded_elems >> 3) + (chunk0 >> 3) * B);
        const uint4* src = reinterpret_cast<const uint4*>(lds_level);
        for (uint32_t i = tid; i < n_elems / 128 * B; i += QP_THREADS) dst[i] = src[i];
    }
}

template <int B, int TILES, int NORM>
__global__ __launch_bounds__(QP_THREADS) void k_quantize_pack(
    const float* __restrict__ grads, int64_t worker_stride, const float* __restrict__ norms, int32_t n_seg,
    const int32_t* __restrict__ granule_cseg, const int32_t* __restrict__ cseg_seg,
    const int64_t* __restrict__ cseg_valid_end, int64_t padded_elems,
    uint32_t key0, uint32_t key1, uint32_t step, uint32_t worker_base, uint8_t* __restrict__ packed,
    int64_t packed_stride, float* __restrict__ norms_out)
{
    quantize_pack_chunk<B, TILES, NORM>(grads, worker_stride, norms, n_seg, granule_cseg, cseg_seg, cseg_valid_end,
                                        padded_elems, key0, key1, step, worker_base, packed, packed_stride, norms_out);
}

// ---------------------------------------------------------------------------------------------
// Per-tensor widths.  Same work split; b, the level count and the place of the level bytes come
// from the widths table per segment instead of the template argument.  A chunk's level bytes are
// still one contiguous stretch of the message (every segment's stretch is a whole number of
// 16-byte pieces per granule), so they are staged and stored the same way.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void quantize4_v(const float4 x, const float scale, const float S, const int b,
                                            const uint32_t (&r)[4], uint32_t& sign, uint32_t& level)
{
    const float v[4] = { x.x, x.y, x.z, x.w };
    level = 0;
#pragma unroll
    for (int k = 3; k >= 0; --k) {
        sign = __builtin_amdgcn_alignbit(sign, __float_as_uint(v[k]), 31);
        const float a = fminf(fabsf(v[k]) * scale, S);
        const float p = __builtin_amdgcn_fractf(a);
        const float u = static_cast<float>(r[k] >> 8) * 0x1p-24f;
        level = (level << b) + static_cast<uint32_t>(a) + (u < p ? 1u : 0u);
    }
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
    constexpr int CHUNK = QP_TILE * TILES;
    constexpr int MAX_LOCAL_SEG = CHUNK / DQ_GRANULE;
    static_assert(NORM == 0 || CHUNK == DQ_CHUNK, "the fused norm works on 4096-element chunks");
    // this worker's row of the table (stride 0: the workers share one row)
    const dq_cseg_width* __restrict__ widths = widths_table + static_cast<int64_t>(blockIdx.y) * widths_worker_stride;

    __shared__ float lds_scale[MAX_LOCAL_SEG];
    __shared__ float lds_levels[MAX_LOCAL_SEG];      // s = 2^b - 1 of the segment
    __shared__ int32_t lds_b[MAX_LOCAL_SEG];
    __shared__ int32_t lds_level_base[MAX_LOCAL_SEG]; // byte offset, in the chunk's level bytes, the
                                                      // segment's fields would have at chunk element 0
    __shared__ int32_t lds_valid_end[MAX_LOCAL_SEG];
    __shared__ __align__(16) uint8_t lds_sign[TILES * QP_THREADS];
    __shared__ __align__(16) uint8_t lds_level[TILES * QP_THREADS * 8];

    const uint32_t tid = threadIdx.x;
    const uint32_t w = blockIdx.y;
    const int64_t chunk0 = static_cast<int64_t>(blockIdx.x) * CHUNK;
    const uint32_t n_elems = static_cast<uint32_t>(padded_elems - chunk0 < CHUNK ? padded_elems - chunk0 : CHUNK);
    const float* g = grads + static_cast<int64_t>(w) * worker_stride + chunk0;
    const int32_t* gseg = granule_cseg + (chunk0 >> 7);

    float4 x[TILES][2];
    int32_t seg[TILES];
#pragma unroll
    for (int it = 0; it < TILES; ++it) {
        uint32_t e = it * QP_TILE + tid * QP_PER_LANE;
        e = e < n_elems ? e : n_elems - QP_PER_LANE;
        x[it][0] = *reinterpret_cast<const float4*>(g + e);
        x[it][1] = *reinterpret_cast<const float4*>(g + e + 4);
        seg[it] = gseg[e >> 7];
    }

    const int32_t seg_first = gseg[0];
    const int32_t seg_last = gseg[(n_elems - 1) >> 7];
    // where the chunk's level bytes start in the level plane (uniform)
    const dq_cseg_width first = widths[seg_first];
    const int64_t chunk_level0 = first.level_start + ((chunk0 - first.seg_start) >> 3) * first.b;
    if (static_cast<int32_t>(tid) <= seg_last - seg_first) {
        const dq_cseg_width e = widths[seg_first + tid];
        const float S = static_cast<float>((1 << e.b) - 1);
        if constexpr (NORM == 0) {
            const float N = norms[static_cast<int64_t>(w) * n_seg + cseg_seg[seg_first + tid]];
            lds_scale[tid] = N >= DQ_MIN_NORM ? S / N : 0.0f;
        }
        lds_levels[tid] = S;
        lds_b[tid] = e.b;
        // chunk0 - seg_start is a multiple of 128 of either sign, so the shift is exact
        lds_level_base[tid] = static_cast<int32_t>(e.level_start + ((chunk0 - e.seg_start) >> 3) * e.b - chunk_level0);
        const int64_t rel = cseg_valid_end[seg_first + tid] - chunk0;
        lds_valid_end[tid] = rel < CHUNK ? static_cast<int32_t>(rel) : CHUNK;
    }
    __syncthreads();
    if constexpr (NORM != 0) {
        __shared__ double lds_gsum[DQ_CHUNK_GRANULES];
        __shared__ int32_t lds_glocal[DQ_CHUNK_GRANULES];
        int valid[TILES], local[TILES];
#pragma unroll
        for (int it = 0; it < TILES; ++it) {
            const uint32_t e = it * QP_TILE + tid * QP_PER_LANE;
            local[it] = seg[it] - seg_first;
            valid[it] = e < n_elems ? lds_valid_end[local[it]] - static_cast<int32_t>(e) : 0;
        }
        dq_chunk_granule_sums<NORM == 2>(x, valid, local, static_cast<int>(tid), lds_gsum, lds_glocal);
        __syncthreads();
        if (tid < DQ_CHUNK_GRANULES)
            dq_chunk_tensor_norms<NORM == 2>(static_cast<int>(tid), static_cast<int>(n_elems >> 7), lds_gsum, lds_glocal,
                                             [&](int j, float N) {
                                                 norms_out[static_cast<int64_t>(w) * n_seg + cseg_seg[seg_first + j]] = N;
                                                 lds_scale[j] = N >= DQ_MIN_NORM ? lds_levels[j] / N : 0.0f;
                                             });
        __syncthreads();
    }

    const uint32_t quad_lo0 = static_cast<uint32_t>(static_cast<uint64_t>(chunk0) >> 2);
    const uint32_t quad_hi = static_cast<uint32_t>(static_cast<uint64_t>(chunk0) >> 34);
    const uint32_t worker = worker_base + w;

#pragma unroll
    for (int it = 0; it < TILES; ++it) {
        const uint32_t e = it * QP_TILE + tid * QP_PER_LANE;
        if (e < n_elems) {
            const int local = seg[it] - seg_first;
            const float scale = lds_scale[local];
            const float S = lds_levels[local];
            const int b = lds_b[local];
            const int32_t n_valid = lds_valid_end[local] - static_cast<int32_t>(e);

            const uint32_t quad = quad_lo0 + (e >> 2);
            uint32_t r0[4], r1[4];
            dq_philox4x32_10(quad, quad_hi, worker, step, key0, key1, r0);
            dq_philox4x32_10(quad + 1u, quad_hi, worker, step, key0, key1, r1);

            uint32_t sign = 0, lv_lo, lv_hi;
            quantize4_v(x[it][1], scale, S, b, r1, sign, lv_hi);
            quantize4_v(x[it][0], scale, S, b, r0, sign, lv_lo);
            uint64_t level = static_cast<uint64_t>(lv_lo) | (static_cast<uint64_t>(lv_hi) << (4 * b));
            if (n_valid < QP_PER_LANE) {
                const int nv = n_valid > 0 ? n_valid : 0;
                sign &= (1u << nv) - 1u;
                level &= (static_cast<uint64_t>(1) << (nv * b)) - 1u;
            }
            lds_sign[it * QP_THREADS + tid] = static_cast<uint8_t>(sign);
            // b bytes at an offset that is a multiple of b past a 16-byte boundary (every tensor's
            // stretch of a chunk starts on one), so the naturally aligned stores of stage_bytes apply
            uint8_t* dst = &lds_level[lds_level_base[local] + static_cast<int32_t>(e >> 3) * b];
            switch (b) {
            case 1: stage_bytes<1>(dst, level); break;
            case 2: stage_bytes<2>(dst, level); break;
            case 3: stage_bytes<3>(dst, level); break;
            case 4: stage_bytes<4>(dst, level); break;
            case 5: stage_bytes<5>(dst, level); break;
            case 6: stage_bytes<6>(dst, level); break;
            case 7: stage_bytes<7>(dst, level); break;
            default: stage_bytes<8>(dst, level); break;
            }
        }
    }
    __syncthreads();

    uint8_t* msg = packed + static_cast<int64_t>(w) * packed_stride;
    {
        uint4* dst = reinterpret_cast<uint4*>(msg + (chunk0 >> 3));
        const uint4* src = reinterpret_cast<const uint4*>(lds_sign);
        for (uint32_t i = tid; i < n_elems / 128; i += QP_THREADS) dst[i] = src[i];
    }
    {
        const int last = seg_last - seg_first;
        const uint32_t level_bytes = static_cast<uint32_t>(lds_level_base[last]) + (n_elems >> 3) * lds_b[last];
        uint4* dst = reinterpret_cast<uint4*>(msg + (padded_elems >> 3) + chunk_level0);
        const uint4* src = reinterpret_cast<const uint4*>(lds_level);
        for (uint32_t i = tid; i < level_bytes / 16; i += QP_THREADS) dst[i] = src[i];
    }
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
    for (uint32_t i = tid; i < n_elems / 128; i += QP_THREADS) dst[i] = src[i];
}

// ---------------------------------------------------------------------------------------------
// One pass over the gradient for ANY plan when each norm is known beforehand to lie in a bracket
// [lo, hi] (say, last iteration's norm give or take a margin) and b is known (Algorithm 1).
//
// For a fixed element and random number the level of Eq. (5)-(6) never grows with the norm:
// s/N rounded to binary32 does not grow with N, |g| * scale rounded does not grow when the scale
// shrinks, and a -> floor(a) + [u < a - floor(a)] never decreases in a (inside one integer interval
// the indicator can only switch on; across intervals floor(a) + 1 <= floor(a')).  So an element
// whose level is the same at both ends of the bracket has that level for every norm inside it.
//
//   k_quantize_pack_bracketed  reads the gradient once: adds up each tensor's squares chunk by
//       chunk (binary64 partial sums, one slot per chunk and tensor), quantizes with both ends of
//       the bracket, writes the decided levels, leaves the undecided fields zero and records those
//       elements (index and value) in the chunk's block of the workspace.
//   k_bracket_norm_finish      adds a tensor's partial sums in a fixed order: the norms.
//   k_bracket_fixup            per chunk: quantizes the recorded elements with the true norm and
//       ORs their levels into the zero fields; a chunk with too many records, with no usable
//       bracket, or whose norm fell outside the bracket is quantized again in full from the
//       gradient (the only case that reads it twice).
// The messages are exactly those of dq_quantize_pack for the norms this path computes.
// ---------------------------------------------------------------------------------------------
template <int B>
__global__ __launch_bounds__(QP_THREADS) void k_quantize_pack_bracketed(
    const float* __restrict__ grads, int64_t worker_stride, const float* __restrict__ norm_lo,
    const float* __restrict__ norm_hi, int32_t n_seg, const int32_t* __restrict__ granule_cseg,
    const int32_t* __restrict__ cseg_seg, const int64_t* __restrict__ cseg_valid_end, int64_t padded_elems,
    uint32_t key0, uint32_t key1, uint32_t step, uint32_t worker_base, uint8_t* __restrict__ packed,
    int64_t packed_stride, double* __restrict__ partials, int64_t n_slots, dq_bracket_block* __restrict__ blocks,
    int64_t n_chunks)
{
    constexpr int TILES = 2;
    constexpr int CHUNK = DQ_CHUNK;
    constexpr float S = static_cast<float>((1 << B) - 1);
    constexpr uint64_t FIELD = (static_cast<uint64_t>(1) << B) - 1u;

    __shared__ float lds_scale_hi[DQ_CHUNK_GRANULES]; // s / lo: the larger scale
    __shared__ float lds_scale_lo[DQ_CHUNK_GRANULES]; // s / hi
    __shared__ int32_t lds_valid_end[DQ_CHUNK_GRANULES];
    __shared__ double lds_gsum[DQ_CHUNK_GRANULES];
    __shared__ int32_t lds_glocal[DQ_CHUNK_GRANULES];
    __shared__ uint32_t lds_count;
    __shared__ __align__(16) uint8_t lds_sign[TILES * QP_THREADS];
    __shared__ __align__(16) uint8_t lds_level[TILES * QP_THREADS * B];

    const uint32_t tid = threadIdx.x;
    const uint32_t w = blockIdx.y;
    const int64_t chunk0 = static_cast<int64_t>(blockIdx.x) * CHUNK;
    const uint32_t n_elems = static_cast<uint32_t>(padded_elems - chunk0 < CHUNK ? padded_elems - chunk0 : CHUNK);
    const float* g = grads + static_cast<int64_t>(w) * worker_stride + chunk0;
    const int32_t* gseg = granule_cseg + (chunk0 >> 7);
    dq_bracket_block* blk = blocks + static_cast<int64_t>(w) * n_chunks + blockIdx.x;

    float4 x[TILES][2];
    int32_t seg[TILES];
#pragma unroll
    for (int it = 0; it < TILES; ++it) {
        uint32_t e = it * QP_TILE + tid * QP_PER_LANE;
        e = e < n_elems ? e : n_elems - QP_PER_LANE; // clamped: always in bounds, result unused
        x[it][0] = *reinterpret_cast<const float4*>(g + e);
        x[it][1] = *reinterpret_cast<const float4*>(g + e + 4);
        seg[it] = gseg[e >> 7];
    }

    const int32_t seg_first = gseg[0];
    const int32_t seg_last = gseg[(n_elems - 1) >> 7];
    if (tid == 0) lds_count = 0;
    int unusable = 0;
    if (static_cast<int32_t>(tid) <= seg_last - seg_first) {
        const int64_t at = static_cast<int64_t>(w) * n_seg + cseg_seg[seg_first + tid];
        const float lo = norm_lo[at], hi = norm_hi[at];
        // the zero path (norm below DQ_MIN_NORM) is not monotone against the rest: no bracket across it
        const bool ok = lo >= DQ_MIN_NORM && hi >= lo && hi <= 3.0e38f; // false for NaN
        lds_scale_hi[tid] = ok ? S / lo : 0.0f;
        lds_scale_lo[tid] = ok ? S / hi : 0.0f;
        unusable = ok ? 0 : 1;
        const int64_t rel = cseg_valid_end[seg_first + tid] - chunk0;
        lds_valid_end[tid] = rel < CHUNK ? static_cast<int32_t>(rel) : CHUNK;
    }
    const int skip = __syncthreads_or(unusable); // also the barrier after the tables

    // partial sums of squares of the chunk's tensors
    int valid[TILES], local[TILES];
#pragma unroll
    for (int it = 0; it < TILES; ++it) {
        const uint32_t e = it * QP_TILE + tid * QP_PER_LANE;
        local[it] = seg[it] - seg_first;
        valid[it] = e < n_elems ? lds_valid_end[local[it]] - static_cast<int32_t>(e) : 0;
    }
    dq_chunk_granule_sums<false>(x, valid, local, static_cast<int>(tid), lds_gsum, lds_glocal);
    __syncthreads();
    if (tid < DQ_CHUNK_GRANULES)
        dq_chunk_tensor_totals<false>(static_cast<int>(tid), static_cast<int>(n_elems >> 7), lds_gsum, lds_glocal,
                                      [&](int j, double total) {
                                          partials[static_cast<int64_t>(w) * n_slots + blockIdx.x + seg_first + j] = total;
                                      });
    if (skip) { // uniform: the fix-up kernel quantizes this chunk from the gradient
        if (tid == 0) {
            blk->count = 0;
            blk->flags = 1;
        }
        return;
    }

    const uint32_t quad_lo0 = static_cast<uint32_t>(static_cast<uint64_t>(chunk0) >> 2);
    const uint32_t quad_hi = static_cast<uint32_t>(static_cast<uint64_t>(chunk0) >> 34);
    const uint32_t worker = worker_base + w;

#pragma unroll
    for (int it = 0; it < TILES; ++it) {
        const uint32_t e = it * QP_TILE + tid * QP_PER_LANE;
        if (e < n_elems) {
            const uint32_t quad = quad_lo0 + (e >> 2);
            uint32_t r0[4], r1[4];
            dq_philox4x32_10(quad, quad_hi, worker, step, key0, key1, r0);
            dq_philox4x32_10(quad + 1u, quad_hi, worker, step, key0, key1, r1);

            // levels at the low end of the bracket: the largest any norm inside it can give
            uint32_t sign = 0, lv_lo, lv_hi;
            quantize4<B>(x[it][1], lds_scale_hi[local[it]], r1, sign, lv_hi);
            quantize4<B>(x[it][0], lds_scale_hi[local[it]], r0, sign, lv_lo);
            uint64_t level = static_cast<uint64_t>(lv_lo) | (static_cast<uint64_t>(lv_hi) << (4 * B));
            const int nv = valid[it] >= QP_PER_LANE ? QP_PER_LANE : (valid[it] > 0 ? valid[it] : 0);
            if (nv < QP_PER_LANE) {
                sign &= (1u << nv) - 1u;
                level &= (static_cast<uint64_t>(1) << (nv * B)) - 1u;
            }
            if (level != 0) { // all zero at the low end: zero everywhere in the bracket
                uint32_t unused = 0, lw_lo, lw_hi;
                quantize4<B>(x[it][1], lds_scale_lo[local[it]], r1, unused, lw_hi);
                quantize4<B>(x[it][0], lds_scale_lo[local[it]], r0, unused, lw_lo);
                uint64_t smallest = static_cast<uint64_t>(lw_lo) | (static_cast<uint64_t>(lw_hi) << (4 * B));
                if (nv < QP_PER_LANE) smallest &= (static_cast<uint64_t>(1) << (nv * B)) - 1u;
                const uint64_t differ = level ^ smallest;
                if (differ != 0) {
                    const float v[8] = { x[it][0].x, x[it][0].y, x[it][0].z, x[it][0].w,
                                         x[it][1].x, x[it][1].y, x[it][1].z, x[it][1].w };
#pragma unroll
                    for (int k = 0; k < QP_PER_LANE; ++k) {
                        if ((differ >> (k * B)) & FIELD) {
                            const uint32_t slot = atomicAdd(&lds_count, 1u);
                            if (slot < DQ_BRACKET_CAP) blk->rec[slot] = make_uint2(e + k, __float_as_uint(v[k]));
                            level &= ~(FIELD << (k * B)); // left zero for the fix-up kernel
                        }
                    }
                }
            }
            lds_sign[it * QP_THREADS + tid] = static_cast<uint8_t>(sign);
            stage_bytes<B>(&lds_level[(it * QP_THREADS + tid) * B], level);
        }
    }
    __syncthreads();

    uint8_t* msg = packed + static_cast<int64_t>(w) * packed_stride;
    {
        uint4* dst = reinterpret_cast<uint4*>(msg + (chunk0 >> 3));
        const uint4* src = reinterpret_cast<const uint4*>(lds_sign);
        for (uint32_t i = tid; i < n_elems / 128; i += QP_THREADS) dst[i] = src[i];
    }
    {
        uint4* dst = reinterpret_cast<uint4*>(msg + (padded_elems >> 3) + (chunk0 >> 3) * B);
        const uint4* src = reinterpret_cast<const uint4*>(lds_level);
        for (uint32_t i = tid; i < n_elems / 128 * B; i += QP_THREADS) dst[i] = src[i];
    }
    if (tid == 0) {
        blk->count = lds_count;
        blk->flags = 0;
    }
}

// grid (n_cseg, M): the norm of tensor c of worker w from its partial sums, slots
// [first chunk + c, last chunk + c], added lane-strided and then by a fixed tree.
__global__ __launch_bounds__(256) void k_bracket_norm_finish(const double* __restrict__ partials, int64_t n_slots,
                                                             const int64_t* __restrict__ cseg_start,
                                                             const int64_t* __restrict__ cseg_valid_end,
                                                             const int32_t* __restrict__ cseg_seg, int32_t n_seg,
                                                             float* __restrict__ norms, unsigned long long* __restrict__ stats)
{
    __shared__ double part[256];
    const int tid = threadIdx.x;
    const int32_t c = blockIdx.x;
    const int w = blockIdx.y;
    const int64_t first = cseg_start[c] / DQ_CHUNK;
    const int64_t last = (cseg_valid_end[c] - 1) / DQ_CHUNK;
    const double* p = partials + static_cast<int64_t>(w) * n_slots + first + c;
    const int64_t n = last - first + 1;
    double acc = 0.0;
    for (int64_t i = tid; i < n; i += 256) acc += p[i];
    part[tid] = acc;
    __syncthreads();
    for (int off = 128; off >= 1; off >>= 1) {
        if (tid < off) part[tid] += part[tid + off];
        __syncthreads();
    }
    if (tid == 0) {
        norms[static_cast<int64_t>(w) * n_seg + cseg_seg[c]] = static_cast<float>(sqrt(part[0]));
        if (stats && c == 0 && w == 0) {
            stats[0] = 0; // the fix-up kernel, next on the stream, counts into these
            stats[1] = 0;
        }
    }
}

template <int B>
__global__ __launch_bounds__(QP_THREADS) void k_bracket_fixup(
    const float* __restrict__ grads, int64_t worker_stride, const float* __restrict__ norms,
    const float* __restrict__ norm_lo, const float* __restrict__ norm_hi, int32_t n_seg,
    const int32_t* __restrict__ granule_cseg, const int32_t* __restrict__ cseg_seg,
    const int64_t* __restrict__ cseg_valid_end, int64_t padded_elems, uint32_t key0, uint32_t key1, uint32_t step,
    uint32_t worker_base, uint8_t* __restrict__ packed, int64_t packed_stride,
    const dq_bracket_block* __restrict__ blocks, int64_t n_chunks, unsigned long long* __restrict__ stats)
{
    constexpr float S = static_cast<float>((1 << B) - 1);
    const uint32_t tid = threadIdx.x;
    const uint32_t w = blockIdx.y;
    const int64_t chunk0 = static_cast<int64_t>(blockIdx.x) * DQ_CHUNK;
    const uint32_t n_elems = static_cast<uint32_t>(padded_elems - chunk0 < DQ_CHUNK ? padded_elems - chunk0 : DQ_CHUNK);
    const int32_t* gseg = granule_cseg + (chunk0 >> 7);
    const dq_bracket_block* blk = blocks + static_cast<int64_t>(w) * n_chunks + blockIdx.x;
    const uint32_t count = blk->count, flags = blk->flags;

    const int32_t seg_first = gseg[0];
    const int32_t seg_last = gseg[(n_elems - 1) >> 7];
    int outside = 0;
    if (static_cast<int32_t>(tid) <= seg_last - seg_first) {
        const int64_t at = static_cast<int64_t>(w) * n_seg + cseg_seg[seg_first + tid];
        const float N = norms[at];
        outside = (N >= norm_lo[at] && N <= norm_hi[at]) ? 0 : 1;
    }
    const int again = __syncthreads_or(outside) || flags != 0 || count > DQ_BRACKET_CAP;
    if (!again) {
        if (tid < count) {
            const uint2 rec = blk->rec[tid];
            const uint32_t e = rec.x; // < n_elems: written by the first kernel for this very chunk
            const float gv = __uint_as_float(rec.y);
            const float N = norms[static_cast<int64_t>(w) * n_seg + cseg_seg[gseg[e >> 7]]];
            const float scale = N >= DQ_MIN_NORM ? S / N : 0.0f;
            const uint64_t P = static_cast<uint64_t>(chunk0) + e;
            uint32_t r[4];
            dq_philox4x32_10(static_cast<uint32_t>(P >> 2), static_cast<uint32_t>(P >> 34), worker_base + w, step, key0,
                             key1, r);
            const uint32_t word = (P & 2u) ? ((P & 1u) ? r[3] : r[2]) : ((P & 1u) ? r[1] : r[0]);
            const float a = fminf(fabsf(gv) * scale, S);
            const float p = __builtin_amdgcn_fractf(a);
            const float u = static_cast<float>(word >> 8) * 0x1p-24f;
            const uint32_t level = static_cast<uint32_t>(a) + (u < p ? 1u : 0u);
            if (level != 0) {
                // the field was left zero; fields of other elements in the same words are not touched
                uint32_t* plane = reinterpret_cast<uint32_t*>(packed + static_cast<int64_t>(w) * packed_stride +
                                                              (padded_elems >> 3));
                const uint64_t bit = P * B;
                const uint32_t sh = static_cast<uint32_t>(bit & 31u);
                atomicOr(plane + (bit >> 5), level << sh);
                if (sh + B > 32) atomicOr(plane + (bit >> 5) + 1, level >> (32 - sh));
            }
        }
        if (tid == 0 && count != 0 && stats) atomicAdd(&stats[0], static_cast<unsigned long long>(count));
        return;
    }
    if (tid == 0 && stats) atomicAdd(&stats[1], 1ull);
    quantize_pack_chunk<B, 2, 0>(grads, worker_stride, norms, n_seg, granule_cseg, cseg_seg, cseg_valid_end, padded_elems,
                                 key0, key1, step, worker_base, packed, packed_stride, nullptr);
}

template <int B>
int launch_bracketed(const dq_plan* plan, const float* grads, int64_t worker_stride, int M, const float* norm_lo,
                     const float* norm_hi, uint64_t seed, uint32_t step, uint32_t worker_base, float* norms,
                     uint8_t* packed, int64_t packed_stride, void* workspace, unsigned long long* stats,
                     hipStream_t stream)
{
    const int64_t n_chunks = (plan->padded_elems + DQ_CHUNK - 1) / DQ_CHUNK;
    if (n_chunks > INT32_MAX) return DQ_ERR_INVALID_ARG;
    const int64_t n_slots = dq_bracket_slots(plan);
    double* partials = static_cast<double*>(workspace);
    dq_bracket_block* blocks =
        reinterpret_cast<dq_bracket_block*>(static_cast<uint8_t*>(workspace) + dq_bracket_partial_bytes(plan, M));
    const dim3 grid(static_cast<unsigned>(n_chunks), M), block(QP_THREADS);
    const uint32_t key0 = static_cast<uint32_t>(seed), key1 = static_cast<uint32_t>(seed >> 32);
    hipLaunchKernelGGL(k_quantize_pack_bracketed<B>, grid, block, 0, stream, grads, worker_stride, norm_lo, norm_hi,
                       plan->n_seg, plan->d_granule_cseg, plan->d_cseg_seg, plan->d_cseg_valid_end, plan->padded_elems,
                       key0, key1, step, worker_base, packed, packed_stride, partials, n_slots, blocks, n_chunks);
    hipLaunchKernelGGL(k_bracket_norm_finish, dim3(plan->n_cseg, M), dim3(256), 0, stream, partials, n_slots,
                       plan->d_cseg_start, plan->d_cseg_valid_end, plan->d_cseg_seg, plan->n_seg, norms, stats);
    hipLaunchKernelGGL(k_bracket_fixup<B>, grid, block, 0, stream, grads, worker_stride, norms, norm_lo, norm_hi,
                       plan->n_seg, plan->d_granule_cseg, plan->d_cseg_seg, plan->d_cseg_valid_end, plan->padded_elems,
                       key0, key1, step, worker_base, packed, packed_stride, blocks, n_chunks, stats);
    return hipGetLastError() == hipSuccess ? DQ_OK : DQ_ERR_HIP;
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

extern "C" int64_t dq_bracketed_workspace_bytes(const dq_plan_t* plan, int M)
{
    if (!plan || M < 1 || M > DQ_MAX_WORKERS) return -1;
    const int64_t n_chunks = (plan->padded_elems + DQ_CHUNK - 1) / DQ_CHUNK;
    const int64_t bytes = dq_bracket_partial_bytes(plan, M) +
                          static_cast<int64_t>(M) * n_chunks * static_cast<int64_t>(sizeof(dq_bracket_block));
    return bytes < 256 ? 256 : bytes;
}

extern "C" int dq_norm_quantize_pack_bracketed(const dq_plan_t* plan, const float* grads_dev,
                                               int64_t worker_stride_elems, int M, const float* norm_lo_dev,
                                               const float* norm_hi_dev, int b, uint64_t seed, uint32_t step,
                                               uint32_t worker_base, float* norms_dev, uint8_t* packed_dev,
                                               int64_t packed_worker_stride_bytes, void* workspace_dev,
                                               int64_t* stats_dev, void* hip_stream)
{
    if (!plan || !grads_dev || !norm_lo_dev || !norm_hi_dev || !norms_dev || !packed_dev || !workspace_dev)
        return DQ_ERR_INVALID_ARG;
    if (M < 1 || M > DQ_MAX_WORKERS || b < 1 || b > 8) return DQ_ERR_INVALID_ARG;
    if (worker_stride_elems < plan->padded_elems || (worker_stride_elems & 3)) return DQ_ERR_INVALID_ARG;
    if (packed_worker_stride_bytes < dq_packed_bytes(plan, b) || (packed_worker_stride_bytes & 15))
        return DQ_ERR_INVALID_ARG;
    if (!dq_aligned16(grads_dev) || !dq_aligned16(packed_dev) || !dq_aligned16(workspace_dev)) return DQ_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(norm_lo_dev) & 3u) || (reinterpret_cast<uintptr_t>(norm_hi_dev) & 3u) ||
        (reinterpret_cast<uintptr_t>(norms_dev) & 3u) || (reinterpret_cast<uintptr_t>(stats_dev) & 7u))
        return DQ_ERR_INVALID_ARG;
    const int rc = dq_plan_check_device(plan);
    if (rc != DQ_OK) return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (plan->n_cseg < plan->n_seg) { // tensors without elements: norm zero
        const int zrc = dq_zero_floats(norms_dev, static_cast<int64_t>(M) * plan->n_seg, stream);
        if (zrc != DQ_OK) return zrc;
    }
    if (plan->padded_elems == 0) return DQ_OK;
    unsigned long long* stats = reinterpret_cast<unsigned long long*>(stats_dev);
#define DQ_BRACKETED(B)                                                                                              \
    case B:                                                                                                          \
        return launch_bracketed<B>(plan, grads_dev, worker_stride_elems, M, norm_lo_dev, norm_hi_dev, seed, step,   \
                                   worker_base, norms_dev, packed_dev, packed_worker_stride_bytes, workspace_dev,   \
                                   stats, stream)
    switch (b) {
        DQ_BRACKETED(1);
        DQ_BRACKETED(2);
        DQ_BRACKETED(3);
        DQ_BRACKETED(4);
        DQ_BRACKETED(5);
        DQ_BRACKETED(6);
        DQ_BRACKETED(7);
    default:
        DQ_BRACKETED(8);
    }
#undef DQ_BRACKETED
}
