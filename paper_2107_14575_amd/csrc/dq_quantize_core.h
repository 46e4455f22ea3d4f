// The quantize+pack work of one 4096-element chunk (Eq. (5)-(6) and the message layout), shared by
// the kernels of dq_quantize_pack.hip and dq_bracketed.hip.
#pragma once
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

// A lane's eight consecutive elements (two Philox blocks with counters quad, quad + 1): the sign
// byte (element 0 in bit 0) and the 8*B level bits (element 0 in the low B bits).  Per element, with
// a = min(|g| * scale, s) in binary32 and u = (word >> 8) * 2^-24: level = floor(a) + [u < a - floor(a)]
// (Eq. (5)-(6)).  Three routes, chosen per wavefront, all giving exactly those bits:
//   * every lane's eight products |g| * scale are zero (exact-zero stretches of a gradient, or a
//     tensor whose norm is unusable): every level is 0 whatever the random numbers, none are drawn;
//   * every product is below 1 (the usual case for a tensor of many elements: |g|/N ~ 1/sqrt(d)):
//     then a = min(a, s) = a, floor(a) = 0 and a - floor(a) = a, so the level is [u < a] -- no clamp,
//     no fract, no float-to-integer conversion;
//   * otherwise the general form: clamp, v_fract, convert, compare, add with carry.
// The wavefront-wide test costs a maximum over the eight products and two votes.
// S, b: the level count and bits of the tensor (template argument B > 0 fixes them at compile time).
// r[h][k] receives the random word of element 4h + k unless the all-zero route was taken (then no
// caller needs it: every level is zero).
template <int B>
__device__ __forceinline__ void quantize8(const float4 x_lo, const float4 x_hi, const float scale, const float S_arg,
                                          const int b_arg, const uint32_t quad, const uint32_t quad_hi,
                                          const uint32_t worker, const uint32_t step, const uint32_t key0,
                                          const uint32_t key1, uint32_t& sign, uint64_t& level, uint32_t (&r)[2][4])
{
    const float S = B > 0 ? static_cast<float>((1 << (B > 0 ? B : 1)) - 1) : S_arg;
    const int b = B > 0 ? B : b_arg;
    const float v[8] = { x_lo.x, x_lo.y, x_lo.z, x_lo.w, x_hi.x, x_hi.y, x_hi.z, x_hi.w };
    float a[8];
    sign = 0;
#pragma unroll
    for (int k = 7; k >= 0; --k) {
        sign = __builtin_amdgcn_alignbit(sign, __float_as_uint(v[k]), 31); // element 0 ends in bit 0
        a[k] = fabsf(v[k]) * scale;                                         // s|g|/N, one rounding
    }
    const float top = fmaxf(fmaxf(__builtin_fmaxf(__builtin_fmaxf(a[0], a[1]), a[2]), __builtin_fmaxf(__builtin_fmaxf(a[3], a[4]), a[5])),
                            __builtin_fmaxf(a[6], a[7]));
    level = 0;
    if (__all(top == 0.0f)) return;
    dq_philox4x32_10(quad, quad_hi, worker, step, key0, key1, r[0]);
    dq_philox4x32_10(quad + 1u, quad_hi, worker, step, key0, key1, r[1]);
    uint32_t lv[2] = { 0u, 0u };
    if (__all(top < 1.0f)) {
#pragma unroll
        for (int h = 1; h >= 0; --h)
#pragma unroll
            for (int k = 3; k >= 0; --k) {
                const float u = static_cast<float>(r[h][k] >> 8) * 0x1p-24f; // exact, in [0,1)
                lv[h] = (lv[h] << b) + (u < a[4 * h + k] ? 1u : 0u);
            }
    } else {
#pragma unroll
        for (int h = 1; h >= 0; --h)
#pragma unroll
            for (int k = 3; k >= 0; --k) {
                const float c = fminf(a[4 * h + k], S);                      // clamped
                const float p = __builtin_amdgcn_fractf(c);                  // c - floor(c), exact
                const float u = static_cast<float>(r[h][k] >> 8) * 0x1p-24f;
                lv[h] = (lv[h] << b) + static_cast<uint32_t>(c) + (u < p ? 1u : 0u);
            }
    }
    level = static_cast<uint64_t>(lv[0]) | (static_cast<uint64_t>(lv[1]) << (4 * b));
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
    int64_t packed_stride, float* __restrict__ norms_out, uint32_t chunk_index)
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
    const int64_t chunk0 = static_cast<int64_t>(chunk_index) * CHUNK;
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
        const int n_scan = dq_chunk_granule_sums<NORM == 2>(x, valid, local, static_cast<int>(tid), lds_gsum, lds_glocal,
                                                            seg_first == seg_last, static_cast<int>(n_elems >> 7));
        __syncthreads();
        if (tid < DQ_CHUNK_GRANULES)
            dq_chunk_tensor_norms<NORM == 2>(static_cast<int>(tid), n_scan, lds_gsum, lds_glocal,
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
            uint32_t sign;
            uint64_t level;
            uint32_t r[2][4];
            quantize8<B>(x[it][0], x[it][1], scale, 0.0f, 0, quad, quad_hi, worker, step, key0, key1, sign, level, r);
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
        for (uint32_t i = tid; i < n_elems / 128; i += QP_THREADS) dq_store_stream(dst + i, src[i]);
    }
    {
        uint4* dst = reinterpret_cast<uint4*>(msg + (padded_elems >> 3) + (chunk0 >> 3) * B);
        const uint4* src = reinterpret_cast<const uint4*>(lds_level);
        for (uint32_t i = tid; i < n_elems / 128 * B; i += QP_THREADS) dq_store_stream(dst + i, src[i]);
    }
}

// ---------------------------------------------------------------------------------------------
// Per-tensor widths.  Same work split; b, the level count and the place of the level bytes come
// from the widths table per segment instead of the template argument.  A chunk's level bytes are
// still one contiguous stretch of the message (every segment's stretch is a whole number of
// 16-byte pieces per granule), so they are staged and stored the same way.
// ---------------------------------------------------------------------------------------------
template <int TILES, int NORM> // NORM as in quantize_pack_chunk
__device__ __forceinline__ void quantize_pack_chunk_v(
    const float* __restrict__ grads, int64_t worker_stride, const float* __restrict__ norms, int32_t n_seg,
    const int32_t* __restrict__ granule_cseg, const int32_t* __restrict__ cseg_seg,
    const int64_t* __restrict__ cseg_valid_end, const dq_cseg_width* __restrict__ widths_table,
    int32_t widths_worker_stride, int64_t padded_elems,
    uint32_t key0, uint32_t key1, uint32_t step, uint32_t worker_base, uint8_t* __restrict__ packed,
    int64_t packed_stride, float* __restrict__ norms_out, uint32_t chunk_index)
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
    const int64_t chunk0 = static_cast<int64_t>(chunk_index) * CHUNK;
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
        const int n_scan = dq_chunk_granule_sums<NORM == 2>(x, valid, local, static_cast<int>(tid), lds_gsum, lds_glocal,
                                                            seg_first == seg_last, static_cast<int>(n_elems >> 7));
        __syncthreads();
        if (tid < DQ_CHUNK_GRANULES)
            dq_chunk_tensor_norms<NORM == 2>(static_cast<int>(tid), n_scan, lds_gsum, lds_glocal,
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
            uint32_t sign, r[2][4];
            uint64_t level;
            quantize8<0>(x[it][0], x[it][1], scale, S, b, quad, quad_hi, worker, step, key0, key1, sign, level, r);
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
        for (uint32_t i = tid; i < n_elems / 128; i += QP_THREADS) dq_store_stream(dst + i, src[i]);
    }
    {
        const int last = seg_last - seg_first;
        const uint32_t level_bytes = static_cast<uint32_t>(lds_level_base[last]) + (n_elems >> 3) * lds_b[last];
        uint4* dst = reinterpret_cast<uint4*>(msg + (padded_elems >> 3) + chunk_level0);
        const uint4* src = reinterpret_cast<const uint4*>(lds_level);
        for (uint32_t i = tid; i < level_bytes / 16; i += QP_THREADS) dq_store_stream(dst + i, src[i]);
    }
}

} // namespace
