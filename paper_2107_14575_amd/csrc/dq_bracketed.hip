// dq_norm_quantize_pack_bracketed: norms and messages in one pass over the gradient for ANY plan,
// given a bracket [lo, hi] for every norm (say, last iteration's norm give or take a margin) and a
// bit-width that is known beforehand (Algorithm 1: the worker received b_t with x_t).
//
// For a fixed element and random number the level of Eq. (5)-(6) never grows with the norm:
// s/N rounded to binary32 does not grow with N, |g| * scale rounded does not grow when the scale
// shrinks, and a -> floor(a) + [u < a - floor(a)] never decreases in a (inside one integer interval
// the indicator can only switch on; across intervals floor(a) + 1 <= floor(a')).  So an element
// whose level is the same at both ends of the bracket has that level for every norm inside it.
//
//   k_quantize_pack_bracketed  reads the gradient once: adds up each tensor's squares chunk by
//       chunk (binary64 partial sums, one slot per chunk and tensor).  A tensor that lies wholly
//       inside the chunk needs no bracket: its norm is finished on the spot and used.  For the
//       others the kernel quantizes with the low end
//       of the bracket (the largest levels), looks at the non-zero levels again with the high end,
//       writes the levels that agree, leaves the others' fields zero and records those elements
//       (index and value) in the chunk's block of the workspace.
//   k_bracket_norm_finish      for the tensors that cross a chunk boundary: adds the partial sums in
//       a fixed order: the norms, and whether each came out inside its bracket.
//   k_bracket_settle[_wide]    one lane per chunk (large plans) or one wavefront per chunk with a
//       lane per record (up to 2^16 chunks): quantizes the chunk's recorded elements with the
//       true norm and ORs their levels into the zero fields; a chunk with too many records, with
//       no usable bracket, or with a norm outside its bracket gets a bit in the redo map instead.
//   k_bracket_redo             quantizes the chunks of the redo map again in full from the
//       gradient (the only case that reads it twice); a few thousand workgroups walk the map, so
//       an empty map costs next to nothing.
// The messages are exactly those of dq_quantize_pack for the norms this path computes.
#include "dq_quantize_core.h"

namespace {

// One element again with another scale: the level of Eq. (5)-(6) for element value v and random word r.
template <int B>
__device__ __forceinline__ uint32_t level_of(float v, float scale, uint32_t r)
{
    constexpr float S = static_cast<float>((1 << B) - 1);
    const float a = fminf(fabsf(v) * scale, S);
    const float p = __builtin_amdgcn_fractf(a);
    const float u = static_cast<float>(r >> 8) * 0x1p-24f;
    return static_cast<uint32_t>(a) + (u < p ? 1u : 0u);
}

// The same with the level count as a value (per-tensor widths).
__device__ __forceinline__ uint32_t level_of_s(float v, float scale, float S, uint32_t r)
{
    const float a = fminf(fabsf(v) * scale, S);
    const float p = __builtin_amdgcn_fractf(a);
    const float u = static_cast<float>(r >> 8) * 0x1p-24f;
    return static_cast<uint32_t>(a) + (u < p ? 1u : 0u);
}

template <int B, bool LINF> // LINF: the max norm (p = infinity in Eq. (5)) instead of the l2 norm
__global__ __launch_bounds__(QP_THREADS) void k_quantize_pack_bracketed(
    const float* __restrict__ grads, int64_t worker_stride, const float* __restrict__ norm_lo,
    const float* __restrict__ norm_hi, int32_t n_seg, const int32_t* __restrict__ granule_cseg,
    const int32_t* __restrict__ cseg_seg, const int64_t* __restrict__ cseg_start,
    const int64_t* __restrict__ cseg_valid_end, int64_t padded_elems, uint32_t key0, uint32_t key1, uint32_t step,
    uint32_t worker_base, uint8_t* __restrict__ packed, int64_t packed_stride, double* __restrict__ partials,
    int64_t n_slots, dq_bracket_block* __restrict__ blocks, int64_t n_chunks, float* __restrict__ norms_out,
    uint8_t* __restrict__ inside, int32_t n_cseg)
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
    __shared__ int32_t lds_whole[DQ_CHUNK_GRANULES]; // the tensor lies wholly inside this chunk
    __shared__ int32_t lds_any_whole;
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
    int unusable = 0, whole_here = 0;
    if (static_cast<int32_t>(tid) <= seg_last - seg_first) { // at most 32 lanes, all in the first wavefront
        const int64_t at = static_cast<int64_t>(w) * n_seg + cseg_seg[seg_first + tid];
        const int64_t valid_end = cseg_valid_end[seg_first + tid];
        const bool whole = cseg_start[seg_first + tid] >= chunk0 && valid_end <= chunk0 + CHUNK;
        const float lo = norm_lo[at], hi = norm_hi[at];
        // the zero path (norm below DQ_MIN_NORM) is not monotone against the rest: no bracket across it
        const bool ok = lo >= DQ_MIN_NORM && hi >= lo && hi <= 3.0e38f; // false for NaN
        lds_scale_hi[tid] = ok ? S / lo : 0.0f; // replaced below for a tensor that is whole
        lds_scale_lo[tid] = ok ? S / hi : 0.0f;
        lds_whole[tid] = whole ? 1 : 0;
        whole_here = whole ? 1 : 0;
        unusable = (ok || whole) ? 0 : 1;
        const int64_t rel = valid_end - chunk0;
        lds_valid_end[tid] = rel < CHUNK ? static_cast<int32_t>(rel) : CHUNK;
    }
    // one lane writes both words: the first wavefront's vote says whether any tensor is whole
    const bool first_wave_any_whole = __ballot(whole_here) != 0;
    if (tid == 0) {
        lds_count = 0;
        lds_any_whole = first_wave_any_whole ? 1 : 0;
    }
    const int skip = __syncthreads_or(unusable); // also the barrier after the tables
    const bool any_whole = lds_any_whole != 0;

    // partial sums of squares (or maxima) of the chunk's tensors
    int valid[TILES], local[TILES];
#pragma unroll
    for (int it = 0; it < TILES; ++it) {
        const uint32_t e = it * QP_TILE + tid * QP_PER_LANE;
        local[it] = seg[it] - seg_first;
        valid[it] = e < n_elems ? lds_valid_end[local[it]] - static_cast<int32_t>(e) : 0;
    }
    const int n_scan = dq_chunk_granule_sums<LINF>(x, valid, local, static_cast<int>(tid), lds_gsum, lds_glocal,
                                                   seg_first == seg_last, static_cast<int>(n_elems >> 7));
    __syncthreads();
    if (tid < DQ_CHUNK_GRANULES)
        dq_chunk_tensor_totals<LINF>(static_cast<int>(tid), n_scan, lds_gsum, lds_glocal,
                                      [&](int j, double total) {
                                          partials[static_cast<int64_t>(w) * n_slots + blockIdx.x + seg_first + j] = total;
                                          if (lds_whole[j]) { // all of the tensor is here: this is its norm, no bracket involved
                                              const float N = LINF ? static_cast<float>(total) : static_cast<float>(sqrt(total));
                                              norms_out[static_cast<int64_t>(w) * n_seg + cseg_seg[seg_first + j]] = N;
                                              inside[static_cast<int64_t>(w) * n_cseg + seg_first + j] = 1;
                                              const float scale = N >= DQ_MIN_NORM ? S / N : 0.0f;
                                              lds_scale_hi[j] = scale;
                                              lds_scale_lo[j] = scale;
                                          }
                                      });
    if (any_whole) __syncthreads(); // uniform: scales written just above
    if (skip) { // uniform: the redo kernel quantizes this chunk from the gradient
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
            // levels at the low end of the bracket: the largest any norm inside it can give
            uint32_t sign, rr[2][4];
            uint64_t level;
            quantize8<B>(x[it][0], x[it][1], lds_scale_hi[local[it]], 0.0f, 0, quad, quad_hi, worker, step, key0, key1,
                         sign, level, rr);
            const int nv = valid[it] >= QP_PER_LANE ? QP_PER_LANE : (valid[it] > 0 ? valid[it] : 0);
            if (nv < QP_PER_LANE) {
                sign &= (1u << nv) - 1u;
                level &= (static_cast<uint64_t>(1) << (nv * B)) - 1u;
            }
            if (level != 0) { // a zero at the low end is a zero everywhere in the bracket
                const float scale_lo = lds_scale_lo[local[it]];
                const float v[8] = { x[it][0].x, x[it][0].y, x[it][0].z, x[it][0].w,
                                     x[it][1].x, x[it][1].y, x[it][1].z, x[it][1].w };
                const uint32_t r[8] = { rr[0][0], rr[0][1], rr[0][2], rr[0][3], rr[1][0], rr[1][1], rr[1][2], rr[1][3] };
#pragma unroll
                for (int k = 0; k < QP_PER_LANE; ++k) {
                    const uint32_t top = static_cast<uint32_t>(level >> (k * B)) & static_cast<uint32_t>(FIELD);
                    if (top != 0 && level_of<B>(v[k], scale_lo, r[k]) != top) {
                        const uint32_t slot = atomicAdd(&lds_count, 1u);
                        if (slot < DQ_BRACKET_CAP) blk->rec[slot] = make_uint2(e + k, __float_as_uint(v[k]));
                        level &= ~(FIELD << (k * B)); // left zero for the settle kernel
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
        for (uint32_t i = tid; i < n_elems / 128; i += QP_THREADS) dq_store_stream(dst + i, src[i]);
    }
    {
        uint4* dst = reinterpret_cast<uint4*>(msg + (padded_elems >> 3) + (chunk0 >> 3) * B);
        const uint4* src = reinterpret_cast<const uint4*>(lds_level);
        for (uint32_t i = tid; i < n_elems / 128 * B; i += QP_THREADS) dq_store_stream(dst + i, src[i]);
    }
    if (tid == 0) {
        blk->count = lds_count;
        blk->flags = 0;
    }
}

// The first kernel with per-tensor widths (dq_widths_t: one row shared by the workers or one row per
// worker): b, the level count and the place of the level bytes of every tensor the chunk touches
// come from the widths table, as in quantize_pack_chunk_v; everything else as above.
template <bool LINF>
__global__ __launch_bounds__(QP_THREADS) void k_quantize_pack_bracketed_v(
    const float* __restrict__ grads, int64_t worker_stride, const float* __restrict__ norm_lo,
    const float* __restrict__ norm_hi, int32_t n_seg, const int32_t* __restrict__ granule_cseg,
    const int32_t* __restrict__ cseg_seg, const int64_t* __restrict__ cseg_start,
    const int64_t* __restrict__ cseg_valid_end, const dq_cseg_width* __restrict__ widths_table,
    int32_t widths_worker_stride, int64_t padded_elems, uint32_t key0, uint32_t key1, uint32_t step,
    uint32_t worker_base, uint8_t* __restrict__ packed, int64_t packed_stride, double* __restrict__ partials,
    int64_t n_slots, dq_bracket_block* __restrict__ blocks, int64_t n_chunks, float* __restrict__ norms_out,
    uint8_t* __restrict__ inside, int32_t n_cseg)
{
    constexpr int TILES = 2;
    constexpr int CHUNK = DQ_CHUNK;
    const dq_cseg_width* __restrict__ widths = widths_table + static_cast<int64_t>(blockIdx.y) * widths_worker_stride;

    __shared__ float lds_scale_hi[DQ_CHUNK_GRANULES];
    __shared__ float lds_scale_lo[DQ_CHUNK_GRANULES];
    __shared__ float lds_levels[DQ_CHUNK_GRANULES]; // s = 2^b - 1 of the tensor
    __shared__ int32_t lds_b[DQ_CHUNK_GRANULES];
    __shared__ int32_t lds_level_base[DQ_CHUNK_GRANULES];
    __shared__ int32_t lds_valid_end[DQ_CHUNK_GRANULES];
    __shared__ double lds_gsum[DQ_CHUNK_GRANULES];
    __shared__ int32_t lds_glocal[DQ_CHUNK_GRANULES];
    __shared__ uint32_t lds_count;
    __shared__ int32_t lds_whole[DQ_CHUNK_GRANULES];
    __shared__ int32_t lds_any_whole;
    __shared__ __align__(16) uint8_t lds_sign[TILES * QP_THREADS];
    __shared__ __align__(16) uint8_t lds_level[TILES * QP_THREADS * 8];

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
        e = e < n_elems ? e : n_elems - QP_PER_LANE;
        x[it][0] = *reinterpret_cast<const float4*>(g + e);
        x[it][1] = *reinterpret_cast<const float4*>(g + e + 4);
        seg[it] = gseg[e >> 7];
    }

    const int32_t seg_first = gseg[0];
    const int32_t seg_last = gseg[(n_elems - 1) >> 7];
    const dq_cseg_width first = widths[seg_first];
    const int64_t chunk_level0 = first.level_start + ((chunk0 - first.seg_start) >> 3) * first.b;
    int unusable = 0, whole_here = 0;
    if (static_cast<int32_t>(tid) <= seg_last - seg_first) { // at most 32 lanes, all in the first wavefront
        const dq_cseg_width e = widths[seg_first + tid];
        const float S = static_cast<float>((1 << e.b) - 1);
        const int64_t at = static_cast<int64_t>(w) * n_seg + cseg_seg[seg_first + tid];
        const int64_t valid_end = cseg_valid_end[seg_first + tid];
        const bool whole = cseg_start[seg_first + tid] >= chunk0 && valid_end <= chunk0 + CHUNK;
        const float lo = norm_lo[at], hi = norm_hi[at];
        const bool ok = lo >= DQ_MIN_NORM && hi >= lo && hi <= 3.0e38f;
        lds_scale_hi[tid] = ok ? S / lo : 0.0f;
        lds_scale_lo[tid] = ok ? S / hi : 0.0f;
        lds_levels[tid] = S;
        lds_b[tid] = e.b;
        lds_level_base[tid] = static_cast<int32_t>(e.level_start + ((chunk0 - e.seg_start) >> 3) * e.b - chunk_level0);
        lds_whole[tid] = whole ? 1 : 0;
        whole_here = whole ? 1 : 0;
        unusable = (ok || whole) ? 0 : 1;
        const int64_t rel = valid_end - chunk0;
        lds_valid_end[tid] = rel < CHUNK ? static_cast<int32_t>(rel) : CHUNK;
    }
    const bool first_wave_any_whole = __ballot(whole_here) != 0;
    if (tid == 0) {
        lds_count = 0;
        lds_any_whole = first_wave_any_whole ? 1 : 0;
    }
    const int skip = __syncthreads_or(unusable);
    const bool any_whole = lds_any_whole != 0;

    int valid[TILES], local[TILES];
#pragma unroll
    for (int it = 0; it < TILES; ++it) {
        const uint32_t e = it * QP_TILE + tid * QP_PER_LANE;
        local[it] = seg[it] - seg_first;
        valid[it] = e < n_elems ? lds_valid_end[local[it]] - static_cast<int32_t>(e) : 0;
    }
    const int n_scan = dq_chunk_granule_sums<LINF>(x, valid, local, static_cast<int>(tid), lds_gsum, lds_glocal,
                                                   seg_first == seg_last, static_cast<int>(n_elems >> 7));
    __syncthreads();
    if (tid < DQ_CHUNK_GRANULES)
        dq_chunk_tensor_totals<LINF>(static_cast<int>(tid), n_scan, lds_gsum, lds_glocal,
                                     [&](int j, double total) {
                                         partials[static_cast<int64_t>(w) * n_slots + blockIdx.x + seg_first + j] = total;
                                         if (lds_whole[j]) {
                                             const float N = LINF ? static_cast<float>(total) : static_cast<float>(sqrt(total));
                                             norms_out[static_cast<int64_t>(w) * n_seg + cseg_seg[seg_first + j]] = N;
                                             inside[static_cast<int64_t>(w) * n_cseg + seg_first + j] = 1;
                                             const float scale = N >= DQ_MIN_NORM ? lds_levels[j] / N : 0.0f;
                                             lds_scale_hi[j] = scale;
                                             lds_scale_lo[j] = scale;
                                         }
                                     });
    if (any_whole) __syncthreads();
    if (skip) {
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
            const float S = lds_levels[local[it]];
            const int b = lds_b[local[it]];
            const uint64_t field = (static_cast<uint64_t>(1) << b) - 1u;
            const uint32_t quad = quad_lo0 + (e >> 2);
            uint32_t sign, rr[2][4];
            uint64_t level;
            quantize8<0>(x[it][0], x[it][1], lds_scale_hi[local[it]], S, b, quad, quad_hi, worker, step, key0, key1,
                         sign, level, rr);
            const int nv = valid[it] >= QP_PER_LANE ? QP_PER_LANE : (valid[it] > 0 ? valid[it] : 0);
            if (nv < QP_PER_LANE) {
                sign &= (1u << nv) - 1u;
                level &= (static_cast<uint64_t>(1) << (nv * b)) - 1u;
            }
            if (level != 0) {
                const float scale_lo = lds_scale_lo[local[it]];
                const float v[8] = { x[it][0].x, x[it][0].y, x[it][0].z, x[it][0].w,
                                     x[it][1].x, x[it][1].y, x[it][1].z, x[it][1].w };
                const uint32_t r[8] = { rr[0][0], rr[0][1], rr[0][2], rr[0][3], rr[1][0], rr[1][1], rr[1][2], rr[1][3] };
#pragma unroll
                for (int k = 0; k < QP_PER_LANE; ++k) {
                    const uint32_t top = static_cast<uint32_t>(level >> (k * b)) & static_cast<uint32_t>(field);
                    if (top != 0 && level_of_s(v[k], scale_lo, S, r[k]) != top) {
                        const uint32_t slot = atomicAdd(&lds_count, 1u);
                        if (slot < DQ_BRACKET_CAP) blk->rec[slot] = make_uint2(e + k, __float_as_uint(v[k]));
                        level &= ~(field << (k * b));
                    }
                }
            }
            lds_sign[it * QP_THREADS + tid] = static_cast<uint8_t>(sign);
            uint8_t* dst = &lds_level[lds_level_base[local[it]] + static_cast<int32_t>(e >> 3) * b];
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
    if (tid == 0) {
        blk->count = lds_count;
        blk->flags = 0;
    }
}

// grid (n_span, M), the tensors that cross a chunk boundary (the others are finished by the first
// kernel): the norm of tensor c of worker w from its partial sums (or maxima), slots
// [first chunk + c, last chunk + c]: eight lane-strided running sums per lane, combined in a fixed
// order, then a fixed tree over the lanes.  Also notes whether the norm lies inside its bracket.
template <bool LINF>
__global__ __launch_bounds__(256) void k_bracket_norm_finish(
    const double* __restrict__ partials, int64_t n_slots, const int64_t* __restrict__ cseg_start,
    const int64_t* __restrict__ cseg_valid_end, const int32_t* __restrict__ cseg_seg, const int32_t* __restrict__ span_cseg,
    int32_t n_seg, int32_t n_cseg, const float* __restrict__ norm_lo, const float* __restrict__ norm_hi,
    float* __restrict__ norms, uint8_t* __restrict__ inside)
{
    __shared__ double part[256];
    const int tid = threadIdx.x;
    const int32_t c = span_cseg[blockIdx.x];
    const int w = blockIdx.y;
    const int64_t first = cseg_start[c] / DQ_CHUNK;
    const int64_t last = (cseg_valid_end[c] - 1) / DQ_CHUNK;
    const double* p = partials + static_cast<int64_t>(w) * n_slots + first + c;
    const int64_t n = last - first + 1;
    double acc[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[k] = 0.0;
    int64_t i = tid;
    for (; i + 7 * 256 < n; i += 8 * 256) {
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[k] = dq_chunk_combine<LINF>(acc[k], p[i + k * 256]);
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) // fewer than eight are left
        if (i + k * 256 < n) acc[k] = dq_chunk_combine<LINF>(acc[k], p[i + k * 256]);
    part[tid] = dq_chunk_combine<LINF>(
        dq_chunk_combine<LINF>(dq_chunk_combine<LINF>(acc[0], acc[1]), dq_chunk_combine<LINF>(acc[2], acc[3])),
        dq_chunk_combine<LINF>(dq_chunk_combine<LINF>(acc[4], acc[5]), dq_chunk_combine<LINF>(acc[6], acc[7])));
    __syncthreads();
    for (int off = 128; off >= 1; off >>= 1) {
        if (tid < off) part[tid] = dq_chunk_combine<LINF>(part[tid], part[tid + off]);
        __syncthreads();
    }
    if (tid == 0) {
        const int64_t at = static_cast<int64_t>(w) * n_seg + cseg_seg[c];
        const float N = LINF ? static_cast<float>(part[0]) : static_cast<float>(sqrt(part[0]));
        norms[at] = N;
        inside[static_cast<int64_t>(w) * n_cseg + c] = (N >= norm_lo[at] && N <= norm_hi[at]) ? 1 : 0;
    }
}

// One recorded element: its level for the true norm, ORed into the zero field the first kernel left.
// B = 0: per-tensor widths, b and the place of the tensor's level fields come from `widths` (this
// worker's row of the table).
template <int B>
__device__ __forceinline__ void settle_record(uint2 rec, int64_t chunk0, uint32_t w, const float* __restrict__ norms,
                                              int32_t n_seg, const int32_t* __restrict__ granule_cseg,
                                              const int32_t* __restrict__ cseg_seg, uint32_t key0, uint32_t key1,
                                              uint32_t step, uint32_t worker, uint32_t* __restrict__ plane,
                                              const dq_cseg_width* __restrict__ widths)
{
    const uint32_t e = rec.x; // < 4096 and inside the layout: written by the first kernel for this chunk
    const int32_t c = granule_cseg[(chunk0 >> 7) + (e >> 7)];
    const float N = norms[static_cast<int64_t>(w) * n_seg + cseg_seg[c]];
    const uint64_t P = static_cast<uint64_t>(chunk0) + e;
    uint32_t r[4];
    dq_philox4x32_10(static_cast<uint32_t>(P >> 2), static_cast<uint32_t>(P >> 34), worker, step, key0, key1, r);
    const uint32_t word = (P & 2u) ? ((P & 1u) ? r[3] : r[2]) : ((P & 1u) ? r[1] : r[0]);
    uint32_t level;
    uint64_t bit;
    int b;
    if constexpr (B == 0) {
        const dq_cseg_width wd = widths[c];
        b = wd.b;
        const float S = static_cast<float>((1 << b) - 1);
        level = level_of_s(__uint_as_float(rec.y), N >= DQ_MIN_NORM ? S / N : 0.0f, S, word);
        bit = static_cast<uint64_t>(wd.level_start) * 8u + (P - static_cast<uint64_t>(wd.seg_start)) * static_cast<uint64_t>(b);
    } else {
        constexpr float S = static_cast<float>((1 << B) - 1);
        b = B;
        level = level_of<B>(__uint_as_float(rec.y), N >= DQ_MIN_NORM ? S / N : 0.0f, word);
        bit = P * B;
    }
    if (level != 0) {
        // fields of other elements in the same words are not touched
        const uint32_t sh = static_cast<uint32_t>(bit & 31u);
        atomicOr(plane + (bit >> 5), level << sh);
        if (sh + b > 32) atomicOr(plane + (bit >> 5) + 1, level >> (32 - sh));
    }
}

// What the settle kernels decide per chunk: true if the chunk has to be quantized again.
__device__ __forceinline__ bool chunk_needs_redo(uint32_t count, uint32_t flags, int64_t chunk0, int64_t padded_elems,
                                                 uint32_t w, int32_t n_cseg, const int32_t* __restrict__ granule_cseg,
                                                 const uint8_t* __restrict__ inside)
{
    const int64_t last_granule = ((chunk0 + DQ_CHUNK < padded_elems ? chunk0 + DQ_CHUNK : padded_elems) - 1) >> 7;
    const int32_t c_first = granule_cseg[chunk0 >> 7], c_last = granule_cseg[last_granule];
    bool again = flags != 0 || count > DQ_BRACKET_CAP;
    for (int32_t c = c_first; c <= c_last; ++c) again = again || inside[static_cast<int64_t>(w) * n_cseg + c] == 0;
    return again;
}

// grid (ceil(n_chunks / 4), M), one wavefront per chunk and one lane per record: for plans of
// moderate size, where a launch of that many wavefronts is cheap and a chunk may hold dozens of
// records.
template <int B>
__global__ __launch_bounds__(256) void k_bracket_settle_wide(
    const float* __restrict__ norms, int32_t n_seg, int32_t n_cseg, const int32_t* __restrict__ granule_cseg,
    const int32_t* __restrict__ cseg_seg, int64_t padded_elems, uint32_t key0, uint32_t key1, uint32_t step,
    uint32_t worker_base, uint8_t* __restrict__ packed, int64_t packed_stride, dq_bracket_block* __restrict__ blocks,
    int64_t n_chunks, const uint8_t* __restrict__ inside, unsigned long long* __restrict__ redo_map, int64_t n_words,
    const dq_cseg_width* __restrict__ widths_table, int32_t widths_worker_stride)
{
    const dq_cseg_width* __restrict__ widths = widths_table + static_cast<int64_t>(blockIdx.y) * widths_worker_stride;
    const uint32_t w = blockIdx.y;
    const uint32_t lane = threadIdx.x & 63;
    const int64_t chunk = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (chunk >= n_chunks) return; // the whole wavefront
    dq_bracket_block* blk = blocks + static_cast<int64_t>(w) * n_chunks + chunk;
    const uint32_t count = blk->count, flags = blk->flags;
    const int64_t chunk0 = chunk * DQ_CHUNK;
    const bool again = chunk_needs_redo(count, flags, chunk0, padded_elems, w, n_cseg, granule_cseg, inside);
    if (again) {
        if (lane == 0) {
            blk->flags = flags | 2u;
            atomicOr(redo_map + static_cast<int64_t>(w) * n_words + (chunk >> 6), 1ull << (chunk & 63));
        }
    } else if (lane < count) {
        uint32_t* plane = reinterpret_cast<uint32_t*>(packed + static_cast<int64_t>(w) * packed_stride + (padded_elems >> 3));
        settle_record<B>(blk->rec[lane], chunk0, w, norms, n_seg, granule_cseg, cseg_seg, key0, key1, step,
                         worker_base + w, plane, widths);
    }
}

__global__ __launch_bounds__(256) void k_zero_words(unsigned long long* __restrict__ dst, int64_t n)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i < n) dst[i] = 0;
}

// grid (ceil(n_chunks / 256), M), one lane per chunk: for large plans with few records per chunk.
template <int B>
__global__ __launch_bounds__(256) void k_bracket_settle(
    const float* __restrict__ norms, int32_t n_seg, int32_t n_cseg, const int32_t* __restrict__ granule_cseg,
    const int32_t* __restrict__ cseg_seg, int64_t padded_elems, uint32_t key0, uint32_t key1, uint32_t step,
    uint32_t worker_base, uint8_t* __restrict__ packed, int64_t packed_stride, dq_bracket_block* __restrict__ blocks,
    int64_t n_chunks, const uint8_t* __restrict__ inside, unsigned long long* __restrict__ redo_map, int64_t n_words,
    const dq_cseg_width* __restrict__ widths_table, int32_t widths_worker_stride)
{
    const dq_cseg_width* __restrict__ widths = widths_table + static_cast<int64_t>(blockIdx.y) * widths_worker_stride;
    const uint32_t w = blockIdx.y;
    const int64_t chunk = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    const bool active = chunk < n_chunks;
    bool again = false;
    if (active) {
        dq_bracket_block* blk = blocks + static_cast<int64_t>(w) * n_chunks + chunk;
        const uint32_t count = blk->count, flags = blk->flags;
        const int64_t chunk0 = chunk * DQ_CHUNK;
        again = chunk_needs_redo(count, flags, chunk0, padded_elems, w, n_cseg, granule_cseg, inside);
        if (again) {
            blk->flags = flags | 2u;
        } else {
            uint32_t* plane = reinterpret_cast<uint32_t*>(packed + static_cast<int64_t>(w) * packed_stride +
                                                          (padded_elems >> 3));
            for (uint32_t k = 0; k < count; ++k)
                settle_record<B>(blk->rec[k], chunk0, w, norms, n_seg, granule_cseg, cseg_seg, key0, key1, step,
                                 worker_base + w, plane, widths);
        }
    }
    // 64 consecutive chunks per wavefront: one word of the redo map (blockDim is a multiple of 64)
    const unsigned long long bits = __ballot(active && again);
    if ((threadIdx.x & 63) == 0 && (chunk >> 6) < n_words) redo_map[static_cast<int64_t>(w) * n_words + (chunk >> 6)] = bits;
}

// grid (ceil(n_words / REDO_WORDS), M): each workgroup walks REDO_WORDS words of the redo map and
// quantizes the chunks whose bit is set.
constexpr int REDO_WORDS = 8;
// up to this many (worker, chunk) pairs the settle kernel runs one wavefront per chunk and the
// redo kernel one workgroup per chunk
constexpr int64_t SETTLE_WIDE_MAX = 1 << 16;

template <int B>
__global__ __launch_bounds__(QP_THREADS) void k_bracket_redo(
    const float* __restrict__ grads, int64_t worker_stride, const float* __restrict__ norms, int32_t n_seg,
    const int32_t* __restrict__ granule_cseg, const int32_t* __restrict__ cseg_seg,
    const int64_t* __restrict__ cseg_valid_end, int64_t padded_elems, uint32_t key0, uint32_t key1, uint32_t step,
    uint32_t worker_base, uint8_t* __restrict__ packed, int64_t packed_stride,
    const unsigned long long* __restrict__ redo_map, int64_t n_words, const dq_cseg_width* __restrict__ widths_table,
    int32_t widths_worker_stride)
{
    const int64_t word0 = static_cast<int64_t>(blockIdx.x) * REDO_WORDS;
    const unsigned long long* map = redo_map + static_cast<int64_t>(blockIdx.y) * n_words;
    for (int k = 0; k < REDO_WORDS && word0 + k < n_words; ++k) {
        // the same value in every lane (one address), made scalar so that the loop below is uniform
        const unsigned long long loaded = map[word0 + k];
        unsigned long long bits =
            (static_cast<unsigned long long>(__builtin_amdgcn_readfirstlane(static_cast<int>(loaded >> 32))) << 32) |
            static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(loaded)));
        while (bits != 0) {
            const int bit = __builtin_ctzll(bits);
            bits &= bits - 1;
            const uint32_t chunk = static_cast<uint32_t>((word0 + k) * 64 + bit);
            if constexpr (B == 0)
                quantize_pack_chunk_v<2, 0>(grads, worker_stride, norms, n_seg, granule_cseg, cseg_seg, cseg_valid_end,
                                            widths_table, widths_worker_stride, padded_elems, key0, key1, step,
                                            worker_base, packed, packed_stride, nullptr, chunk);
            else
                quantize_pack_chunk<B, 2, 0>(grads, worker_stride, norms, n_seg, granule_cseg, cseg_seg, cseg_valid_end,
                                             padded_elems, key0, key1, step, worker_base, packed, packed_stride, nullptr,
                                             chunk);
            __syncthreads(); // the chunk's staging in LDS is reused by the next one
        }
    }
}

// grid (n_chunks, M): the same with one workgroup per chunk that looks up its own bit -- for plans of
// moderate size, where that many workgroups start in a few microseconds and flagged chunks that
// sit next to each other are then quantized side by side instead of one after the other.
template <int B>
__global__ __launch_bounds__(QP_THREADS) void k_bracket_redo_direct(
    const float* __restrict__ grads, int64_t worker_stride, const float* __restrict__ norms, int32_t n_seg,
    const int32_t* __restrict__ granule_cseg, const int32_t* __restrict__ cseg_seg,
    const int64_t* __restrict__ cseg_valid_end, int64_t padded_elems, uint32_t key0, uint32_t key1, uint32_t step,
    uint32_t worker_base, uint8_t* __restrict__ packed, int64_t packed_stride,
    const unsigned long long* __restrict__ redo_map, int64_t n_words, const dq_cseg_width* __restrict__ widths_table,
    int32_t widths_worker_stride)
{
    const unsigned long long word = redo_map[static_cast<int64_t>(blockIdx.y) * n_words + (blockIdx.x >> 6)];
    if (((word >> (blockIdx.x & 63)) & 1ull) == 0) return; // uniform: one address for the whole workgroup
    if constexpr (B == 0)
        quantize_pack_chunk_v<2, 0>(grads, worker_stride, norms, n_seg, granule_cseg, cseg_seg, cseg_valid_end, widths_table,
                                    widths_worker_stride, padded_elems, key0, key1, step, worker_base, packed,
                                    packed_stride, nullptr, blockIdx.x);
    else
        quantize_pack_chunk<B, 2, 0>(grads, worker_stride, norms, n_seg, granule_cseg, cseg_seg, cseg_valid_end,
                                     padded_elems, key0, key1, step, worker_base, packed, packed_stride, nullptr,
                                     blockIdx.x);
}

// Statistics of one call, from the blocks: elements settled afterwards and chunks quantized again.
// 256 workgroups at most add their totals to the two counters.
constexpr int BS_PER_LANE = 16;

__global__ __launch_bounds__(256) void k_bracket_stats(const dq_bracket_block* __restrict__ blocks, int64_t n_blocks,
                                                       unsigned long long* __restrict__ stats)
{
    __shared__ unsigned long long part[2][256];
    const int tid = threadIdx.x;
    unsigned long long settled = 0, again = 0;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + tid; i < n_blocks;
         i += static_cast<int64_t>(gridDim.x) * 256) {
        const uint32_t count = blocks[i].count, flags = blocks[i].flags;
        if (flags & 2u)
            ++again;
        else
            settled += count;
    }
    part[0][tid] = settled;
    part[1][tid] = again;
    __syncthreads();
    for (int off = 128; off >= 1; off >>= 1) {
        if (tid < off) {
            part[0][tid] += part[0][tid + off];
            part[1][tid] += part[1][tid + off];
        }
        __syncthreads();
    }
    if (tid == 0) {
        if (part[0][0]) atomicAdd(&stats[0], part[0][0]);
        if (part[1][0]) atomicAdd(&stats[1], part[1][0]);
    }
}

__global__ void k_zero_two(unsigned long long* __restrict__ stats)
{
    stats[threadIdx.x] = 0;
}

// B = 0: per-tensor widths from `widths_table` (row stride `widths_row`: 0 when the workers share a row)
template <int B, bool LINF>
int launch_bracketed(const dq_plan* plan, const float* grads, int64_t worker_stride, int M, const float* norm_lo,
                     const float* norm_hi, uint64_t seed, uint32_t step, uint32_t worker_base, float* norms,
                     uint8_t* packed, int64_t packed_stride, void* workspace, unsigned long long* stats,
                     hipStream_t stream, const dq_cseg_width* widths_table = nullptr, int32_t widths_row = 0)
{
    const dq_bracket_layout L = dq_bracket_layout_of(plan, M);
    if (L.n_chunks > INT32_MAX) return DQ_ERR_INVALID_ARG;
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    double* partials = reinterpret_cast<double*>(ws);
    dq_bracket_block* blocks = reinterpret_cast<dq_bracket_block*>(ws + L.blocks_at);
    uint8_t* inside = ws + L.inside_at;
    unsigned long long* redo_map = reinterpret_cast<unsigned long long*>(ws + L.redo_at);
    const dim3 grid(static_cast<unsigned>(L.n_chunks), M), block(QP_THREADS);
    const uint32_t key0 = static_cast<uint32_t>(seed), key1 = static_cast<uint32_t>(seed >> 32);
    if constexpr (B == 0)
        hipLaunchKernelGGL(k_quantize_pack_bracketed_v<LINF>, grid, block, 0, stream, grads, worker_stride, norm_lo, norm_hi,
                           plan->n_seg, plan->d_granule_cseg, plan->d_cseg_seg, plan->d_cseg_start, plan->d_cseg_valid_end,
                           widths_table, widths_row, plan->padded_elems, key0, key1, step, worker_base, packed,
                           packed_stride, partials, L.n_slots, blocks, L.n_chunks, norms, inside, plan->n_cseg);
    else
        hipLaunchKernelGGL((k_quantize_pack_bracketed<(B == 0 ? 1 : B), LINF>), grid, block, 0, stream, grads, worker_stride,
                           norm_lo, norm_hi, plan->n_seg, plan->d_granule_cseg, plan->d_cseg_seg, plan->d_cseg_start,
                           plan->d_cseg_valid_end, plan->padded_elems, key0, key1, step, worker_base, packed,
                           packed_stride, partials, L.n_slots, blocks, L.n_chunks, norms, inside, plan->n_cseg);
    if (plan->n_span > 0)
        hipLaunchKernelGGL(k_bracket_norm_finish<LINF>, dim3(plan->n_span, M), dim3(256), 0, stream, partials, L.n_slots,
                           plan->d_cseg_start, plan->d_cseg_valid_end, plan->d_cseg_seg, plan->d_span_cseg, plan->n_seg,
                           plan->n_cseg, norm_lo, norm_hi, norms, inside);
    if (static_cast<int64_t>(M) * L.n_chunks <= SETTLE_WIDE_MAX) {
        const int64_t words = static_cast<int64_t>(M) * L.n_words;
        hipLaunchKernelGGL(k_zero_words, dim3(static_cast<unsigned>((words + 255) / 256)), dim3(256), 0, stream,
                           redo_map, words);
        hipLaunchKernelGGL(k_bracket_settle_wide<B>, dim3(static_cast<unsigned>((L.n_chunks + 3) / 4), M), dim3(256), 0,
                           stream, norms, plan->n_seg, plan->n_cseg, plan->d_granule_cseg, plan->d_cseg_seg,
                           plan->padded_elems, key0, key1, step, worker_base, packed, packed_stride, blocks, L.n_chunks,
                           inside, redo_map, L.n_words, widths_table, widths_row);
    } else {
        hipLaunchKernelGGL(k_bracket_settle<B>, dim3(static_cast<unsigned>((L.n_chunks + 255) / 256), M), dim3(256), 0,
                           stream, norms, plan->n_seg, plan->n_cseg, plan->d_granule_cseg, plan->d_cseg_seg,
                           plan->padded_elems, key0, key1, step, worker_base, packed, packed_stride, blocks, L.n_chunks,
                           inside, redo_map, L.n_words, widths_table, widths_row);
    }
    if (static_cast<int64_t>(M) * L.n_chunks <= SETTLE_WIDE_MAX)
        hipLaunchKernelGGL(k_bracket_redo_direct<B>, grid, block, 0, stream, grads, worker_stride, norms, plan->n_seg,
                           plan->d_granule_cseg, plan->d_cseg_seg, plan->d_cseg_valid_end, plan->padded_elems, key0, key1,
                           step, worker_base, packed, packed_stride, redo_map, L.n_words, widths_table, widths_row);
    else
        hipLaunchKernelGGL(k_bracket_redo<B>, dim3(static_cast<unsigned>((L.n_words + REDO_WORDS - 1) / REDO_WORDS), M),
                           block, 0, stream, grads, worker_stride, norms, plan->n_seg, plan->d_granule_cseg,
                           plan->d_cseg_seg, plan->d_cseg_valid_end, plan->padded_elems, key0, key1, step, worker_base,
                           packed, packed_stride, redo_map, L.n_words, widths_table, widths_row);
    if (stats) {
        const int64_t n_blocks = static_cast<int64_t>(M) * L.n_chunks;
        const int64_t wgs = (n_blocks + 256 * BS_PER_LANE - 1) / (256 * BS_PER_LANE);
        hipLaunchKernelGGL(k_zero_two, dim3(1), dim3(2), 0, stream, stats);
        hipLaunchKernelGGL(k_bracket_stats, dim3(static_cast<unsigned>(wgs < 256 ? wgs : 256)), dim3(256), 0, stream,
                           blocks, n_blocks, stats);
    }
    return hipGetLastError() == hipSuccess ? DQ_OK : DQ_ERR_HIP;
}

} // namespace

namespace {

__global__ __launch_bounds__(256) void k_norm_bracket(const float* __restrict__ norms, int64_t n, float below, float above,
                                                      float* __restrict__ lo, float* __restrict__ hi)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i < n) {
        const float N = norms[i];
        lo[i] = N * below;
        hi[i] = N * above;
    }
}

} // namespace

extern "C" int dq_norm_bracket(const float* norms_dev, int64_t n, float margin, float* norm_lo_dev, float* norm_hi_dev,
                               void* hip_stream)
{
    if (!norms_dev || !norm_lo_dev || !norm_hi_dev || n < 0 || n > (INT64_C(1) << 38)) return DQ_ERR_INVALID_ARG;
    if (!(margin >= 0.0f) || !(margin < 1.0f)) return DQ_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(norms_dev) & 3u) || (reinterpret_cast<uintptr_t>(norm_lo_dev) & 3u) ||
        (reinterpret_cast<uintptr_t>(norm_hi_dev) & 3u))
        return DQ_ERR_INVALID_ARG;
    if (n == 0) return DQ_OK;
    hipLaunchKernelGGL(k_norm_bracket, dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), norms_dev, n, 1.0f - margin, 1.0f + margin, norm_lo_dev,
                       norm_hi_dev);
    return hipGetLastError() == hipSuccess ? DQ_OK : DQ_ERR_HIP;
}

extern "C" int64_t dq_bracketed_workspace_bytes(const dq_plan_t* plan, int M)
{
    if (!plan || M < 1 || M > DQ_MAX_WORKERS) return -1;
    return dq_bracket_layout_of(plan, M).total;
}

extern "C" int dq_norm_quantize_pack_bracketed(const dq_plan_t* plan, const float* grads_dev,
                                               int64_t worker_stride_elems, int M, int linf, const float* norm_lo_dev,
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
        return linf ? launch_bracketed<B, true>(plan, grads_dev, worker_stride_elems, M, norm_lo_dev, norm_hi_dev,  \
                                                seed, step, worker_base, norms_dev, packed_dev,                      \
                                                packed_worker_stride_bytes, workspace_dev, stats, stream)            \
                    : launch_bracketed<B, false>(plan, grads_dev, worker_stride_elems, M, norm_lo_dev, norm_hi_dev, \
                                                 seed, step, worker_base, norms_dev, packed_dev,                     \
                                                 packed_worker_stride_bytes, workspace_dev, stats, stream)
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

extern "C" int dq_norm_quantize_pack_bracketed_v(const dq_plan_t* plan, const dq_widths_t* widths, const float* grads_dev,
                                                 int64_t worker_stride_elems, int M, int linf, const float* norm_lo_dev,
                                                 const float* norm_hi_dev, uint64_t seed, uint32_t step,
                                                 uint32_t worker_base, float* norms_dev, uint8_t* packed_dev,
                                                 int64_t packed_worker_stride_bytes, void* workspace_dev,
                                                 int64_t* stats_dev, void* hip_stream)
{
    if (!plan || !widths || !grads_dev || !norm_lo_dev || !norm_hi_dev || !norms_dev || !packed_dev || !workspace_dev)
        return DQ_ERR_INVALID_ARG;
    if (widths->plan != plan || widths->packed_bytes < 0) return DQ_ERR_INVALID_ARG;
    if (M < 1 || M > DQ_MAX_WORKERS) return DQ_ERR_INVALID_ARG;
    if (widths->n_workers != 1 && widths->n_workers != M) return DQ_ERR_INVALID_ARG;
    const int32_t row_stride = widths->n_workers == 1 ? 0 : plan->n_cseg;
    if (worker_stride_elems < plan->padded_elems || (worker_stride_elems & 3)) return DQ_ERR_INVALID_ARG;
    if (packed_worker_stride_bytes < widths->packed_bytes || (packed_worker_stride_bytes & 15))
        return DQ_ERR_INVALID_ARG;
    if (!dq_aligned16(grads_dev) || !dq_aligned16(packed_dev) || !dq_aligned16(workspace_dev)) return DQ_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(norm_lo_dev) & 3u) || (reinterpret_cast<uintptr_t>(norm_hi_dev) & 3u) ||
        (reinterpret_cast<uintptr_t>(norms_dev) & 3u) || (reinterpret_cast<uintptr_t>(stats_dev) & 7u))
        return DQ_ERR_INVALID_ARG;
    const int rc = dq_plan_check_device(plan);
    if (rc != DQ_OK) return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (plan->n_cseg < plan->n_seg) {
        const int zrc = dq_zero_floats(norms_dev, static_cast<int64_t>(M) * plan->n_seg, stream);
        if (zrc != DQ_OK) return zrc;
    }
    if (plan->padded_elems == 0) return DQ_OK;
    unsigned long long* stats = reinterpret_cast<unsigned long long*>(stats_dev);
    return linf ? launch_bracketed<0, true>(plan, grads_dev, worker_stride_elems, M, norm_lo_dev, norm_hi_dev, seed, step,
                                            worker_base, norms_dev, packed_dev, packed_worker_stride_bytes, workspace_dev,
                                            stats, stream, widths->d_table, row_stride)
                : launch_bracketed<0, false>(plan, grads_dev, worker_stride_elems, M, norm_lo_dev, norm_hi_dev, seed, step,
                                             worker_base, norms_dev, packed_dev, packed_worker_stride_bytes, workspace_dev,
                                             stats, stream, widths->d_table, row_stride);
}
