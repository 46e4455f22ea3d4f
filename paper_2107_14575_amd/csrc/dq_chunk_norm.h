// Norms of the tensors inside one 4096-element chunk, for plans in which no tensor crosses a
// chunk boundary ("chunk-local" plans: a gradient cut into buckets, or small tensors laid out
// that way).  Used by the norm kernel for such plans and by the quantize kernel that computes
// the norms itself, so that the gradient is read once.
//
// A workgroup of 256 lanes owns the chunk; lane t holds elements [8t, 8t+8) of each of its two
// 2048-element tiles.  Squares are summed in binary64 (exact products) in a fixed order: the
// lane's eight, the 16 lanes of a 128-element granule by four rotate-and-add steps inside the
// 16-lane DPP row (the granule's first lane keeps the result), then the granules of a tensor by a
// segmented scan over the chunk's 32 granules.  The max norm takes the same route with maxima.
#pragma once
#include "dq_internal.h"

constexpr int DQ_CHUNK = 4096;
constexpr int DQ_CHUNK_GRANULES = DQ_CHUNK / DQ_GRANULE; // 32

// value of the lane N places further on in the same 16-lane row (DPP row_ror:N)
template <int N>
__device__ __forceinline__ float dq_row_ror(float v)
{
    return __uint_as_float(static_cast<uint32_t>(
        __builtin_amdgcn_update_dpp(0, static_cast<int>(__float_as_uint(v)), 0x120 + N, 0xF, 0xF, false)));
}

template <int N>
__device__ __forceinline__ double dq_row_ror(double v)
{
    const uint64_t bits = static_cast<uint64_t>(__double_as_longlong(v));
    const uint32_t lo = static_cast<uint32_t>(
        __builtin_amdgcn_update_dpp(0, static_cast<int>(static_cast<uint32_t>(bits)), 0x120 + N, 0xF, 0xF, false));
    const uint32_t hi = static_cast<uint32_t>(
        __builtin_amdgcn_update_dpp(0, static_cast<int>(static_cast<uint32_t>(bits >> 32)), 0x120 + N, 0xF, 0xF, false));
    return __longlong_as_double(static_cast<long long>((static_cast<uint64_t>(hi) << 32) | lo));
}

// Step 1 (every lane): x[it][h] are the lane's float4 halves of tile it; valid[it] says how many
// of the lane's eight elements of tile `it` belong to their tensor (<= 0: none, >= 8: all);
// local[it] is the index of that tensor among the chunk's tensors.  Leaves the sum (or maximum)
// of every 128-element granule in lds_gsum[32] and the granule's tensor index in lds_glocal[32].
// The caller puts a barrier between the two steps.
//
// `single` (the same for the whole workgroup): the chunk holds (part of) one tensor only.  Then a
// lane's two tiles are added first and one reduction serves both: 16 row totals instead of 32
// granule totals, all of tensor 0.  Returns the number of entries step 2 has to scan.
template <bool LINF>
__device__ __forceinline__ int dq_chunk_granule_sums(const float4 (&x)[2][2], const int (&valid)[2],
                                                     const int (&local)[2], int tid, double* lds_gsum,
                                                     int32_t* lds_glocal, bool single, int n_granules)
{
    if (single) {
        double row;
        if constexpr (LINF) {
            float m = 0.0f;
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const float v[8] = { x[it][0].x, x[it][0].y, x[it][0].z, x[it][0].w,
                                     x[it][1].x, x[it][1].y, x[it][1].z, x[it][1].w };
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const float a = k < valid[it] ? fabsf(v[k]) : 0.0f;
                    m = a > m ? a : m;
                }
            }
            float o;
            o = dq_row_ror<8>(m); m = o > m ? o : m;
            o = dq_row_ror<4>(m); m = o > m ? o : m;
            o = dq_row_ror<2>(m); m = o > m ? o : m;
            o = dq_row_ror<1>(m); m = o > m ? o : m;
            row = static_cast<double>(m);
        } else {
            double acc = 0.0;
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const float v[8] = { x[it][0].x, x[it][0].y, x[it][0].z, x[it][0].w,
                                     x[it][1].x, x[it][1].y, x[it][1].z, x[it][1].w };
                if (valid[it] >= 8) {
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        const double e = static_cast<double>(v[k]);
                        acc = __builtin_fma(e, e, acc);
                    }
                } else {
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        const double e = static_cast<double>(k < valid[it] ? v[k] : 0.0f);
                        acc = __builtin_fma(e, e, acc);
                    }
                }
            }
            acc += dq_row_ror<8>(acc);
            acc += dq_row_ror<4>(acc);
            acc += dq_row_ror<2>(acc);
            acc += dq_row_ror<1>(acc);
            row = acc;
        }
        if ((tid & 15) == 0) {
            lds_gsum[tid >> 4] = row;
            lds_glocal[tid >> 4] = 0;
        }
        return 16;
    }
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const float v[8] = { x[it][0].x, x[it][0].y, x[it][0].z, x[it][0].w,
                             x[it][1].x, x[it][1].y, x[it][1].z, x[it][1].w };
        double granule;
        if constexpr (LINF) { // maxima are exact in binary32
            float m = 0.0f;
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const float a = k < valid[it] ? fabsf(v[k]) : 0.0f;
                m = a > m ? a : m;
            }
            float o;
            o = dq_row_ror<8>(m); m = o > m ? o : m;
            o = dq_row_ror<4>(m); m = o > m ? o : m;
            o = dq_row_ror<2>(m); m = o > m ? o : m;
            o = dq_row_ror<1>(m); m = o > m ? o : m;
            granule = static_cast<double>(m);
        } else {
            double acc = 0.0;
            if (valid[it] >= 8) { // all eight belong to the tensor (almost every lane): no masking
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const double e = static_cast<double>(v[k]);
                    acc = __builtin_fma(e, e, acc);
                }
            } else {
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const double e = static_cast<double>(k < valid[it] ? v[k] : 0.0f);
                    acc = __builtin_fma(e, e, acc);
                }
            }
            acc += dq_row_ror<8>(acc);
            acc += dq_row_ror<4>(acc);
            acc += dq_row_ror<2>(acc);
            acc += dq_row_ror<1>(acc);
            granule = acc; // every lane of the row now has all sixteen terms; the first lane's order is the one used
        }
        if ((tid & 15) == 0) {
            lds_gsum[it * 16 + (tid >> 4)] = granule;
            lds_glocal[it * 16 + (tid >> 4)] = local[it];
        }
    }
    return n_granules;
}

// value of the lane N places back in the same 16-lane row, 0 for the first N lanes (DPP row_shr:N)
template <int N>
__device__ __forceinline__ int dq_row_shr(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, 0x110 + N, 0xF, 0xF, true);
}

template <int N>
__device__ __forceinline__ double dq_row_shr(double v)
{
    const uint64_t bits = static_cast<uint64_t>(__double_as_longlong(v));
    const uint32_t lo = static_cast<uint32_t>(dq_row_shr<N>(static_cast<int>(static_cast<uint32_t>(bits))));
    const uint32_t hi = static_cast<uint32_t>(dq_row_shr<N>(static_cast<int>(static_cast<uint32_t>(bits >> 32))));
    return __longlong_as_double(static_cast<long long>((static_cast<uint64_t>(hi) << 32) | lo));
}

template <bool LINF>
__device__ __forceinline__ double dq_chunk_combine(double a, double b)
{
    if constexpr (LINF)
        return b > a ? b : a;
    else
        return a + b;
}

// Step 2 (the first 32 lanes of the workgroup, one per granule; call it under `if (tid < 32)`):
// a segmented scan over the granules -- four shift-and-combine steps inside each 16-lane row, then
// the second row takes over what the first row's last granule has gathered when a tensor spans
// both -- after which the lane of a tensor's last granule holds the tensor's total and calls
// emit(local tensor index, total): the sum of squares (or the maximum) of the tensor's elements in
// this chunk, in binary64.  A fixed combination order, the same wherever this is used.
template <bool LINF, typename Emit>
__device__ __forceinline__ void dq_chunk_tensor_totals(int g, int n_granules, const double* lds_gsum,
                                                       const int32_t* lds_glocal, Emit&& emit)
{
    const bool used = g < n_granules;
    double v = used ? lds_gsum[g] : 0.0;
    const int t = used ? lds_glocal[g] + 1 : 0; // 0: unused slot, and what a shift past the row's start reads
    double pv;
    int pt;
    pv = dq_row_shr<1>(v); pt = dq_row_shr<1>(t); if (pt == t) v = dq_chunk_combine<LINF>(v, pv);
    pv = dq_row_shr<2>(v); pt = dq_row_shr<2>(t); if (pt == t) v = dq_chunk_combine<LINF>(v, pv);
    pv = dq_row_shr<4>(v); pt = dq_row_shr<4>(t); if (pt == t) v = dq_chunk_combine<LINF>(v, pv);
    pv = dq_row_shr<8>(v); pt = dq_row_shr<8>(t); if (pt == t) v = dq_chunk_combine<LINF>(v, pv);
    // lane 15: the total of the tensor that ends the first row, as far as that row goes
    const uint64_t bits = static_cast<uint64_t>(__double_as_longlong(v));
    const uint32_t tail_lo = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(static_cast<uint32_t>(bits)), 15));
    const uint32_t tail_hi = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(static_cast<uint32_t>(bits >> 32)), 15));
    const int tail_t = __builtin_amdgcn_readlane(t, 15);
    const double tail = __longlong_as_double(static_cast<long long>((static_cast<uint64_t>(tail_hi) << 32) | tail_lo));
    if (g >= 16 && t == tail_t) v = dq_chunk_combine<LINF>(tail, v);
    if (used && (g == n_granules - 1 || lds_glocal[g + 1] + 1 != t)) emit(t - 1, v);
}

// The same for chunk-local plans, where the chunk holds whole tensors: emit(local tensor index, norm).
template <bool LINF, typename Emit>
__device__ __forceinline__ void dq_chunk_tensor_norms(int g, int n_granules, const double* lds_gsum,
                                                      const int32_t* lds_glocal, Emit&& emit)
{
    dq_chunk_tensor_totals<LINF>(g, n_granules, lds_gsum, lds_glocal, [&](int j, double total) {
        emit(j, LINF ? static_cast<float>(total) : static_cast<float>(sqrt(total)));
    });
}
