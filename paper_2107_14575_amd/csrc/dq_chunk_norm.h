// Norms of the tensors inside one 4096-element chunk, for plans in which no tensor crosses a
// chunk boundary ("chunk-local" plans: a gradient cut into buckets, or small tensors laid out
// that way).  Used by the norm kernel for such plans and by the quantize kernel that computes
// the norms itself, so that the gradient is read once.
//
// A workgroup of 256 lanes owns the chunk; lane t holds elements [8t, 8t+8) of each of its two
// 2048-element tiles.  Squares are summed in binary64 (exact products) in a fixed order: the
// lane's eight, the 16 lanes of a 128-element granule by a butterfly, then the granules of a
// tensor in ascending order by one lane.  The max norm takes the same route with maxima.
#pragma once
#include "dq_internal.h"

constexpr int DQ_CHUNK = 4096;
constexpr int DQ_CHUNK_GRANULES = DQ_CHUNK / DQ_GRANULE; // 32

// x[it][h]: the lane's float4 halves of tile it; valid[it]: how many of the lane's eight elements of
// tile `it` belong to their tensor (<= 0: none, >= 8: all).  After the call (which contains
// barriers) lds_norm[j] holds the norm of the chunk's j-th tensor, j < n_local.
//   lds_gsum   [32] doubles of scratch;  gseg: granule -> compact tensor index, at the chunk's start
template <bool LINF>
__device__ __forceinline__ void dq_chunk_norms(const float4 (&x)[2][2], const int (&valid)[2], int tid,
                                               uint32_t n_elems, const int32_t* __restrict__ gseg,
                                               int32_t seg_first, int n_local, double* lds_gsum, float* lds_norm)
{
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
#pragma unroll
            for (int off = 8; off >= 1; off >>= 1) {
                const float o = __shfl_xor(m, off, 16);
                m = o > m ? o : m;
            }
            granule = static_cast<double>(m);
        } else {
            double acc = 0.0;
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const double e = k < valid[it] ? static_cast<double>(v[k]) : 0.0;
                acc = __builtin_fma(e, e, acc);
            }
#pragma unroll
            for (int off = 8; off >= 1; off >>= 1)
                acc += __shfl_xor(acc, off, 16); // both partners add the same two values: the 16 lanes end equal
            granule = acc;
        }
        if ((tid & 15) == 0) lds_gsum[it * 16 + (tid >> 4)] = granule;
    }
    __syncthreads();
    if (tid < n_local) {
        const int n_gran = static_cast<int>(n_elems >> 7);
        double total = 0.0;
        for (int g = 0; g < n_gran; ++g) {
            if (gseg[g] - seg_first != tid) continue;
            if constexpr (LINF)
                total = lds_gsum[g] > total ? lds_gsum[g] : total;
            else
                total += lds_gsum[g];
        }
        lds_norm[tid] = LINF ? static_cast<float>(total) : static_cast<float>(sqrt(total));
    }
    __syncthreads();
}
