// dq_unpack_dequant_reduce: the server average of Algorithm 1 / Eq. (2),
//     out_P = (1/M) sum_i sgn_{i,P} * level_{i,P} * (N_{i,l} / s),
// with every worker's message read exactly once.
//
// Work split.  One workgroup (256 lanes) owns 8192 consecutive padded elements; a lane owns 32 of
// them, so per worker it reads one sign dword and B level dwords -- every load is dword aligned
// for every B -- and keeps 32 binary32 accumulators.
//
// Arithmetic per (worker, element).  B <= 4: the level fields are spread one per byte word-wise
// (byte permutes and a shift/mask per four elements), the four sign bits of the word's elements go
// onto bit 7 of its bytes with one shift and one and-or, and each byte -- (sign << 7) | level --
// is converted as an 8-bit float, which is exactly +-level * 2^-9: half a conversion instruction
// and one FMA per element, no sign handling per element (about 2.6-3.4 vector instructions per
// worker and element against 4.5 with a conversion, a sign shift, a sign merge and an FMA each).
// B >= 5 (bound by memory): convert the level (one v_cvt_f32_ubyteN at B = 8, a field extract and a
// convert otherwise), put the sign bit on the worker's unit (shift, v_and_or), one FMA.
//
// The 32 results of a lane are consecutive in memory, so storing them directly would be 16-byte
// pieces 128 bytes apart; they go through LDS (XOR-swizzled 16-byte slots, conflict free both
// ways) and leave as fully coalesced 16-byte stores.
//
// The units N/s of the segments a workgroup touches are computed once per workgroup into LDS.
//
// HBM traffic per output element: M(B+1)/8 bytes read, 4 bytes written.
//
// With a model vector x the epilogue also applies the update of Algorithm 1, x <- x - eta * g_hat
// (8 more bytes per element, read and written with the same coalesced 16-byte accesses).
#include <utility>

#include "dq_internal.h"

namespace {

#ifndef UR_THREADS_N
#define UR_THREADS_N 256
#endif
constexpr int UR_THREADS = UR_THREADS_N;
constexpr int UR_PER_LANE = 32;
constexpr int UR_TILE = UR_THREADS * UR_PER_LANE; // 8192 elements
constexpr int UR_MAX_LOCAL_SEG = UR_TILE / DQ_GRANULE;

// level k (0..31) of a lane's B dwords; fields may straddle two dwords when B is not a power of two
template <int B>
__device__ __forceinline__ uint32_t level_field(const uint32_t (&wd)[B], int k)
{
    const int bit = k * B;
    const int word = bit >> 5, off = bit & 31;
    if (off + B <= 32) return __builtin_amdgcn_ubfe(wd[word], off, B);
    // straddles: funnel-shift the pair down, then mask
    const uint32_t lo = __builtin_amdgcn_alignbit(wd[word + 1 < B ? word + 1 : word], wd[word], off);
    return lo & ((1u << B) - 1u);
}

// Calls f(k, (float)level_k) for the 32 levels of a lane.  When B divides 8 the fields of a dword
// are first spread to one per byte (a shift and a mask serve four levels), so each conversion is
// a single v_cvt_f32_ubyteN with no separate field extract.
template <int B, typename F>
__device__ __forceinline__ void for_each_level(const uint32_t (&wd)[B], F&& f)
{
    if constexpr (8 % B == 0) {
        constexpr int R = 8 / B;                                   // fields per byte
        constexpr uint32_t MASK = ((1u << B) - 1u) * 0x01010101u;  // one field per byte
#pragma unroll
        for (int w = 0; w < B; ++w) {
#pragma unroll
            for (int s = 0; s < R; ++s) {
                uint32_t t = B == 8 ? wd[w] : (wd[w] >> (s * B)) & MASK;
                // keep the spread form: without this the compiler folds shift, mask and byte select
                // back into one field extract per level
                if constexpr (B != 8) asm("" : "+v"(t));
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    f(w * (32 / B) + j * R + s, static_cast<float>((t >> (8 * j)) & 0xFFu));
            }
        }
    } else {
#pragma unroll
        for (int k = 0; k < UR_PER_LANE; ++k) f(k, static_cast<float>(level_field<B>(wd, k)));
    }
}

// Widths 1 to 4 take the sign-and-level route below: the byte (sign << 7) | level, level <= 15,
// read as an 8-bit float (E4M3: 4 exponent bits with bias 7, 3 fraction bits) is exactly
// +-level * 2^-9 -- its subnormals and its first binade of normal numbers share one spacing -- so
// one conversion instruction turns two such bytes into two signed binary32 levels, with no
// separate sign handling per element.  Sums formed this way carry the factor 2^-9; the caller
// takes it out together with 1/M (UR_FP8_SCALE).
__host__ __device__ constexpr bool ur_fp8_width(int b) { return b >= 1 && b <= 4; }
constexpr float UR_FP8_SCALE = 512.0f;
// the 32 KiB output tile in LDS allows four workgroups per CU, i.e. four wavefronts per SIMD: the register
// budget is held to what keeps that many resident
constexpr int UR_MIN_WAVES = 4;
constexpr int UR_SUM_BLOCK = 8; // workers per block of the two-level sum (a power of two)
// workers whose loads are issued together (measured per width at D = 2^28, M = 16)
__host__ __device__ constexpr int ur_group(int b) { return b <= 4 ? 16 : b <= 6 ? 2 : 4; }

// bytes of {hi, lo} picked by the four selector bytes of sel: 0..3 = bytes of lo, 4..7 = bytes of hi
__device__ __forceinline__ uint32_t byte_perm(uint32_t hi, uint32_t lo, uint32_t sel)
{
    return __builtin_amdgcn_perm(hi, lo, sel);
}

// t holds the levels (<= 15) of elements e, e+8, e+16, e+24 of the lane, one per byte; the sign bits
// of those elements are bits e, e+8, e+16, e+24 of sg.  acc[.] += sgn * level * 2^-9 * unit.
template <int E>
__device__ __forceinline__ void fma_signed_bytes(uint32_t t, uint32_t sg, float unit, float (&acc)[UR_PER_LANE])
{
    const uint32_t coded = ((sg << (7 - E)) & 0x80808080u) | t; // sign bits onto bit 7 of each byte
    const auto lo = __builtin_amdgcn_cvt_pk_f32_fp8(static_cast<int>(coded), false); // bytes 0, 1
    const auto hi = __builtin_amdgcn_cvt_pk_f32_fp8(static_cast<int>(coded), true);  // bytes 2, 3
    acc[E] = __builtin_fmaf(lo[0], unit, acc[E]);
    acc[E + 8] = __builtin_fmaf(lo[1], unit, acc[E + 8]);
    acc[E + 16] = __builtin_fmaf(hi[0], unit, acc[E + 16]);
    acc[E + 24] = __builtin_fmaf(hi[1], unit, acc[E + 24]);
}

// Width 3: y[i] holds byte i of each of the lane's four 24-bit runs (eight 3-bit fields each); the
// levels of elements E, E+8, E+16, E+24 one per byte.  Fields 2 and 5 of a run straddle two bytes.
template <int E>
__device__ __forceinline__ uint32_t level_bytes_b3(const uint32_t (&y)[3])
{
    constexpr int bit = 3 * E, word = bit >> 3, off = bit & 7;
    if constexpr (off + 3 <= 8) {
        return (y[word] >> off) & 0x07070707u;
    } else {
        constexpr uint32_t lo_mask = ((1u << (8 - off)) - 1u) * 0x01010101u;
        constexpr uint32_t hi_mask = ((1u << (off + 3 - 8)) - 1u) * 0x01010101u;
        return ((y[word] >> off) & lo_mask) | ((y[word + 1] & hi_mask) << (8 - off));
    }
}

template <int B, int... E>
__device__ __forceinline__ void accumulate_words_fp8(uint32_t sg, const uint32_t (&wd)[B], float unit,
                                                     float (&acc)[UR_PER_LANE], std::integer_sequence<int, E...>)
{
    static_assert(sizeof...(E) == 8, "eight groups of four elements");
    if constexpr (B == 1) {
        // bit e + 8j of the one level dword is bit e of its byte j
        (fma_signed_bytes<E>((wd[0] >> E) & 0x01010101u, sg, unit, acc), ...);
    } else if constexpr (B == 2) {
        // byte r of dword q holds elements 16q + 4r .. + 3: gather bytes r, r+2 of both dwords
        const uint32_t q[2] = { byte_perm(wd[1], wd[0], 0x06040200u), byte_perm(wd[1], wd[0], 0x07050301u) };
        (fma_signed_bytes<E>((q[E / 4] >> (2 * (E % 4))) & 0x03030303u, sg, unit, acc), ...);
    } else if constexpr (B == 3) {
        // the lane's 96 level bits are four runs of 24 (elements 8j .. 8j+7): gather byte i of every run
        const uint32_t y[3] = { byte_perm(wd[2], byte_perm(wd[1], wd[0], 0x00060300u), 0x05020100u),
                                byte_perm(wd[2], byte_perm(wd[1], wd[0], 0x00070401u), 0x06020100u),
                                byte_perm(wd[2], byte_perm(wd[1], wd[0], 0x00000502u), 0x07040100u) };
        (fma_signed_bytes<E>(level_bytes_b3<E>(y), sg, unit, acc), ...);
    } else {
        // byte r of dword j holds elements 8j + 2r, 8j + 2r + 1: transpose the 4x4 bytes so that word r
        // holds byte r of every dword
        const uint32_t ab_lo = byte_perm(wd[1], wd[0], 0x05010400u), ab_hi = byte_perm(wd[1], wd[0], 0x07030602u);
        const uint32_t cd_lo = byte_perm(wd[3], wd[2], 0x05010400u), cd_hi = byte_perm(wd[3], wd[2], 0x07030602u);
        const uint32_t p[4] = { byte_perm(cd_lo, ab_lo, 0x05040100u), byte_perm(cd_lo, ab_lo, 0x07060302u),
                                byte_perm(cd_hi, ab_hi, 0x05040100u), byte_perm(cd_hi, ab_hi, 0x07060302u) };
        (fma_signed_bytes<E>((p[E / 2] >> (4 * (E % 2))) & 0x0F0F0F0Fu, sg, unit, acc), ...);
    }
}

// One worker's contribution to a lane's 32 elements from the worker's sign dword and its B level
// dwords: acc[k] += sgn_k * level_k * unit, times 2^-9 when ur_fp8_width(B).
template <int B>
__device__ __forceinline__ void accumulate_words(uint32_t sg, const uint32_t (&wd)[B], float unit,
                                                 float (&acc)[UR_PER_LANE])
{
    if constexpr (ur_fp8_width(B)) {
        accumulate_words_fp8<B>(sg, wd, unit, acc, std::make_integer_sequence<int, 8>{});
    } else {
        for_each_level<B>(wd, [&](int k, float lv) {
            // sign bit of element k on top of the unit, whose own sign bit is always clear
            const float su = __uint_as_float(__float_as_uint(unit) | ((sg << (31 - k)) & 0x80000000u));
            acc[k] = __builtin_fmaf(lv, su, acc[k]);
        });
    }
}

// The same from eight loaded dwords of which the first B count (per-worker widths).
template <int B>
__device__ __forceinline__ void accumulate_first_words(uint32_t sg, const uint32_t (&wd8)[8], float unit,
                                                       float (&acc)[UR_PER_LANE])
{
    uint32_t wd[B];
#pragma unroll
    for (int q = 0; q < B; ++q) wd[q] = wd8[q];
    accumulate_words<B>(sg, wd, unit, acc);
}

// A lane's eight 16-byte slots of the workgroup's output tile in LDS (XOR-swizzled: conflict free for
// the lane's own accesses and for the transposed read of finish_tile).  Before that read a lane's
// slots are its own, so it also keeps the running total of its block sums there.
struct lane_slots {
    float4* wave_out; // this wavefront's 512 slots
    int lane;
    __device__ __forceinline__ float4& operator[](int q) const { return wave_out[lane * 8 + (q ^ (lane & 7))]; }
};
__device__ __forceinline__ lane_slots slots_of(float4* lds_out, int tid)
{
    return lane_slots{ lds_out + (tid >> 6) * 512, tid & 63 };
}

// Sum of blocks, kept without a second set of 32 registers: every block but the last is added to the
// lane's slots (the first one stored), and the accumulators start the next block from zero.
struct block_total {
    lane_slots slots;
    int n_flushed = 0;
    __device__ __forceinline__ void flush(float (&acc)[UR_PER_LANE])
    {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            float4 t = make_float4(acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
            if (n_flushed) {
                const float4 o = slots[q];
                t = make_float4(o.x + t.x, o.y + t.y, o.z + t.z, o.w + t.w);
            }
            slots[q] = t;
            acc[4 * q] = acc[4 * q + 1] = acc[4 * q + 2] = acc[4 * q + 3] = 0.0f;
        }
        ++n_flushed;
    }
    // total of the flushed blocks plus the block still in the accumulators
    __device__ __forceinline__ void finish(float (&acc)[UR_PER_LANE]) const
    {
        if (!n_flushed) return;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const float4 o = slots[q];
            acc[4 * q] = o.x + acc[4 * q];
            acc[4 * q + 1] = o.y + acc[4 * q + 1];
            acc[4 * q + 2] = o.z + acc[4 * q + 2];
            acc[4 * q + 3] = o.w + acc[4 * q + 3];
        }
    }
};

// The M workers' contributions to a lane's 32 elements: acc[k] += sgn * level * unit, workers in
// ascending order.  sign_ptr / level_ptr address worker 0's sign dword and B level dwords of the
// lane; unit_ptr[w] is worker w's N/s for the lane's segment.
template <int B>
__device__ __forceinline__ void accumulate_lane(const uint8_t* __restrict__ sign_ptr,
                                                const uint8_t* __restrict__ level_ptr, int64_t packed_stride,
                                                int M, const float* unit_ptr, float (&acc)[UR_PER_LANE],
                                                lane_slots slots)
{
    // one worker's sign dword and B level dwords of this lane
    auto load_worker = [&](int w, uint32_t& sg, uint32_t (&wd)[B]) {
        sg = dq_load_stream(reinterpret_cast<const uint32_t*>(sign_ptr + static_cast<int64_t>(w) * packed_stride));
        const uint32_t* lp = reinterpret_cast<const uint32_t*>(level_ptr + static_cast<int64_t>(w) * packed_stride);
        if constexpr (B % 4 == 0) {
#pragma unroll
            for (int q = 0; q < B / 4; ++q) {
                const uint4 t = dq_load_stream(reinterpret_cast<const uint4*>(lp) + q);
                wd[4 * q] = t.x; wd[4 * q + 1] = t.y; wd[4 * q + 2] = t.z; wd[4 * q + 3] = t.w;
            }
        } else if constexpr (B % 2 == 0) {
#pragma unroll
            for (int q = 0; q < B / 2; ++q) {
                const uint2 t = dq_load_stream(reinterpret_cast<const uint2*>(lp) + q);
                wd[2 * q] = t.x; wd[2 * q + 1] = t.y;
            }
        } else {
#pragma unroll
            for (int q = 0; q < B; ++q) wd[q] = dq_load_stream(lp + q);
        }
    };
    // Workers in groups whose loads are all issued before the first is used: the pass is bound by
    // memory latency once the arithmetic is cheap, so narrow widths (few registers per worker) take
    // large groups.  Groups halve towards the end, so any M keeps its loads batched.
    //
    // Order of the additions: workers ascending inside blocks of UR_SUM_BLOCK workers (an FMA chain
    // from zero), the block sums added in block order.  However the loads are grouped, a value
    // passes through at most 7 + ceil(M/8) roundings: 15 at M = 64, where a single chain over all
    // workers would take 63 (and measurably leaves the 1e-6 tolerance when one worker's norm
    // dominates).  Up to eight workers nothing is flushed: the plain chain.
    block_total total{ slots };
    auto group = [&](auto g, int w) { // w is a multiple of G
        constexpr int G = decltype(g)::value;
        uint32_t sg[G], wd[G][B];
#pragma unroll
        for (int i = 0; i < G; ++i) load_worker(w + i, sg[i], wd[i]);
#pragma unroll
        for (int i = 0; i < G; ++i) {
            accumulate_words<B>(sg[i], wd[i], unit_ptr[w + i], acc);
            if constexpr (G >= UR_SUM_BLOCK) {
                if ((i + 1) % UR_SUM_BLOCK == 0 && w + i + 1 < M) total.flush(acc);
            }
        }
        if constexpr (G < UR_SUM_BLOCK) {
            if (((w + G) & (UR_SUM_BLOCK - 1)) == 0 && w + G < M) total.flush(acc);
        }
    };
    constexpr int GROUP = ur_group(B);
    int w = 0;
    for (; w + GROUP <= M; w += GROUP) group(std::integral_constant<int, GROUP>{}, w);
    if constexpr (GROUP > 8) if (w + 8 <= M) { group(std::integral_constant<int, 8>{}, w); w += 8; }
    if constexpr (GROUP > 4) if (w + 4 <= M) { group(std::integral_constant<int, 4>{}, w); w += 4; }
    if constexpr (GROUP > 2) if (w + 2 <= M) { group(std::integral_constant<int, 2>{}, w); w += 2; }
    if (w < M) group(std::integral_constant<int, 1>{}, w);
    total.finish(acc);
}

// Scales a lane's sums by 1/M (zero beyond the tensor's end), transposes the workgroup's tile
// through LDS and writes it out; with UPDATE it also applies the model update to x (and then
// `out` may be null).
template <bool UPDATE>
__device__ __forceinline__ void finish_tile(float (&acc)[UR_PER_LANE], bool active, int64_t n_valid, float inv_M,
                                            float4* lds_out, int tid, int64_t tile0, int64_t tile_end,
                                            float* __restrict__ out, float* __restrict__ x, float eta)
{
    if (active) {
        const int nv = n_valid >= UR_PER_LANE ? UR_PER_LANE : (n_valid > 0 ? static_cast<int>(n_valid) : 0);
#pragma unroll
        for (int k = 0; k < UR_PER_LANE; ++k) acc[k] = k < nv ? acc[k] * inv_M : 0.0f;
    }
    // lane t of wave v holds elements [v*2048 + 32t, +32): slot (t, q) -> t*8 + (q ^ (t & 7))
    const int wave = tid >> 6, lane = tid & 63;
    float4* wave_out = lds_out + wave * 512;
#pragma unroll
    for (int q = 0; q < 8; ++q)
        wave_out[lane * 8 + (q ^ (lane & 7))] = make_float4(acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
    // the transposition stays inside the wavefront's own 512 slots: its lanes only have to see one
    // another's LDS writes, no other wavefront's
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        // store j of the wave covers its elements [256j, 256j + 256); this lane takes 4 of them
        const int src_lane = 8 * j + (lane >> 3), q = lane & 7;
        const float4 v = wave_out[src_lane * 8 + (q ^ (src_lane & 7))];
        const int64_t P = tile0 + wave * 2048 + 256 * j + 4 * lane;
        if (P < tile_end) {
            if (!UPDATE || out) dq_store_stream(reinterpret_cast<float4*>(out + P), v);
            if constexpr (UPDATE) { // model update of Algorithm 1: x <- x - eta * g_hat (pads: g_hat is +0, x unchanged)
                float4 xv = *reinterpret_cast<const float4*>(x + P);
                xv.x = __builtin_fmaf(-eta, v.x, xv.x);
                xv.y = __builtin_fmaf(-eta, v.y, xv.y);
                xv.z = __builtin_fmaf(-eta, v.z, xv.z);
                xv.w = __builtin_fmaf(-eta, v.w, xv.w);
                *reinterpret_cast<float4*>(x + P) = xv;
            }
        }
    }
}

template <int B, bool UPDATE>
__global__ __launch_bounds__(UR_THREADS, UR_MIN_WAVES) void k_unpack_dequant_reduce(
    const uint8_t* __restrict__ packed, int64_t packed_stride, int M, const float* __restrict__ norms,
    int32_t n_seg, const int32_t* __restrict__ granule_cseg, const int32_t* __restrict__ cseg_seg,
    const int64_t* __restrict__ cseg_valid_end, int64_t padded_elems, float inv_M, float* __restrict__ out,
    float* __restrict__ x, float eta)
{
    constexpr float S = static_cast<float>((1 << B) - 1);
    extern __shared__ __align__(16) uint8_t lds_raw[];
    float4* lds_out = reinterpret_cast<float4*>(lds_raw);                       // [UR_TILE / 4]
    float* lds_unit = reinterpret_cast<float*>(lds_raw + UR_TILE * sizeof(float)); // [local seg][M]

    const int tid = threadIdx.x;
    const int64_t tile0 = static_cast<int64_t>(blockIdx.x) * UR_TILE;
    const int64_t tile_end = tile0 + UR_TILE < padded_elems ? tile0 + UR_TILE : padded_elems;
    const int64_t P0 = tile0 + tid * UR_PER_LANE;
    const bool active = P0 < tile_end;

    const int32_t seg_first = granule_cseg[tile0 >> 7];
    const int32_t seg_last = granule_cseg[(tile_end - 1) >> 7];
    const int n_local = seg_last - seg_first + 1; // <= UR_MAX_LOCAL_SEG: compact indices grow by <= 1 per granule
    for (int i = tid; i < n_local * M; i += UR_THREADS) {
        const int local = i / M, w = i - local * M;
        const float N = norms[static_cast<int64_t>(w) * n_seg + cseg_seg[seg_first + local]];
        lds_unit[i] = N >= DQ_MIN_NORM ? N / S : 0.0f;
    }
    int local = 0;
    int64_t n_valid = 0;
    if (active) {
        const int32_t c = granule_cseg[P0 >> 7];
        local = c - seg_first;
        n_valid = cseg_valid_end[c] - P0;
    }
    __syncthreads();

    float acc[UR_PER_LANE];
#pragma unroll
    for (int k = 0; k < UR_PER_LANE; ++k) acc[k] = 0.0f;

    if (active)
        accumulate_lane<B>(packed + (P0 >> 3), packed + (padded_elems >> 3) + (P0 >> 3) * B, packed_stride, M,
                           lds_unit + local * M, acc, slots_of(lds_out, tid));
    finish_tile<UPDATE>(acc, active, n_valid, ur_fp8_width(B) ? inv_M * UR_FP8_SCALE : inv_M, lds_out, tid, tile0,
                        tile_end, out, x, eta);
}

// Per-tensor widths: each lane takes its segment's b and the place of its level dwords from the
// widths table and runs the accumulation specialised for that b.  A lane's 32 elements lie in one
// 128-element granule, hence in one segment; lanes of a wave differ in b only where a wave
// straddles two tensors.
template <bool UPDATE>
__global__ __launch_bounds__(UR_THREADS, UR_MIN_WAVES) void k_unpack_dequant_reduce_v(
    const uint8_t* __restrict__ packed, int64_t packed_stride, int M, const float* __restrict__ norms,
    int32_t n_seg, const int32_t* __restrict__ granule_cseg, const int32_t* __restrict__ cseg_seg,
    const int64_t* __restrict__ cseg_valid_end, const dq_cseg_width* __restrict__ widths, int64_t padded_elems,
    float inv_M, float* __restrict__ out, float* __restrict__ x, float eta)
{
    extern __shared__ __align__(16) uint8_t lds_raw[];
    float4* lds_out = reinterpret_cast<float4*>(lds_raw);
    float* lds_unit = reinterpret_cast<float*>(lds_raw + UR_TILE * sizeof(float));

    const int tid = threadIdx.x;
    const int64_t tile0 = static_cast<int64_t>(blockIdx.x) * UR_TILE;
    const int64_t tile_end = tile0 + UR_TILE < padded_elems ? tile0 + UR_TILE : padded_elems;
    const int64_t P0 = tile0 + tid * UR_PER_LANE;
    const bool active = P0 < tile_end;

    const int32_t seg_first = granule_cseg[tile0 >> 7];
    const int32_t seg_last = granule_cseg[(tile_end - 1) >> 7];
    const int n_local = seg_last - seg_first + 1;
    for (int i = tid; i < n_local * M; i += UR_THREADS) {
        const int local = i / M, w = i - local * M;
        const float S = static_cast<float>((1 << widths[seg_first + local].b) - 1);
        const float N = norms[static_cast<int64_t>(w) * n_seg + cseg_seg[seg_first + local]];
        lds_unit[i] = N >= DQ_MIN_NORM ? N / S : 0.0f;
    }
    int local = 0, b = 0;
    int64_t n_valid = 0, level_off = 0;
    if (active) {
        const int32_t c = granule_cseg[P0 >> 7];
        const dq_cseg_width e = widths[c];
        local = c - seg_first;
        n_valid = cseg_valid_end[c] - P0;
        b = e.b;
        level_off = e.level_start + ((P0 - e.seg_start) >> 3) * e.b; // 4*b bytes per lane: dword aligned
    }
    __syncthreads();

    float acc[UR_PER_LANE];
#pragma unroll
    for (int k = 0; k < UR_PER_LANE; ++k) acc[k] = 0.0f;

    if (active) {
        const uint8_t* sign_ptr = packed + (P0 >> 3);
        const uint8_t* level_ptr = packed + (padded_elems >> 3) + level_off;
        const float* unit_ptr = lds_unit + local * M;
        switch (b) {
        case 1: accumulate_lane<1>(sign_ptr, level_ptr, packed_stride, M, unit_ptr, acc, slots_of(lds_out, tid)); break;
        case 2: accumulate_lane<2>(sign_ptr, level_ptr, packed_stride, M, unit_ptr, acc, slots_of(lds_out, tid)); break;
        case 3: accumulate_lane<3>(sign_ptr, level_ptr, packed_stride, M, unit_ptr, acc, slots_of(lds_out, tid)); break;
        case 4: accumulate_lane<4>(sign_ptr, level_ptr, packed_stride, M, unit_ptr, acc, slots_of(lds_out, tid)); break;
        case 5: accumulate_lane<5>(sign_ptr, level_ptr, packed_stride, M, unit_ptr, acc, slots_of(lds_out, tid)); break;
        case 6: accumulate_lane<6>(sign_ptr, level_ptr, packed_stride, M, unit_ptr, acc, slots_of(lds_out, tid)); break;
        case 7: accumulate_lane<7>(sign_ptr, level_ptr, packed_stride, M, unit_ptr, acc, slots_of(lds_out, tid)); break;
        case 8: accumulate_lane<8>(sign_ptr, level_ptr, packed_stride, M, unit_ptr, acc, slots_of(lds_out, tid)); break;
        default: break; // the host only uploads widths in 1..8
        }
    }
    finish_tile<UPDATE>(acc, active, n_valid, ur_fp8_width(b) ? inv_M * UR_FP8_SCALE : inv_M, lds_out, tid, tile0,
                        tile_end, out, x, eta);
}

// Per-worker widths: every worker's message has its own layout, so a lane looks up b and the
// place of its level dwords once per worker and decodes that worker's dwords with the code
// specialised for its b.
struct worker_entry { // what a lane needs to decode one worker's tensor: 16 bytes, one LDS read
    float unit;         // N / s for that worker and tensor
    int32_t b;          // level bits
    int64_t level_base; // level-plane byte offset of padded index P is level_base + (P >> 3) * b
};

template <bool UPDATE>
__global__ __launch_bounds__(UR_THREADS, UR_MIN_WAVES) void k_unpack_dequant_reduce_w(
    const uint8_t* __restrict__ packed, int64_t packed_stride, int M, const float* __restrict__ norms,
    int32_t n_seg, int32_t n_cseg, const int32_t* __restrict__ granule_cseg, const int32_t* __restrict__ cseg_seg,
    const int64_t* __restrict__ cseg_valid_end, const dq_cseg_width* __restrict__ widths, int64_t padded_elems,
    float inv_M, float* __restrict__ out, float* __restrict__ x, float eta)
{
    extern __shared__ __align__(16) uint8_t lds_raw[];
    float4* lds_out = reinterpret_cast<float4*>(lds_raw);
    worker_entry* lds_entry = reinterpret_cast<worker_entry*>(lds_raw + UR_TILE * sizeof(float)); // [local seg][M]

    const int tid = threadIdx.x;
    const int64_t tile0 = static_cast<int64_t>(blockIdx.x) * UR_TILE;
    const int64_t tile_end = tile0 + UR_TILE < padded_elems ? tile0 + UR_TILE : padded_elems;
    const int64_t P0 = tile0 + tid * UR_PER_LANE;
    const bool active = P0 < tile_end;

    const int32_t seg_first = granule_cseg[tile0 >> 7];
    const int32_t seg_last = granule_cseg[(tile_end - 1) >> 7];
    const int n_local = seg_last - seg_first + 1;
    for (int i = tid; i < n_local * M; i += UR_THREADS) {
        const int local = i / M, w = i - local * M;
        const dq_cseg_width e = widths[static_cast<int64_t>(w) * n_cseg + seg_first + local];
        const float S = static_cast<float>((1 << e.b) - 1);
        const float N = norms[static_cast<int64_t>(w) * n_seg + cseg_seg[seg_first + local]];
        worker_entry we;
        // every worker's sum is kept with the factor 2^-9 of the sign-and-level route: the widths that
        // do not take it get the factor on their unit (exact: a usable norm is at least 2^-100)
        const float unit = N >= DQ_MIN_NORM ? N / S : 0.0f;
        we.unit = ur_fp8_width(e.b) ? unit : unit * (1.0f / UR_FP8_SCALE);
        we.b = e.b;
        we.level_base = e.level_start - (e.seg_start >> 3) * e.b; // seg_start is a multiple of 128
        lds_entry[i] = we;
    }
    int32_t c = 0;
    int64_t n_valid = 0;
    if (active) {
        c = granule_cseg[P0 >> 7];
        n_valid = cseg_valid_end[c] - P0;
    }
    __syncthreads();

    float acc[UR_PER_LANE];
#pragma unroll
    for (int k = 0; k < UR_PER_LANE; ++k) acc[k] = 0.0f;

    if (active) {
        const worker_entry* entry = lds_entry + (c - seg_first) * M;
        const uint8_t* sign_ptr = packed + (P0 >> 3);
        const uint8_t* level_plane = packed + (padded_elems >> 3);
        // workers four at a time: sign dwords and up to eight level dwords each are fetched first
        // (loads past a worker's width are skipped), then decoded width by width
        constexpr int GROUP = 4;
        block_total total{ slots_of(lds_out, tid) }; // the block sums of accumulate_lane: same order of additions
        for (int w0 = 0; w0 < M; w0 += GROUP) {
            uint32_t sg[GROUP], wd[GROUP][8];
            worker_entry we[GROUP];
#pragma unroll
            for (int i = 0; i < GROUP; ++i) {
                we[i].b = 0;
                if (w0 + i < M) {
                    we[i] = entry[w0 + i];
                    const int64_t msg = static_cast<int64_t>(w0 + i) * packed_stride;
                    const uint32_t* lp =
                        reinterpret_cast<const uint32_t*>(level_plane + msg + we[i].level_base + (P0 >> 3) * we[i].b);
                    sg[i] = dq_load_stream(reinterpret_cast<const uint32_t*>(sign_ptr + msg));
#pragma unroll
                    for (int q = 0; q < 8; ++q) wd[i][q] = q < we[i].b ? dq_load_stream(lp + q) : 0u;
                }
            }
#pragma unroll
            for (int i = 0; i < GROUP; ++i) {
                switch (we[i].b) {
                case 1: accumulate_first_words<1>(sg[i], wd[i], we[i].unit, acc); break;
                case 2: accumulate_first_words<2>(sg[i], wd[i], we[i].unit, acc); break;
                case 3: accumulate_first_words<3>(sg[i], wd[i], we[i].unit, acc); break;
                case 4: accumulate_first_words<4>(sg[i], wd[i], we[i].unit, acc); break;
                case 5: accumulate_first_words<5>(sg[i], wd[i], we[i].unit, acc); break;
                case 6: accumulate_first_words<6>(sg[i], wd[i], we[i].unit, acc); break;
                case 7: accumulate_first_words<7>(sg[i], wd[i], we[i].unit, acc); break;
                case 8: accumulate_first_words<8>(sg[i], wd[i], we[i].unit, acc); break;
                default: break; // past the last worker, or a width the host never uploads
                }
            }
            if (((w0 + GROUP) & (UR_SUM_BLOCK - 1)) == 0 && w0 + GROUP < M) total.flush(acc);
        }
        total.finish(acc);
    }
    finish_tile<UPDATE>(acc, active, n_valid, inv_M * UR_FP8_SCALE, lds_out, tid, tile0, tile_end, out, x, eta);
}

// acc[k] += sgn_k * scale for a lane's 32 elements: the scale with its sign flipped where the bit is set.
// (The conversion route of the quantized average -- (sign << 7) | 0x38 is +-1 as an 8-bit float -- was
// measured here too: 0.40 ms against 0.35 ms at D = 2^28, M = 16, so the integer form stays.)
__device__ __forceinline__ void add_signed_scale(uint32_t sg, float scale, float (&acc)[UR_PER_LANE])
{
    const uint32_t unit = __float_as_uint(scale);
#pragma unroll
    for (int k = 0; k < UR_PER_LANE; ++k) acc[k] += __uint_as_float(unit ^ ((sg << (31 - k)) & 0x80000000u));
}

// Sign-only messages (the one-bit baseline of the paper's Table 2): the mean of scale * sgn,
// summed over workers ascending like the quantized average.
// HBM traffic per output element: M/8 bytes read, 4 bytes written.
__global__ __launch_bounds__(UR_THREADS) void k_sign_reduce_scaled(
    const uint8_t* __restrict__ packed, int64_t packed_stride, int M, const float* __restrict__ scales,
    int32_t n_seg, const int32_t* __restrict__ granule_cseg, const int32_t* __restrict__ cseg_seg,
    const int64_t* __restrict__ cseg_valid_end, int64_t padded_elems, float inv_M, float* __restrict__ out)
{
    extern __shared__ __align__(16) uint8_t lds_raw[];
    float4* lds_out = reinterpret_cast<float4*>(lds_raw);
    float* lds_unit = reinterpret_cast<float*>(lds_raw + UR_TILE * sizeof(float)); // [local seg][M]

    const int tid = threadIdx.x;
    const int64_t tile0 = static_cast<int64_t>(blockIdx.x) * UR_TILE;
    const int64_t tile_end = tile0 + UR_TILE < padded_elems ? tile0 + UR_TILE : padded_elems;
    const int64_t P0 = tile0 + tid * UR_PER_LANE;
    const bool active = P0 < tile_end;

    const int32_t seg_first = granule_cseg[tile0 >> 7];
    const int32_t seg_last = granule_cseg[(tile_end - 1) >> 7];
    const int n_local = seg_last - seg_first + 1;
    for (int i = tid; i < n_local * M; i += UR_THREADS) {
        const int local = i / M, w = i - local * M;
        lds_unit[i] = scales[static_cast<int64_t>(w) * n_seg + cseg_seg[seg_first + local]];
    }
    int local = 0;
    int64_t n_valid = 0;
    if (active) {
        const int32_t c = granule_cseg[P0 >> 7];
        local = c - seg_first;
        n_valid = cseg_valid_end[c] - P0;
    }
    __syncthreads();

    float acc[UR_PER_LANE];
#pragma unroll
    for (int k = 0; k < UR_PER_LANE; ++k) acc[k] = 0.0f;
    if (active) {
        const uint8_t* sign_ptr = packed + (P0 >> 3);
        const float* unit_ptr = lds_unit + local * M;
        constexpr int GROUP = 8;
        int w = 0;
        for (; w + GROUP <= M; w += GROUP) {
            uint32_t sg[GROUP];
#pragma unroll
            for (int i = 0; i < GROUP; ++i)
                sg[i] = dq_load_stream(reinterpret_cast<const uint32_t*>(sign_ptr + static_cast<int64_t>(w + i) * packed_stride));
#pragma unroll
            for (int i = 0; i < GROUP; ++i) add_signed_scale(sg[i], unit_ptr[w + i], acc);
        }
        for (; w < M; ++w) {
            const uint32_t sg = dq_load_stream(reinterpret_cast<const uint32_t*>(sign_ptr + static_cast<int64_t>(w) * packed_stride));
            add_signed_scale(sg, unit_ptr[w], acc);
        }
    }
    finish_tile<false>(acc, active, n_valid, inv_M, lds_out, tid, tile0, tile_end, out, nullptr, 0.0f);
}

// Sign-only messages without scales: per element only the number of workers whose bit is set
// matters.  A lane keeps that count for its 32 elements bit-sliced in PLANES dwords (bit k of
// plane j = bit j of element k's count, PLANES >= bit length of M) and adds each worker's sign
// dword with a ripple of half adders -- two bit operations per plane for 32 elements at once.
// MAJORITY: out = sgn(M - 2*count) in {-1, 0, +1}; otherwise out = (M - 2*count) / M.
template <int PLANES, bool MAJORITY>
__global__ __launch_bounds__(UR_THREADS) void k_sign_reduce_count(
    const uint8_t* __restrict__ packed, int64_t packed_stride, int M, const int32_t* __restrict__ granule_cseg,
    const int64_t* __restrict__ cseg_valid_end, int64_t padded_elems, float inv_M, float* __restrict__ out)
{
    extern __shared__ __align__(16) uint8_t lds_raw[];
    float4* lds_out = reinterpret_cast<float4*>(lds_raw);

    const int tid = threadIdx.x;
    const int64_t tile0 = static_cast<int64_t>(blockIdx.x) * UR_TILE;
    const int64_t tile_end = tile0 + UR_TILE < padded_elems ? tile0 + UR_TILE : padded_elems;
    const int64_t P0 = tile0 + tid * UR_PER_LANE;
    const bool active = P0 < tile_end;

    float acc[UR_PER_LANE];
#pragma unroll
    for (int k = 0; k < UR_PER_LANE; ++k) acc[k] = 0.0f;
    int64_t n_valid = 0;
    if (active) {
        n_valid = cseg_valid_end[granule_cseg[P0 >> 7]] - P0;
        const uint8_t* sign_ptr = packed + (P0 >> 3);
        uint32_t plane[PLANES];
#pragma unroll
        for (int j = 0; j < PLANES; ++j) plane[j] = 0u;
        auto add = [&](uint32_t carry) {
#pragma unroll
            for (int j = 0; j < PLANES; ++j) {
                const uint32_t t = plane[j] & carry;
                plane[j] ^= carry;
                carry = t;
            }
        };
        constexpr int GROUP = 8;
        int w = 0;
        for (; w + GROUP <= M; w += GROUP) {
            uint32_t sg[GROUP];
#pragma unroll
            for (int i = 0; i < GROUP; ++i)
                sg[i] = dq_load_stream(reinterpret_cast<const uint32_t*>(sign_ptr + static_cast<int64_t>(w + i) * packed_stride));
#pragma unroll
            for (int i = 0; i < GROUP; ++i) add(sg[i]);
        }
        for (; w < M; ++w)
            add(dq_load_stream(reinterpret_cast<const uint32_t*>(sign_ptr + static_cast<int64_t>(w) * packed_stride)));
#pragma unroll
        for (int k = 0; k < UR_PER_LANE; ++k) {
            uint32_t count = 0;
#pragma unroll
            for (int j = 0; j < PLANES; ++j) count |= __builtin_amdgcn_ubfe(plane[j], k, 1) << j;
            const int votes = M - 2 * static_cast<int>(count);
            if constexpr (MAJORITY)
                acc[k] = votes > 0 ? 1.0f : (votes < 0 ? -1.0f : 0.0f);
            else
                acc[k] = static_cast<float>(votes);
        }
    }
    finish_tile<false>(acc, active, n_valid, MAJORITY ? 1.0f : inv_M, lds_out, tid, tile0, tile_end, out, nullptr, 0.0f);
}

template <int B>
int launch(const dq_plan* plan, const uint8_t* packed, int64_t packed_stride, int M, const float* norms,
           float* out, float* x, float eta, hipStream_t stream)
{
    const int64_t n_tiles = (plan->padded_elems + UR_TILE - 1) / UR_TILE;
    if (n_tiles > INT32_MAX) return DQ_ERR_INVALID_ARG;
    const size_t lds_bytes = UR_TILE * sizeof(float) + static_cast<size_t>(UR_MAX_LOCAL_SEG) * M * sizeof(float);
    const dim3 grid(static_cast<unsigned>(n_tiles)), block(UR_THREADS);
    const float inv_M = 1.0f / static_cast<float>(M);
    if (x)
        hipLaunchKernelGGL((k_unpack_dequant_reduce<B, true>), grid, block, lds_bytes, stream, packed, packed_stride, M,
                           norms, plan->n_seg, plan->d_granule_cseg, plan->d_cseg_seg, plan->d_cseg_valid_end,
                           plan->padded_elems, inv_M, out, x, eta);
    else
        hipLaunchKernelGGL((k_unpack_dequant_reduce<B, false>), grid, block, lds_bytes, stream, packed, packed_stride, M,
                           norms, plan->n_seg, plan->d_granule_cseg, plan->d_cseg_seg, plan->d_cseg_valid_end,
                           plan->padded_elems, inv_M, out, x, eta);
    return hipGetLastError() == hipSuccess ? DQ_OK : DQ_ERR_HIP;
}

int reduce_entry(const dq_plan_t* plan, const uint8_t* packed_dev, int64_t packed_worker_stride_bytes, int M,
                 const float* norms_dev, int b, float* out_dev, float* x_dev, float eta, void* hip_stream)
{
    if (!plan || !packed_dev || !norms_dev || (!out_dev && !x_dev)) return DQ_ERR_INVALID_ARG;
    if (M < 1 || M > DQ_MAX_WORKERS || b < 1 || b > 8) return DQ_ERR_INVALID_ARG;
    if (packed_worker_stride_bytes < dq_packed_bytes(plan, b) || (packed_worker_stride_bytes & 15))
        return DQ_ERR_INVALID_ARG;
    if (!dq_aligned16(packed_dev) || !dq_aligned16(out_dev) || !dq_aligned16(x_dev) ||
        (reinterpret_cast<uintptr_t>(norms_dev) & 3u))
        return DQ_ERR_INVALID_ARG;
    if (x_dev && !(eta == eta)) return DQ_ERR_INVALID_ARG; // NaN learning rate
    const int rc = dq_plan_check_device(plan);
    if (rc != DQ_OK) return rc;
    if (plan->padded_elems == 0) return DQ_OK;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    switch (b) {
    case 1: return launch<1>(plan, packed_dev, packed_worker_stride_bytes, M, norms_dev, out_dev, x_dev, eta, stream);
    case 2: return launch<2>(plan, packed_dev, packed_worker_stride_bytes, M, norms_dev, out_dev, x_dev, eta, stream);
    case 3: return launch<3>(plan, packed_dev, packed_worker_stride_bytes, M, norms_dev, out_dev, x_dev, eta, stream);
    case 4: return launch<4>(plan, packed_dev, packed_worker_stride_bytes, M, norms_dev, out_dev, x_dev, eta, stream);
    case 5: return launch<5>(plan, packed_dev, packed_worker_stride_bytes, M, norms_dev, out_dev, x_dev, eta, stream);
    case 6: return launch<6>(plan, packed_dev, packed_worker_stride_bytes, M, norms_dev, out_dev, x_dev, eta, stream);
    case 7: return launch<7>(plan, packed_dev, packed_worker_stride_bytes, M, norms_dev, out_dev, x_dev, eta, stream);
    default: return launch<8>(plan, packed_dev, packed_worker_stride_bytes, M, norms_dev, out_dev, x_dev, eta, stream);
    }
}

int reduce_entry_v(const dq_plan_t* plan, const dq_widths_t* widths, const uint8_t* packed_dev,
                   int64_t packed_worker_stride_bytes, int M, const float* norms_dev, float* out_dev, float* x_dev,
                   float eta, void* hip_stream)
{
    if (!plan || !widths || !packed_dev || !norms_dev || (!out_dev && !x_dev)) return DQ_ERR_INVALID_ARG;
    if (widths->plan != plan || widths->packed_bytes < 0) return DQ_ERR_INVALID_ARG;
    if (M < 1 || M > DQ_MAX_WORKERS) return DQ_ERR_INVALID_ARG;
    if (widths->n_workers != 1 && widths->n_workers != M) return DQ_ERR_INVALID_ARG;
    if (packed_worker_stride_bytes < widths->packed_bytes || (packed_worker_stride_bytes & 15))
        return DQ_ERR_INVALID_ARG;
    if (!dq_aligned16(packed_dev) || !dq_aligned16(out_dev) || !dq_aligned16(x_dev) ||
        (reinterpret_cast<uintptr_t>(norms_dev) & 3u))
        return DQ_ERR_INVALID_ARG;
    if (x_dev && !(eta == eta)) return DQ_ERR_INVALID_ARG;
    const int rc = dq_plan_check_device(plan);
    if (rc != DQ_OK) return rc;
    if (plan->padded_elems == 0) return DQ_OK;
    const int64_t n_tiles = (plan->padded_elems + UR_TILE - 1) / UR_TILE;
    if (n_tiles > INT32_MAX) return DQ_ERR_INVALID_ARG;
    const size_t lds_bytes = UR_TILE * sizeof(float) + static_cast<size_t>(UR_MAX_LOCAL_SEG) * M * sizeof(float);
    const dim3 grid(static_cast<unsigned>(n_tiles)), block(UR_THREADS);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const float inv_M = 1.0f / static_cast<float>(M);
    if (widths->n_workers != 1) {
        const size_t lds_w = UR_TILE * sizeof(float) + static_cast<size_t>(UR_MAX_LOCAL_SEG) * M * sizeof(worker_entry);
        // beyond 64 KiB of LDS per workgroup (M > 32) the kernel has to be told, and the GPU has to have it
        if (lds_w > 64 * 1024) {
            int max_lds = 0;
            if (hipDeviceGetAttribute(&max_lds, hipDeviceAttributeMaxSharedMemoryPerBlock, plan->device) != hipSuccess)
                return DQ_ERR_HIP;
            if (lds_w > static_cast<size_t>(max_lds)) return DQ_ERR_INVALID_ARG;
            const void* fn = x_dev ? reinterpret_cast<const void*>(&k_unpack_dequant_reduce_w<true>)
                                   : reinterpret_cast<const void*>(&k_unpack_dequant_reduce_w<false>);
            if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds_w)) != hipSuccess) {
                (void)hipGetLastError();
                return DQ_ERR_HIP;
            }
        }
        if (x_dev)
            hipLaunchKernelGGL(k_unpack_dequant_reduce_w<true>, grid, block, lds_w, stream, packed_dev,
                               packed_worker_stride_bytes, M, norms_dev, plan->n_seg, plan->n_cseg,
                               plan->d_granule_cseg, plan->d_cseg_seg, plan->d_cseg_valid_end, widths->d_table,
                               plan->padded_elems, inv_M, out_dev, x_dev, eta);
        else
            hipLaunchKernelGGL(k_unpack_dequant_reduce_w<false>, grid, block, lds_w, stream, packed_dev,
                               packed_worker_stride_bytes, M, norms_dev, plan->n_seg, plan->n_cseg,
                               plan->d_granule_cseg, plan->d_cseg_seg, plan->d_cseg_valid_end, widths->d_table,
                               plan->padded_elems, inv_M, out_dev, x_dev, eta);
        return hipGetLastError() == hipSuccess ? DQ_OK : DQ_ERR_HIP;
    }
    if (x_dev)
        hipLaunchKernelGGL(k_unpack_dequant_reduce_v<true>, grid, block, lds_bytes, stream, packed_dev,
                           packed_worker_stride_bytes, M, norms_dev, plan->n_seg, plan->d_granule_cseg,
                           plan->d_cseg_seg, plan->d_cseg_valid_end, widths->d_table, plan->padded_elems, inv_M,
                           out_dev, x_dev, eta);
    else
        hipLaunchKernelGGL(k_unpack_dequant_reduce_v<false>, grid, block, lds_bytes, stream, packed_dev,
                           packed_worker_stride_bytes, M, norms_dev, plan->n_seg, plan->d_granule_cseg,
                           plan->d_cseg_seg, plan->d_cseg_valid_end, widths->d_table, plan->padded_elems, inv_M,
                           out_dev, x_dev, eta);
    return hipGetLastError() == hipSuccess ? DQ_OK : DQ_ERR_HIP;
}

int sign_reduce_entry(bool majority, const dq_plan_t* plan, const uint8_t* packed_dev,
                      int64_t packed_worker_stride_bytes, int M, const float* scales_dev, float* out_dev,
                      void* hip_stream)
{
    if (!plan || !packed_dev || !out_dev) return DQ_ERR_INVALID_ARG;
    if (M < 1 || M > DQ_MAX_WORKERS) return DQ_ERR_INVALID_ARG;
    if (packed_worker_stride_bytes < plan->padded_elems / 8 || (packed_worker_stride_bytes & 15))
        return DQ_ERR_INVALID_ARG;
    if (!dq_aligned16(packed_dev) || !dq_aligned16(out_dev) || (reinterpret_cast<uintptr_t>(scales_dev) & 3u))
        return DQ_ERR_INVALID_ARG;
    const int rc = dq_plan_check_device(plan);
    if (rc != DQ_OK) return rc;
    if (plan->padded_elems == 0) return DQ_OK;
    const int64_t n_tiles = (plan->padded_elems + UR_TILE - 1) / UR_TILE;
    if (n_tiles > INT32_MAX) return DQ_ERR_INVALID_ARG;
    const dim3 grid(static_cast<unsigned>(n_tiles)), block(UR_THREADS);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const float inv_M = 1.0f / static_cast<float>(M);
    const size_t tile_bytes = UR_TILE * sizeof(float);
    if (!majority && scales_dev) {
        const size_t lds_bytes = tile_bytes + static_cast<size_t>(UR_MAX_LOCAL_SEG) * M * sizeof(float);
        hipLaunchKernelGGL(k_sign_reduce_scaled, grid, block, lds_bytes, stream, packed_dev,
                           packed_worker_stride_bytes, M, scales_dev, plan->n_seg, plan->d_granule_cseg,
                           plan->d_cseg_seg, plan->d_cseg_valid_end, plan->padded_elems, inv_M, out_dev);
        return hipGetLastError() == hipSuccess ? DQ_OK : DQ_ERR_HIP;
    }
    // planes for the bit-sliced count: the bit length of M, rounded up to 3, 5 or 7 (M <= 64)
#define DQ_LAUNCH_COUNT(PLANES, MAJ)                                                                              \
    hipLaunchKernelGGL((k_sign_reduce_count<PLANES, MAJ>), grid, block, tile_bytes, stream, packed_dev,          \
                       packed_worker_stride_bytes, M, plan->d_granule_cseg, plan->d_cseg_valid_end,              \
                       plan->padded_elems, inv_M, out_dev)
    if (M < 8) {
        if (majority) DQ_LAUNCH_COUNT(3, true); else DQ_LAUNCH_COUNT(3, false);
    } else if (M < 32) {
        if (majority) DQ_LAUNCH_COUNT(5, true); else DQ_LAUNCH_COUNT(5, false);
    } else {
        if (majority) DQ_LAUNCH_COUNT(7, true); else DQ_LAUNCH_COUNT(7, false);
    }
#undef DQ_LAUNCH_COUNT
    return hipGetLastError() == hipSuccess ? DQ_OK : DQ_ERR_HIP;
}

} // namespace

extern "C" int dq_sign_reduce(const dq_plan_t* plan, const uint8_t* packed_dev, int64_t packed_worker_stride_bytes,
                              int M, const float* scales_dev, float* out_dev, void* hip_stream)
{
    return sign_reduce_entry(false, plan, packed_dev, packed_worker_stride_bytes, M, scales_dev, out_dev, hip_stream);
}

extern "C" int dq_sign_majority(const dq_plan_t* plan, const uint8_t* packed_dev, int64_t packed_worker_stride_bytes,
                                int M, float* out_dev, void* hip_stream)
{
    return sign_reduce_entry(true, plan, packed_dev, packed_worker_stride_bytes, M, nullptr, out_dev, hip_stream);
}

extern "C" int dq_unpack_dequant_reduce_v(const dq_plan_t* plan, const dq_widths_t* widths,
                                          const uint8_t* packed_dev, int64_t packed_worker_stride_bytes, int M,
                                          const float* norms_dev, float* out_dev, void* hip_stream)
{
    if (!out_dev) return DQ_ERR_INVALID_ARG;
    return reduce_entry_v(plan, widths, packed_dev, packed_worker_stride_bytes, M, norms_dev, out_dev, nullptr,
                          0.0f, hip_stream);
}

extern "C" int dq_unpack_dequant_reduce_update_v(const dq_plan_t* plan, const dq_widths_t* widths,
                                                 const uint8_t* packed_dev, int64_t packed_worker_stride_bytes,
                                                 int M, const float* norms_dev, float eta, float* x_dev,
                                                 float* ghat_dev, void* hip_stream)
{
    if (!x_dev) return DQ_ERR_INVALID_ARG;
    return reduce_entry_v(plan, widths, packed_dev, packed_worker_stride_bytes, M, norms_dev, ghat_dev, x_dev, eta,
                          hip_stream);
}

extern "C" int dq_unpack_dequant_reduce(const dq_plan_t* plan, const uint8_t* packed_dev,
                                        int64_t packed_worker_stride_bytes, int M, const float* norms_dev,
                                        int b, float* out_dev, void* hip_stream)
{
    if (!out_dev) return DQ_ERR_INVALID_ARG;
    return reduce_entry(plan, packed_dev, packed_worker_stride_bytes, M, norms_dev, b, out_dev, nullptr, 0.0f,
                        hip_stream);
}

extern "C" int dq_unpack_dequant_reduce_update(const dq_plan_t* plan, const uint8_t* packed_dev,
                                               int64_t packed_worker_stride_bytes, int M,
                                               const float* norms_dev, int b, float eta, float* x_dev,
                                               float* ghat_dev, void* hip_stream)
{
    if (!x_dev) return DQ_ERR_INVALID_ARG;
    return reduce_entry(plan, packed_dev, packed_worker_stride_bytes, M, norms_dev, b, ghat_dev, x_dev, eta,
                        hip_stream);
}
