// Internal declarations shared by the translation units of libdq (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dq.h"

// One piece of a segment handed to one workgroup of the norm kernel: `count` valid elements
// starting at padded index `start` (a multiple of 128), all inside segment `seg`.
struct dq_norm_item {
    int64_t start;
    int32_t count;
    int32_t seg;
};

constexpr int DQ_NORM_CHUNK = 4096; // elements per norm item (one workgroup, 4 float4 per lane)

struct dq_plan {
    int32_t n_seg;
    int64_t padded_elems; // D'
    int64_t* seg_len;     // host [n_seg]
    int64_t* seg_start;   // host [n_seg + 1]
    int32_t n_items;      // norm work items
    int device;           // HIP device the tables live on, -1 if none
    int32_t n_cseg;       // number of non-empty segments
    bool chunk_local;     // no segment crosses a multiple of 4096 in the padded index space
    // device tables.  Kernels address segments through a compact index c that counts only the
    // non-empty ones, so consecutive granules differ by at most one in c.
    int32_t* d_granule_cseg;       // [D'/128]  compact segment index of each 128-element granule
    int32_t* d_cseg_seg;           // [n_nonempty] segment l of compact index c
    int64_t* d_cseg_valid_end;     // [n_nonempty] P_l + len_l: first padded index past the data
    int64_t* d_cseg_start;         // [n_nonempty] P_l
    int32_t* d_span_cseg;          // [n_span] compact indices of the tensors that cross a multiple of 4096
    int32_t n_span;                //          padded elements (all others lie inside one chunk)
    dq_norm_item* d_items;         // [n_items]
    int32_t* d_seg_item_begin;     // [n_seg + 1] items of segment l are [begin[l], begin[l+1])
    int32_t* d_finish_seg;         // [n_finish] segments whose norm needs the finishing kernel: all but
    int32_t n_finish;              //            those of exactly one item (the first kernel finishes these)
};

// Per-tensor bit-widths (dq_widths_*): one entry per non-empty segment, indexed like the plan's
// compact tables.
struct dq_cseg_width {
    int64_t level_start; // byte offset of the segment's level fields inside the level plane (multiple of 16)
    int64_t seg_start;   // P_l
    int32_t b;           // level bits of the segment, 1..8
    int32_t reserved;
};

struct dq_widths {
    const dq_plan* plan;
    int32_t n_workers;       // 1: the workers share the widths; M: one row of the table per worker
    dq_cseg_width* d_table;  // device [n_workers][plan->n_cseg]
    dq_cseg_width* h_stage;  // pinned host staging of the same size
    hipEvent_t uploaded;     // recorded after the last upload; the staging is reused only after it
    double* d_worker_sq;     // device [DQ_MAX_WORKERS]: per-worker squared norms between the rule's kernels
    int64_t packed_bytes;    // message size for the widths last set (the longest worker's), -1 before the first set
    int64_t* worker_bytes;   // [n_workers] message size of each row
    int32_t* b_host;         // [n_workers][n_seg] widths last set
};

// Workspace of dq_norm_quantize_pack_bracketed, four parts, each starting on a multiple of 256 bytes:
//   partial sums of squares, one binary64 slot per (worker, chunk, tensor in the chunk) at index
//     chunk + c (c = the tensor's compact index: both grow along the layout, so the sum is unique
//     and a tensor's slots are contiguous);
//   one 512-byte block per (worker, chunk) with the elements whose level the bracket left open;
//   one byte per (worker, non-empty tensor): 1 if the norm came out inside its bracket;
//   one bit per (worker, chunk), 64 chunks to a word: chunks that have to be quantized again.
constexpr int DQ_BRACKET_CAP = 63; // records per block
struct dq_bracket_block {
    uint32_t count; // open elements found (may exceed DQ_BRACKET_CAP: then the chunk is redone)
    uint32_t flags; // bit 0: a tensor in the chunk had no usable bracket, nothing was quantized;
                    // bit 1: the chunk was quantized again in full
    uint2 rec[DQ_BRACKET_CAP]; // .x = element index inside the chunk, .y = the gradient value's bits
};
static_assert(sizeof(dq_bracket_block) == 512, "one block per (worker, chunk), 512 bytes");

struct dq_bracket_layout {
    int64_t n_chunks, n_slots, n_words;
    int64_t blocks_at, inside_at, redo_at, total; // byte offsets into the workspace
};
static inline dq_bracket_layout dq_bracket_layout_of(const dq_plan* plan, int M)
{
    auto up = [](int64_t v) { return (v + 255) / 256 * 256; };
    dq_bracket_layout L;
    L.n_chunks = (plan->padded_elems + 4095) / 4096;
    L.n_slots = L.n_chunks + plan->n_cseg;
    L.n_words = (L.n_chunks + 63) / 64;
    L.blocks_at = up(static_cast<int64_t>(M) * L.n_slots * 8);
    L.inside_at = L.blocks_at + static_cast<int64_t>(M) * L.n_chunks * static_cast<int64_t>(sizeof(dq_bracket_block));
    L.redo_at = L.inside_at + up(static_cast<int64_t>(M) * plan->n_cseg);
    L.total = L.redo_at + up(static_cast<int64_t>(M) * L.n_words * 8);
    return L;
}

static inline bool dq_aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// sum_l N_l^2 of one worker's row of norms in binary64: blocks of DQ_SUM_BLOCK tensors, each added
// in index order, then the block sums in index order (the plain running sum up to 1024 tensors).
// Host and device rules share this order so that they agree bit for bit.
constexpr int DQ_SUM_BLOCK = 1024;
static inline double dq_worker_squared_norm(const float* row, int32_t n_seg)
{
    double total = 0.0;
    for (int32_t base = 0; base < n_seg; base += DQ_SUM_BLOCK) {
        double block = 0.0;
        for (int32_t l = base; l < n_seg && l < base + DQ_SUM_BLOCK; ++l)
            block += static_cast<double>(row[l]) * static_cast<double>(row[l]);
        total += block;
    }
    return total;
}

// Looks up this GPU's copy of dq_norm_static_scratch's scratch array (`device` is the current
// device), so that the entry point itself finds it ready.
void dq_norm_static_scratch_prepare(int device);

// Fills n floats with +0 (a kernel, not a memset: callers may capture the entry points in a graph).
int dq_zero_floats(float* dst_dev, int64_t n, hipStream_t stream);

// Checks shared by the device entry points; returns DQ_OK when `plan` can launch work on its GPU
// and makes that GPU current.
int dq_plan_check_device(const dq_plan* plan);

// Streaming accesses: data that passes through once (a message being written or read, the averaged
// gradient) is stored and loaded with the non-temporal hint, so it does not displace what the caches
// could keep.  Measured at D = 2^28, M = 16, b = 4: quantize+pack 3.67 -> 3.48 ms with such stores,
// the reduce 0.68 -> 0.59 ms with such loads and stores, the norm pass 2.69 -> 2.57 ms with such loads
// (in quantize+pack non-temporal loads of the gradients cost 4 % instead: they stay plain there).
typedef uint32_t dq_v4u __attribute__((ext_vector_type(4)));
typedef uint32_t dq_v2u __attribute__((ext_vector_type(2)));
typedef float dq_v4f __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void dq_store_stream(uint4* dst, const uint4& v)
{
    const dq_v4u t = { v.x, v.y, v.z, v.w };
    __builtin_nontemporal_store(t, reinterpret_cast<dq_v4u*>(dst));
}
__device__ __forceinline__ void dq_store_stream(float4* dst, const float4& v)
{
    const dq_v4f t = { v.x, v.y, v.z, v.w };
    __builtin_nontemporal_store(t, reinterpret_cast<dq_v4f*>(dst));
}
__device__ __forceinline__ float4 dq_load_stream(const float4* src)
{
    const dq_v4f t = __builtin_nontemporal_load(reinterpret_cast<const dq_v4f*>(src));
    return make_float4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ uint4 dq_load_stream(const uint4* src)
{
    const dq_v4u t = __builtin_nontemporal_load(reinterpret_cast<const dq_v4u*>(src));
    return make_uint4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ uint2 dq_load_stream(const uint2* src)
{
    const dq_v2u t = __builtin_nontemporal_load(reinterpret_cast<const dq_v2u*>(src));
    return make_uint2(t.x, t.y);
}
__device__ __forceinline__ uint32_t dq_load_stream(const uint32_t* src) { return __builtin_nontemporal_load(src); }

// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): ten rounds of two 32x32->64 multiplies, key
// bumped by the Weyl constants between rounds.  The three-input XOR is one v_bitop3_b32.
__device__ __forceinline__ uint32_t dq_xor3(uint32_t a, uint32_t b, uint32_t c)
{
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

__device__ __forceinline__ void dq_philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                 uint32_t k0, uint32_t k1, uint32_t (&out)[4])
{
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = static_cast<uint64_t>(M0) * c0;
        const uint64_t p1 = static_cast<uint64_t>(M1) * c2;
        const uint32_t n0 = dq_xor3(static_cast<uint32_t>(p1 >> 32), c1, k0);
        const uint32_t n2 = dq_xor3(static_cast<uint32_t>(p0 >> 32), c3, k1);
        c1 = static_cast<uint32_t>(p1);
        c3 = static_cast<uint32_t>(p0);
        c0 = n0;
        c2 = n2;
        k0 += W0;
        k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}
