/*
 * dq -- MI355X (gfx950) stochastic gradient quantizer: the per-iteration data-parallel hot path of
 * DQ-SGD (arXiv 2107.14575, "Dynamic Quantization in SGD for Communication-Efficient Distributed
 * Learning").
 *
 * One step of the path, for M workers simulated on one GPU (Algorithm 1):
 *     dq_norm                    ||g^(i)||_2 per worker and tensor          (the norm in Eq. (5))
 *     dq_select_bits             b_t from the dynamic rule                   (Eq. (17))
 *     dq_quantize_pack           sign + stochastic level per element, packed (Eq. (5)-(6), Eq. (7))
 *     dq_unpack_dequant_reduce   server average of the M messages            (Alg. 1 "Average", Eq. (2))
 *     dq_unpack_dequant_reduce_update   the same fused with x <- x - eta*g_hat  (Alg. 1 "Update")
 *
 * CONVENTIONS
 *   b       number of LEVEL bits, 1..8.  s = 2^b - 1 quantization levels; one element costs b + 1
 *           bits on the wire (sign + level).  The paper counts the sign bit inside its b, so
 *           b_paper = b + 1 and its s = 2^(b_paper-1) - 1 is the same s.
 *   layout  Tensors ("segments") live in a padded flat index space P.  Segment l starts at P_l with
 *           P_0 = 0 and P_{l+1} = P_l + 128*ceil(len_l/128); D' = P_{n_seg}.  Gradients, the output
 *           and both bit planes are indexed by P.  Pad elements are ignored on input, encode as
 *           zero bits and are written as +0.0f on output.
 *   message One worker's message is [sign plane | level plane]: sign plane = D'/8 bytes, bit P of a
 *           little-endian bit array (byte P>>3, bit P&7), set when the IEEE sign bit of g_P is set;
 *           level plane = D'*b/8 bytes, element P in bits [P*b, P*b+b), least significant level bit
 *           first.  The norms and b travel beside the message (the B_pre bits of Eq. (7)).
 *   random  Element P of worker w at iteration `step` uses word P&3 of
 *           Philox4x32-10(counter = {lo32(P>>2), hi32(P>>2), w, step}, key = {lo32(seed), hi32(seed)});
 *           u = (word >> 8) * 2^-24; the level rounds up iff u < p_r (Eq. (6)).
 *
 * MEMORY    Pointers named *_dev are device pointers on the plan's GPU, 16-byte aligned, owned by
 *           the caller and borrowed until the enqueued work has finished.  Pointers named *_host
 *           are host pointers, read or written before the call returns.  The library allocates
 *           only the plan's tables (dq_plan_create / dq_plan_destroy) and the per-tensor width
 *           tables (dq_widths_create / dq_widths_destroy).
 * STREAMS   Device entry points enqueue on `hip_stream` (a hipStream_t passed as void*; NULL is
 *           the default stream) and return without synchronising.  They enqueue kernels only -- no
 *           allocation, memset or copy -- so a sequence of them can be captured into a HIP graph;
 *           the exceptions are dq_plan_create, dq_widths_create and dq_widths_set (allocation,
 *           host-to-device copies), which belong outside a capture.
 * ERRORS    Every int-returning function returns DQ_OK (0) or a negative dq_status; nothing
 *           throws, aborts or sets errno.  On error nothing has been enqueued.
 */
#ifndef DQ_H
#define DQ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum dq_status {
    DQ_OK = 0,
    DQ_ERR_INVALID_ARG = -1, /* null pointer, b outside 1..8, M < 1, misalignment, short stride ... */
    DQ_ERR_HIP = -2,         /* a HIP runtime call failed (no device, launch failure)            */
    DQ_ERR_ALLOC = -3        /* host or device allocation of the plan failed                     */
} dq_status;

#define DQ_GRANULE 128      /* segments are padded to a multiple of this many elements            */
#define DQ_MAX_WORKERS 64   /* largest M one call accepts                                         */
#define DQ_MIN_NORM 0x1p-100f /* a norm that is not >= this (zero, tiny, NaN) quantizes to zeros   */

typedef struct dq_plan dq_plan_t; /* opaque, immutable after creation, bound to one GPU */

/* Builds the layout of n_seg tensors of seg_len_host[l] >= 0 elements and uploads its tables to
 * the current HIP device.  Without a usable device the plan is still created for the host-side
 * size queries below, and every device entry point given it returns DQ_ERR_HIP. */
int dq_plan_create(const int64_t* seg_len_host, int32_t n_seg, dq_plan_t** plan_out);
void dq_plan_destroy(dq_plan_t* plan);

int32_t dq_plan_num_segments(const dq_plan_t* plan);
int64_t dq_plan_padded_elems(const dq_plan_t* plan);               /* D'                              */
int64_t dq_plan_segment_start(const dq_plan_t* plan, int32_t l);   /* P_l; -1 if l is out of range    */
int64_t dq_packed_bytes(const dq_plan_t* plan, int b);             /* per worker: D'/8 + D'*b/8; -1 on bad b */
int64_t dq_workspace_bytes(const dq_plan_t* plan, int M);          /* scratch dq_norm needs; -1 on bad M */
int dq_plan_has_device(const dq_plan_t* plan);                     /* 1 if the tables are on a GPU    */
/* 1 if no tensor crosses a multiple of 4096 in the padded index space -- e.g. a gradient cut into
 * buckets of 128*2^k <= 4096 elements, the practice of the scheme the paper builds on, or small
 * tensors laid out that way.  For such "chunk-local" plans dq_norm finishes every norm in one pass
 * however small the tensors, and dq_norm_quantize_pack is available. */
int dq_plan_is_chunk_local(const dq_plan_t* plan);

/* N[i][l] = ||g_l^(i)||_2, the norm of Eq. (5) (p = 2), for worker i's tensor l.
 *   grads_dev            [M] gradients in padded layout, worker i at grads_dev + i*worker_stride_elems
 *   worker_stride_elems  >= D', multiple of 4
 *   norms_dev            [M][n_seg] float, written
 *   workspace_dev        dq_workspace_bytes(plan, M) bytes of scratch, 16-byte aligned
 * Squares accumulate in binary64 in a fixed order, so the result is reproducible run to run. */
int dq_norm(const dq_plan_t* plan, const float* grads_dev, int64_t worker_stride_elems, int M,
            float* norms_dev, void* workspace_dev, void* hip_stream);

/* The same with p = infinity in Eq. (5): N[i][l] = max_j |g_j| over tensor l of worker i (0 for
 * an empty tensor; NaN elements are skipped).  With it no ratio |g_j|/N exceeds 1 and b = 1 is
 * the ternary scheme of the related work.  Arguments as dq_norm; the result is exact. */
int dq_norm_linf(const dq_plan_t* plan, const float* grads_dev, int64_t worker_stride_elems, int M,
                 float* norms_dev, void* workspace_dev, void* hip_stream);

/* dq_norm (linf = 0) or dq_norm_linf (linf != 0) for callers that cannot allocate device memory --
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc -- and so have
 * no workspace to hand over.  The partial results live in a fixed array inside the library instead
 * (DQ_NORM_STATIC_SCRATCH_BYTES of device memory on every GPU the library is loaded on, held until
 * the process ends); the call allocates and frees nothing and only enqueues the kernels of dq_norm,
 * so norms_dev receives exactly dq_norm's values.
 *   limit   dq_workspace_bytes(plan, M) <= DQ_NORM_STATIC_SCRATCH_BYTES, i.e. M * (number of
 *           4096-element pieces of the tensors) <= 2^20 -- e.g. M = 16 workers of 2^28 elements;
 *           DQ_ERR_INVALID_ARG beyond it (use dq_norm with a workspace of the caller's then).
 *   sharing every call on a GPU uses that GPU's one array: calls that may overlap on one GPU (two
 *           streams, two threads) race on it and give wrong norms; order them, or use dq_norm.
 *           Nothing in the array has to be cleared between calls.
 * The array's address is looked up when a plan is created on the GPU (at the latest by the first
 * call), never during later calls.  Other arguments and errors as dq_norm. */
#define DQ_NORM_STATIC_SCRATCH_BYTES (8 << 20)
int64_t dq_norm_static_scratch_max_bytes(void);
int dq_norm_static_scratch(const dq_plan_t* plan, const float* grads_dev, int64_t worker_stride_elems,
                           int M, int linf, float* norms_dev, void* hip_stream);

/* The bit rule, Eq. (17), in level-bit convention.  Pure host code, no GPU work.
 *   Gbar^2 = (1/M) sum_i sum_l N[i][l]^2        (mean square of the workers' gradient norms, Lemma 1)
 *   s*     = sqrt(T/eps_hat_q) * alpha^((T-1-t)/2) * Gbar
 *   b      = the smallest integer in [b_min, b_max] with 2^b - 1 >= s*, else b_max
 * which is Eq. (17) rounded up to an integer (b_paper = b + 1), so the error constraint of
 * Eq. (16) still holds.  Requires 0 <= t < T, eps_hat_q > 0, 0 < alpha <= 1, 1 <= b_min <= b_max <= 8.
 *   norms_host  [M][n_seg] float;  b_out receives b;  gbar_out (nullable) receives Gbar. */
int dq_select_bits(const float* norms_host, int M, int n_seg, int64_t t, int64_t T,
                   double eps_hat_q, double alpha, int b_min, int b_max, int* b_out,
                   double* gbar_out);

/* Eq. (17) for norms from dq_norm_linf: a worker's whole-gradient max norm is the largest of its
 * tensor norms, so Gbar^2 = (1/M) sum_i max_l N[i][l]^2 (with one scale per tensor the variance
 * bound of Lemma 1 is sum_l d_l N_l^2/(4 s^2) <= d max_l N_l^2/(4 s^2), so the constraint of
 * Eq. (16) is kept).  Otherwise identical to dq_select_bits. */
int dq_select_bits_linf(const float* norms_host, int M, int n_seg, int64_t t, int64_t T,
                        double eps_hat_q, double alpha, int b_min, int b_max, int* b_out,
                        double* gbar_out);

/* EWU quantizer of Eq. (5)-(6) fused with the packing of the message whose size Eq. (7) counts.
 * For worker w = worker_base + i, element P of tensor l with norm N = norms_dev[i][l]:
 *     a = min(|g_P| * (s / N), s);  level = floor(a) + [u < a - floor(a)]      (binary32, no FMA)
 * and level = 0 for every element of a tensor whose norm is not >= DQ_MIN_NORM.
 *   norms_dev   [M][n_seg] float, read (normally dq_norm's output)
 *   packed_dev  [M] messages, worker i at packed_dev + i*packed_worker_stride_bytes, written in
 *               full (dq_packed_bytes bytes each, pad bits zero)
 *   packed_worker_stride_bytes  >= dq_packed_bytes(plan, b), multiple of 16
 * Non-finite gradient values never cause an out-of-range access; their codes are unspecified. */
int dq_quantize_pack(const dq_plan_t* plan, const float* grads_dev, int64_t worker_stride_elems,
                     int M, const float* norms_dev, int b, uint64_t seed, uint32_t step,
                     uint32_t worker_base, uint8_t* packed_dev, int64_t packed_worker_stride_bytes,
                     void* hip_stream);

/* dq_norm (linf = 0) or dq_norm_linf (linf != 0) and dq_quantize_pack in one pass over the
 * gradient, for chunk-local plans and a bit-width that is already known (Algorithm 1: the worker
 * received b_t with x_t): every workgroup computes the norms of the tensors in its 4096-element
 * chunk from the values it holds in registers and quantizes them straight away, so the gradient
 * is read once, 4 + (b+1)/8 bytes per element in all.  norms_dev [M][n_seg] is written (the same
 * values dq_norm gives for this plan); the messages are those of dq_quantize_pack for these norms.
 * DQ_ERR_INVALID_ARG when the plan is not chunk-local. */
int dq_norm_quantize_pack(const dq_plan_t* plan, const float* grads_dev, int64_t worker_stride_elems,
                          int M, int linf, int b, uint64_t seed, uint32_t step, uint32_t worker_base,
                          float* norms_dev, uint8_t* packed_dev, int64_t packed_worker_stride_bytes,
                          void* hip_stream);

/* Server side of Algorithm 1: out_P = (1/M) sum_i sgn_{i,P} * level_{i,P} * (N[i][l] / s), every
 * worker's message read once.  The sum runs in binary32: workers ascending inside blocks of eight
 * (fused multiply-adds from zero), the block sums added in block order, then times 1/M -- at most
 * 7 + ceil(M/8) + 1 roundings for any element, so the result is within (M/8 + 8) * 2^-24 <= 1e-6
 * of the exact average of the dequantized terms, relative to their mean magnitude, for every
 * M <= DQ_MAX_WORKERS.
 *   out_dev  [D'] float, written in full (pads +0.0f). */
int dq_unpack_dequant_reduce(const dq_plan_t* plan, const uint8_t* packed_dev,
                             int64_t packed_worker_stride_bytes, int M, const float* norms_dev,
                             int b, float* out_dev, void* hip_stream);

/* dq_unpack_dequant_reduce fused with the server's model update of Algorithm 1 ("Update the
 * global parameters"): x_P <- x_P - eta * g_hat_P for every element, g_hat as above.
 *   x_dev     [D'] float, read and written (pad elements unchanged)
 *   ghat_dev  [D'] float or NULL: when given, g_hat is also written there as by
 *             dq_unpack_dequant_reduce. */
int dq_unpack_dequant_reduce_update(const dq_plan_t* plan, const uint8_t* packed_dev,
                                    int64_t packed_worker_stride_bytes, int M, const float* norms_dev,
                                    int b, float eta, float* x_dev, float* ghat_dev, void* hip_stream);

/* ---- one bit-width per tensor -------------------------------------------------------------
 * The single b of Algorithm 1 generalised to one b_l per tensor, all workers sharing it.
 *   message  [sign plane | level plane] as before; in the level plane the tensors' fields follow
 *            one another, tensor l taking 128*ceil(len_l/128) * b_l bits (a whole number of 16-byte
 *            pieces), its element j at bits [j*b_l, j*b_l + b_l) of that stretch.  With all b_l
 *            equal this is the single-width message.
 */

/* The bit rule per tensor.  Carrying the Lagrangian argument behind Eq. (17) (appendix "Proof of
 * Eq. (17)") through with one level count per tensor -- variance bound sum_l d_l Nbar_l^2/(4 s_l^2)
 * in place of Lemma 1's d Gbar^2/(4 s^2), cost sum_l d_l b_l -- gives
 *     s*_l = sqrt(T/eps_hat_q) * alpha^((T-1-t)/2) * Nbar_l,   Nbar_l^2 = (1/M) sum_i N[i][l]^2,
 * i.e. Eq. (17) with the tensor's own root-mean-square norm; b_l = smallest integer in
 * [b_min, b_max] with 2^b_l - 1 >= s*_l, else b_max.  No tensor gets more bits than dq_select_bits
 * gives the whole gradient.  Host code; arguments as dq_select_bits.
 *   b_out_host [n_seg] int32, written;  nbar_out_host [n_seg] double or NULL. */
int dq_select_bits_per_tensor(const float* norms_host, int M, int n_seg, int64_t t, int64_t T,
                              double eps_hat_q, double alpha, int b_min, int b_max,
                              int32_t* b_out_host, double* nbar_out_host);

/* Message size per worker for the widths b_host[n_seg] (each 1..8): D'/8 + sum_l pad_l*b_l/8.
 * Host code, needs no GPU.  -1 on a bad argument. */
int64_t dq_packed_bytes_v(const dq_plan_t* plan, const int32_t* b_host);

/* Eq. (7) with per-tensor widths, one iteration: W * sum_l (len_l*(b_l + 1) + B_pre) bits.  Host
 * code.  -1 on a bad argument. */
int64_t dq_comm_cost_bits_per_tensor(int W, const int64_t* seg_len_host, const int32_t* b_host,
                                     int32_t n_seg, int B_pre);

/* The widths as the kernels read them: a small table on the plan's GPU (24 bytes per tensor) that
 * dq_widths_set refills.  The plan must outlive it. */
typedef struct dq_widths dq_widths_t;
int dq_widths_create(const dq_plan_t* plan, dq_widths_t** widths_out); /* allocates; DQ_ERR_HIP without a GPU */
void dq_widths_destroy(dq_widths_t* widths);
/* Enqueues the upload of b_host[n_seg] (each 1..8; read before the call returns) on hip_stream.
 * Work that uses `widths` must be ordered after it, and work enqueued earlier with the previous
 * widths before it (same stream, or events).  Blocks only if the previous upload of this object
 * has not finished yet. */
int dq_widths_set(dq_widths_t* widths, const int32_t* b_host, void* hip_stream);
int64_t dq_widths_packed_bytes(const dq_widths_t* widths); /* for the widths last set; -1 before */

/* ---- one bit-width per worker (and tensor) ---------------------------------------------------
 * Lemma 1 is written for workers that share b_t.  With worker i using s_i levels the variance of
 * the average is (1/M^2) sum_i d N_i^2/(4 s_i^2); the Lagrangian argument behind Eq. (17) then
 * gives s*_i = sqrt(T/eps_hat_q) alpha^((T-1-t)/2) N_i -- Eq. (17) with the worker's own norm,
 * which a worker can evaluate without the server -- and N[i][l] in that place when every worker
 * also has a width per tensor.  Messages of one step then differ in length; each is the
 * per-tensor message for its worker's widths.
 */

/* b_out_host [M][n_seg]: per_tensor = 0: row i holds b_i from N_i = sqrt(sum_l N[i][l]^2);
 * per_tensor != 0: b[i][l] from N[i][l].  Rounding and clamping as dq_select_bits.  Host code. */
int dq_select_bits_per_worker(const float* norms_host, int M, int n_seg, int64_t t, int64_t T,
                              double eps_hat_q, double alpha, int b_min, int b_max, int per_tensor,
                              int32_t* b_out_host);

/* A widths table with one row per worker: dq_widths_set then takes b_host [M][n_seg], and the
 * *_v entry points given it must be called with the same M.  dq_widths_packed_bytes returns the
 * longest worker's message (what packed_worker_stride_bytes must cover),
 * dq_widths_worker_packed_bytes one worker's.  dq_select_bits_device does not accept such a table. */
int dq_widths_create_per_worker(const dq_plan_t* plan, int M, dq_widths_t** widths_out);
int64_t dq_widths_worker_packed_bytes(const dq_widths_t* widths, int worker);

/* The bit rules evaluated on the GPU, so that a step needs no round trip to the host: reads
 * norms_dev [M][n_seg] and fills `widths` for the kernels enqueued after it on the same stream.
 *   rule  0: dq_select_bits (one b for every tensor), 1: dq_select_bits_linf, 2: dq_select_bits_per_tensor
 * Same binary64 arithmetic and summation order as those host functions, hence the same widths.
 *   b_out_dev            [n_seg] int32 or NULL: the widths chosen (b_min for an empty tensor)
 *   gbar_out_dev         NULL, or [1] double for rules 0/1 (Gbar), [n_seg] double for rule 2 (Nbar_l)
 *   packed_bytes_out_dev NULL, or [1] int64: the message size for the widths chosen
 * Afterwards dq_widths_packed_bytes returns the size for b_max everywhere, the room every message
 * buffer used with these widths must have. */
int dq_select_bits_device(const dq_plan_t* plan, dq_widths_t* widths, const float* norms_dev, int M,
                          int64_t t, int64_t T, double eps_hat_q, double alpha, int b_min, int b_max,
                          int rule, int32_t* b_out_dev, double* gbar_out_dev,
                          int64_t* packed_bytes_out_dev, void* hip_stream);

/* dq_quantize_pack, dq_unpack_dequant_reduce and dq_unpack_dequant_reduce_update with the widths
 * of `widths` (created from `plan`, set at least once) in place of b.  Same arithmetic per element
 * with s = 2^(b_l) - 1 for tensor l; packed_worker_stride_bytes >= dq_widths_packed_bytes. */
int dq_quantize_pack_v(const dq_plan_t* plan, const dq_widths_t* widths, const float* grads_dev,
                       int64_t worker_stride_elems, int M, const float* norms_dev, uint64_t seed,
                       uint32_t step, uint32_t worker_base, uint8_t* packed_dev,
                       int64_t packed_worker_stride_bytes, void* hip_stream);
int dq_unpack_dequant_reduce_v(const dq_plan_t* plan, const dq_widths_t* widths, const uint8_t* packed_dev,
                               int64_t packed_worker_stride_bytes, int M, const float* norms_dev,
                               float* out_dev, void* hip_stream);
int dq_unpack_dequant_reduce_update_v(const dq_plan_t* plan, const dq_widths_t* widths,
                                      const uint8_t* packed_dev, int64_t packed_worker_stride_bytes, int M,
                                      const float* norms_dev, float eta, float* x_dev, float* ghat_dev,
                                      void* hip_stream);

/* ---- sign-only messages ---------------------------------------------------------------------
 * The one-bit-per-element baseline of the paper's Table 2 ("SignSGD": W*T*d bits, i.e. Eq. (7)
 * with b_paper = 1 and no norm; dq_comm_cost_bits with b = 0, n_norms = 0).  A worker's message is
 * the sign plane alone, D'/8 bytes in the layout above.  The paper does not say how the server
 * combines such messages; both rules in use are offered.
 */

/* packed_dev [M] sign planes, worker i at packed_dev + i*packed_worker_stride_bytes (>= D'/8,
 * multiple of 16), written in full; bit P set when the IEEE sign bit of g_P is set, pad bits 0. */
int dq_sign_pack(const dq_plan_t* plan, const float* grads_dev, int64_t worker_stride_elems, int M,
                 uint8_t* packed_dev, int64_t packed_worker_stride_bytes, void* hip_stream);

/* out_P = (1/M) sum_i c[i][l] * sgn_{i,P}, sgn = -1 where the bit is set, else +1; binary32 sum
 * over i ascending, then times 1/M.  scales_dev [M][n_seg] float (a scale per worker and tensor
 * that travelled beside the message, e.g. mean |g|) or NULL for c = 1.  Pads +0.0f. */
int dq_sign_reduce(const dq_plan_t* plan, const uint8_t* packed_dev, int64_t packed_worker_stride_bytes,
                   int M, const float* scales_dev, float* out_dev, void* hip_stream);

/* Majority vote: out_P = sgn(sum_i sgn_{i,P}) in {-1, 0, +1}, 0 on a tie.  Exact. */
int dq_sign_majority(const dq_plan_t* plan, const uint8_t* packed_dev, int64_t packed_worker_stride_bytes,
                     int M, float* out_dev, void* hip_stream);

/* dq_norm_quantize_pack with the widths of `widths`: one pass over the gradient for chunk-local
 * plans, per-tensor (e.g. per-bucket) widths that were decided beforehand. */
int dq_norm_quantize_pack_v(const dq_plan_t* plan, const dq_widths_t* widths, const float* grads_dev,
                            int64_t worker_stride_elems, int M, int linf, uint64_t seed, uint32_t step,
                            uint32_t worker_base, float* norms_dev, uint8_t* packed_dev,
                            int64_t packed_worker_stride_bytes, void* hip_stream);

/* One pass over the gradient for ANY plan, given a bracket for every norm and a bit-width that is
 * already known (Algorithm 1: the worker received b_t with x_t; the bracket is, say, the previous
 * iteration's norm give or take a margin).  Computes the norms of Eq. (5) -- l2 (linf = 0) or max
 * (linf != 0), as dq_norm / dq_norm_linf -- and the messages of dq_quantize_pack for exactly those
 * norms.
 *
 * Why one pass can be exact: for a fixed element and random number the level of Eq. (5)-(6) never
 * grows with the norm (s/N, its product with |g| and floor(a) + [u < a - floor(a)] are all monotone,
 * roundings included), so an element that gets the same level at both ends of the bracket gets it
 * for every norm inside.  The first kernel reads the gradient once, quantizes with both ends,
 * writes what is decided and records the few undecided elements (index and value); after the
 * norms are known a second kernel settles the recorded elements.  A tensor that lies inside one
 * 4096-element chunk needs no bracket (its norm is finished on the spot).  A chunk with
 * more than 63 undecided elements, a tensor whose bracket is unusable (not lo >= DQ_MIN_NORM,
 * lo <= hi, hi finite) or whose norm falls outside its bracket is quantized again from the
 * gradient: the result is the same for any bracket, only the time differs (a bracket that misses
 * every norm costs about a third more than the two separate calls).
 *   norm_lo_dev, norm_hi_dev  [M][n_seg] float, read
 *   norms_dev      [M][n_seg] float, written (l2: within 1 ulp of dq_norm's, same squares summed
 *                  chunk-wise; max: exact)
 *   packed_dev     as dq_quantize_pack
 *   workspace_dev  dq_bracketed_workspace_bytes(plan, M) bytes, 16-byte aligned; contents on entry
 *                  are ignored; two calls that may run at the same time need a workspace each
 *   stats_dev      NULL, or two int64 (8-byte aligned), written: [0] elements settled by the second
 *                  kernel, [1] chunks quantized again in full
 * Errors as dq_quantize_pack. */
int64_t dq_bracketed_workspace_bytes(const dq_plan_t* plan, int M); /* -1 on bad arguments */
/* The usual bracket: lo = N * (1 - margin), hi = N * (1 + margin) (binary32) for n norms N of an
 * earlier iteration, 0 <= margin < 1; all three arrays on the device, lo/hi written.  The call runs
 * on the current device (there is no plan to say which): make the norms' GPU current first. */
int dq_norm_bracket(const float* norms_dev, int64_t n, float margin, float* norm_lo_dev, float* norm_hi_dev,
                    void* hip_stream);
int dq_norm_quantize_pack_bracketed(const dq_plan_t* plan, const float* grads_dev, int64_t worker_stride_elems,
                                    int M, int linf, const float* norm_lo_dev, const float* norm_hi_dev, int b,
                                    uint64_t seed, uint32_t step, uint32_t worker_base, float* norms_dev,
                                    uint8_t* packed_dev, int64_t packed_worker_stride_bytes, void* workspace_dev,
                                    int64_t* stats_dev, void* hip_stream);

/* The same single pass with the widths of `widths` (one per tensor, shared by the workers or one
 * row per worker): the messages of dq_quantize_pack_v for the norms the call computes.  The table
 * may have been filled on the GPU (dq_select_bits_device), so a whole iteration -- this call, the
 * rule for the next iteration, dq_unpack_dequant_reduce_update_v -- needs no host round trip.
 * packed_worker_stride_bytes >= dq_widths_packed_bytes(widths); everything else as above. */
int dq_norm_quantize_pack_bracketed_v(const dq_plan_t* plan, const dq_widths_t* widths, const float* grads_dev,
                                      int64_t worker_stride_elems, int M, int linf, const float* norm_lo_dev,
                                      const float* norm_hi_dev, uint64_t seed, uint32_t step, uint32_t worker_base,
                                      float* norms_dev, uint8_t* packed_dev, int64_t packed_worker_stride_bytes,
                                      void* workspace_dev, int64_t* stats_dev, void* hip_stream);

/* Eq. (24), the practical estimate of the convergence factor: alpha_est = (F(x_t)/F(x_0))^(1/t).
 * Host code.  Returns -1 unless t >= 1, F_t > 0 and F_0 > 0. */
double dq_alpha_est(double F_t, double F_0, int64_t t);

/* Eq. (7), the communication cost of one iteration in bits: W * (d * (b + 1) + n_norms * B_pre),
 * b level bits plus the sign bit per element and B_pre bits for each norm a worker sends (the
 * paper has one norm per gradient; with per-tensor norms n_norms = n_seg).  b = 31 with
 * n_norms = 0 is uncompressed SGD.  Host code.  Returns -1 on a negative or out-of-range argument. */
int64_t dq_comm_cost_bits(int W, int64_t d, int b, int32_t n_norms, int B_pre);

const char* dq_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* DQ_H */
