/*
 * dqo -- CPU oracle for the DQ-SGD stochastic gradient quantizer hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the GPU library is
 * checked against.  It shares no code with the GPU library and is never called from it; only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may load it.
 *
 * What it computes, following the paper (arXiv 2107.14575):
 *   - the element-wise uniform (EWU) quantizer of Section 4.1, Eq. (5)-(6):
 *       Q_b[g_j] = ||g|| * sgn(g_j) * zeta(g_j, s),  zeta in {0, 1/s, ..., 1}, stochastic rounding
 *       with round-up probability p_r = s*|g_j|/||g|| - l;
 *   - the wire message whose size Eq. (7) counts: one sign bit plus the level bits per element
 *     (the norm travels beside it, the B_pre bits of Eq. (7));
 *   - the server average of Algorithm 1 (line "Average") / Eq. (2): (1/W) * sum_i Q_b[g^(i)];
 *   - the bit rule Eq. (17) with the mean square of worker norms G-bar_t^2 of Lemma 1.
 *
 * Conventions (the paper is silent or ambiguous on each; every choice is listed in the design
 * notes of the repository):
 *   - b counts LEVEL bits: s = 2^b - 1 levels, wire width b + 1.  The paper's b is b + 1.
 *   - the norm is the l2 norm, taken per tensor ("segment"); G-bar^2 uses the whole-gradient norm,
 *     i.e. the sum of squared segment norms of a worker.
 *   - tensors live in a padded flat index space P: segment l starts at P_l, P_0 = 0,
 *     P_{l+1} = P_l + 128*ceil(len_l/128).  Pad elements are ignored on input and encode as zero.
 *   - randomness: Philox4x32-10 (Salmon et al., SC'11), counter {lo32(P>>2), hi32(P>>2), worker,
 *     step}, key {lo32(seed), hi32(seed)}; element P uses output word P&3; u = (r>>8) * 2^-24;
 *     round up iff u < p (strict).
 *   - all float arithmetic touching the rounding decision is single IEEE binary32 operations
 *     (compile with -ffp-contract=off); the norm and the average accumulate in binary64.
 *
 * Pins (tests that do not use this file to check itself): Philox known answers and a big-integer
 * Python twin; exact enumeration of rounding outcomes for d <= 4; Monte-Carlo unbiasedness and
 * the Lemma 1 variance bound; grid reproduction; zero vector; numpy.linalg.norm; the closed form
 * of the Eq. (16) constraint for the bit rule.  Nothing here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

#define DQO_OK 0
#define DQO_ERR_INVALID_ARG (-1)

#define DQO_GRANULE 128

/* ------------------------------------------------------------------------------------------- */
/* Philox4x32-10: 10 rounds of two 32x32->64 multiplies; the key is bumped by the Weyl constants  */
/* between rounds (9 bumps).  Written from the published definition of the generator.             */
/* ------------------------------------------------------------------------------------------- */
void dqo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t prod0 = M0 * (uint64_t)c0;
        uint64_t prod1 = M1 * (uint64_t)c2;
        uint32_t hi0 = (uint32_t)(prod0 >> 32), lo0 = (uint32_t)prod0;
        uint32_t hi1 = (uint32_t)(prod1 >> 32), lo1 = (uint32_t)prod1;
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        if (round != 9) { k0 += W0; k1 += W1; }
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* ------------------------------------------------------------------------------------------- */
/* Layout helpers                                                                                 */
/* ------------------------------------------------------------------------------------------- */
static int64_t padded_len(int64_t len)
{
    return (len + DQO_GRANULE - 1) / DQO_GRANULE * DQO_GRANULE;
}

/* D' = total padded elements; -1 on invalid input */
int64_t dqo_padded_elems(const int64_t *seg_len, int32_t n_seg)
{
    if (!seg_len || n_seg < 1) return -1;
    int64_t total = 0;
    for (int32_t l = 0; l < n_seg; ++l) {
        if (seg_len[l] < 0) return -1;
        total += padded_len(seg_len[l]);
    }
    return total;
}

/* start of segment l in the padded space */
int64_t dqo_seg_start(const int64_t *seg_len, int32_t n_seg, int32_t l)
{
    int64_t p = 0;
    (void)n_seg;
    for (int32_t k = 0; k < l; ++k) p += padded_len(seg_len[k]);
    return p;
}

/* bytes of one worker's message: sign plane D'/8 then level plane D'*b/8 */
int64_t dqo_packed_bytes(const int64_t *seg_len, int32_t n_seg, int b)
{
    int64_t dp = dqo_padded_elems(seg_len, n_seg);
    if (dp < 0 || b < 1 || b > 8) return -1;
    return dp / 8 + dp * b / 8;
}

/* ------------------------------------------------------------------------------------------- */
/* O1: per-worker, per-segment l2 norm (the ||g||_p of Eq. (5) with p = 2).                       */
/* Squares of binary32 values are exact in binary64; the sum runs in index order in binary64.    */
/* ------------------------------------------------------------------------------------------- */
int dqo_norm(const int64_t *seg_len, int32_t n_seg, const float *grads, int64_t worker_stride,
             int32_t M, float *norms /* [M][n_seg] */)
{
    if (!seg_len || !grads || !norms || n_seg < 1 || M < 1) return DQO_ERR_INVALID_ARG;
    for (int32_t i = 0; i < M; ++i) {
        const float *g = grads + (int64_t)i * worker_stride;
        int64_t start = 0;
        for (int32_t l = 0; l < n_seg; ++l) {
            double acc = 0.0;
            for (int64_t j = 0; j < seg_len[l]; ++j) {
                double x = (double)g[start + j];
                acc += x * x;
            }
            norms[(int64_t)i * n_seg + l] = (float)sqrt(acc);
            start += padded_len(seg_len[l]);
        }
    }
    return DQO_OK;
}

/* A worker's squared whole-gradient norm ||g^(i)||^2 = sum_l N_{i,l}^2 (the term Lemma 1       */
/* averages over workers into G-bar_t^2): a plain running sum in binary64, tensors in index      */
/* order.  The squares of binary32 norms are exact in binary64.                                  */
static double worker_squared_norm(const float *row, int32_t n_seg)
{
    double total = 0.0;
    for (int32_t l = 0; l < n_seg; ++l) {
        double n = (double)row[l];
        total += n * n;
    }
    return total;
}

/* ------------------------------------------------------------------------------------------- */
/* O2: the bit rule, Eq. (17), in level-bit convention.                                           */
/*   G2 = (1/M) sum_i ||g^(i)||^2, ||g^(i)||^2 = sum_l N_{i,l}^2   (G-bar_t^2 of Lemma 1)         */
/*   s* = sqrt(T/eps_hat) * alpha^((T-1-t)/2) * sqrt(G2)                                          */
/* Eq. (17) reads b_paper = log2(s* + 1) + 1, i.e. 2^(b_paper-1) - 1 = s*; with b = b_paper - 1   */
/* and rounding up to an integer this is: the smallest b with 2^b - 1 >= s*, clamped.             */
/* ------------------------------------------------------------------------------------------- */
int dqo_select_bits(const float *norms /* [M][n_seg] */, int32_t M, int32_t n_seg, int64_t t,
                    int64_t T, double eps_hat_q, double alpha, int b_min, int b_max, int *b_out,
                    double *gbar_out)
{
    if (!norms || !b_out || M < 1 || n_seg < 1 || T < 1 || t < 0 || t >= T) return DQO_ERR_INVALID_ARG;
    if (!(eps_hat_q > 0.0) || !(alpha > 0.0) || !(alpha <= 1.0)) return DQO_ERR_INVALID_ARG;
    if (b_min < 1 || b_max > 8 || b_min > b_max) return DQO_ERR_INVALID_ARG;
    double sum = 0.0;
    for (int32_t i = 0; i < M; ++i) {
        /* ||g^(i)||^2 = sum_l N_{i,l}^2: a worker's squared norm first ...                        */
        double worker_sq = worker_squared_norm(norms + (int64_t)i * n_seg, n_seg);
        sum += worker_sq;       /* ... then the mean over workers, as Lemma 1 writes G-bar_t^2   */
    }
    double G2 = sum / (double)M;
    double gbar = sqrt(G2);
    double s_star = sqrt((double)T / eps_hat_q) * pow(alpha, (double)(T - 1 - t) / 2.0) * gbar;
    int b = b_max;
    for (int cand = b_min; cand <= b_max; ++cand) {
        double levels = (double)((1 << cand) - 1);
        if (levels >= s_star) { b = cand; break; }
    }
    *b_out = b;
    if (gbar_out) *gbar_out = gbar;
    return DQO_OK;
}

/* ------------------------------------------------------------------------------------------- */
/* The p = infinity choice of the norm in Eq. (5): N = max_j |g_j| per worker and segment.        */
/* A NaN element never becomes the maximum (every comparison with it is false).                  */
/* ------------------------------------------------------------------------------------------- */
int dqo_norm_linf(const int64_t *seg_len, int32_t n_seg, const float *grads, int64_t worker_stride,
                  int32_t M, float *norms /* [M][n_seg] */)
{
    if (!seg_len || !grads || !norms || n_seg < 1 || M < 1) return DQO_ERR_INVALID_ARG;
    for (int32_t i = 0; i < M; ++i) {
        const float *g = grads + (int64_t)i * worker_stride;
        int64_t start = 0;
        for (int32_t l = 0; l < n_seg; ++l) {
            float m = 0.0f;
            for (int64_t j = 0; j < seg_len[l]; ++j) {
                float a = fabsf(g[start + j]);
                if (a > m) m = a;
            }
            norms[(int64_t)i * n_seg + l] = m;
            start += padded_len(seg_len[l]);
        }
    }
    return DQO_OK;
}

/* The bit rule, Eq. (17), for p = infinity.  A worker's whole-gradient norm is the largest of    */
/* its segment norms, so G2 = (1/M) sum_i max_l N_{i,l}^2; with one scale per segment the         */
/* variance bound of Lemma 1 is sum_l d_l N_l^2 / (4 s^2) <= d max_l N_l^2 / (4 s^2), so the      */
/* constraint of Eq. (16) still holds with this G-bar.  The rest is as for p = 2.                 */
int dqo_select_bits_linf(const float *norms /* [M][n_seg] */, int32_t M, int32_t n_seg, int64_t t,
                         int64_t T, double eps_hat_q, double alpha, int b_min, int b_max,
                         int *b_out, double *gbar_out)
{
    if (!norms || !b_out || M < 1 || n_seg < 1 || T < 1 || t < 0 || t >= T) return DQO_ERR_INVALID_ARG;
    if (!(eps_hat_q > 0.0) || !(alpha > 0.0) || !(alpha <= 1.0)) return DQO_ERR_INVALID_ARG;
    if (b_min < 1 || b_max > 8 || b_min > b_max) return DQO_ERR_INVALID_ARG;
    double sum = 0.0;
    for (int32_t i = 0; i < M; ++i) {
        double top = 0.0;
        for (int32_t l = 0; l < n_seg; ++l) {
            double n = (double)norms[(int64_t)i * n_seg + l];
            if (n > top) top = n;
        }
        sum += top * top;
    }
    double gbar = sqrt(sum / (double)M);
    double s_star = sqrt((double)T / eps_hat_q) * pow(alpha, (double)(T - 1 - t) / 2.0) * gbar;
    int b = b_max;
    for (int cand = b_min; cand <= b_max; ++cand) {
        double levels = (double)((1 << cand) - 1);
        if (levels >= s_star) { b = cand; break; }
    }
    *b_out = b;
    if (gbar_out) *gbar_out = gbar;
    return DQO_OK;
}

/* ------------------------------------------------------------------------------------------- */
/* O3: sign and stochastic level of every element (Eq. (5)-(6)).                                  */
/* sign[i][P], level[i][P] are one byte per padded element; pads get 0/0.                         */
/* ------------------------------------------------------------------------------------------- */
static int norm_is_usable(float N)
{
    return N >= 0x1p-100f; /* false for zero, tiny and NaN norms: the zero-vector path */
}

/* Range form: only padded indices p_begin <= P < p_end (both multiples of 128) are computed.
 * grads points at element p_begin of worker 0 and worker i's slice starts worker_stride later;
 * sign/level are [M][p_end - p_begin].  The Philox counter uses the absolute index P. */
static int widths_ok(const int32_t *b_seg, int32_t n_seg)
{
    if (!b_seg) return 0;
    for (int32_t l = 0; l < n_seg; ++l)
        if (b_seg[l] < 1 || b_seg[l] > 8) return 0;
    return 1;
}

/* b_seg == NULL: every tensor uses b level bits; otherwise worker i's tensor l uses
 * b_seg[i * b_worker_stride + l] (b_worker_stride = 0: the workers share one set of per-tensor
 * widths; = n_seg: every worker has its own; both further down) and b is ignored. */
static int quantize_range(const int64_t *seg_len, int32_t n_seg, const float *grads,
                          int64_t worker_stride, int32_t M, const float *norms /* [M][n_seg] */, int b,
                          const int32_t *b_seg, int32_t b_worker_stride, uint64_t seed, uint32_t step,
                          uint32_t worker_base, int64_t p_begin, int64_t p_end, uint8_t *sign, uint8_t *level)
{
    if (!seg_len || !grads || !norms || !sign || !level) return DQO_ERR_INVALID_ARG;
    if (n_seg < 1 || M < 1) return DQO_ERR_INVALID_ARG;
    if (!b_seg && (b < 1 || b > 8)) return DQO_ERR_INVALID_ARG;
    for (int32_t i = 0; b_seg && i < (b_worker_stride ? M : 1); ++i)
        if (!widths_ok(b_seg + (int64_t)i * b_worker_stride, n_seg)) return DQO_ERR_INVALID_ARG;
    int64_t dp = dqo_padded_elems(seg_len, n_seg);
    if (dp < 0 || p_begin < 0 || p_end > dp || p_begin > p_end) return DQO_ERR_INVALID_ARG;
    if (p_begin % DQO_GRANULE || p_end % DQO_GRANULE) return DQO_ERR_INVALID_ARG;
    const int64_t span = p_end - p_begin;
    const uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };

#pragma omp parallel for schedule(static)
    for (int32_t i = 0; i < M; ++i) {
        const float *g = grads + (int64_t)i * worker_stride;
        uint8_t *sg = sign + (int64_t)i * span;
        uint8_t *lv = level + (int64_t)i * span;
        memset(sg, 0, (size_t)span);
        memset(lv, 0, (size_t)span);
        int64_t start = 0;
        for (int32_t l = 0; l < n_seg; ++l) {
            const int width = b_seg ? b_seg[(int64_t)i * b_worker_stride + l] : b;
            const float s = (float)((1u << width) - 1u); /* quantization levels */
            const float N = norms[(int64_t)i * n_seg + l];
            const int usable = norm_is_usable(N);
            const float scale = usable ? s / N : 0.0f; /* one binary32 division per segment */
            /* the tensor's elements that lie in [p_begin, p_end) */
            const int64_t j_lo = p_begin > start ? p_begin - start : 0;
            const int64_t j_hi = p_end - start < seg_len[l] ? p_end - start : seg_len[l];
            for (int64_t j = j_lo; j < j_hi; ++j) {
                const int64_t P = start + j;
                const int64_t q = P - p_begin;
                const float x = g[q];
                uint32_t bits;
                memcpy(&bits, &x, 4);
                sg[q] = (uint8_t)(bits >> 31);
                if (!usable) { lv[q] = 0; continue; }
                float a = fabsf(x) * scale;       /* s*|g_j|/||g||, one rounding            */
                a = fminf(a, s);                  /* |g_j|/||g|| may round above 1          */
                const float fl = floorf(a);       /* l of Eq. (6)                            */
                const float p = a - fl;           /* p_r of Eq. (6); exact                   */
                const uint64_t quad = (uint64_t)P >> 2;
                const uint32_t ctr[4] = { (uint32_t)quad, (uint32_t)(quad >> 32),
                                          worker_base + (uint32_t)i, step };
                uint32_t r[4];
                dqo_philox4x32_10(ctr, key, r);
                const float u = (float)(r[P & 3] >> 8) * 0x1p-24f; /* exact, in [0,1)        */
                lv[q] = (uint8_t)((uint32_t)fl + (u < p ? 1u : 0u));
            }
            start += padded_len(seg_len[l]);
        }
    }
    return DQO_OK;
}

int dqo_quantize_range(const int64_t *seg_len, int32_t n_seg, const float *grads,
                       int64_t worker_stride, int32_t M, const float *norms /* [M][n_seg] */, int b,
                       uint64_t seed, uint32_t step, uint32_t worker_base, int64_t p_begin,
                       int64_t p_end, uint8_t *sign, uint8_t *level)
{
    return quantize_range(seg_len, n_seg, grads, worker_stride, M, norms, b, NULL, 0, seed, step,
                          worker_base, p_begin, p_end, sign, level);
}

int dqo_quantize(const int64_t *seg_len, int32_t n_seg, const float *grads, int64_t worker_stride,
                 int32_t M, const float *norms /* [M][n_seg] */, int b, uint64_t seed,
                 uint32_t step, uint32_t worker_base, uint8_t *sign /* [M][D'] */,
                 uint8_t *level /* [M][D'] */)
{
    int64_t dp = dqo_padded_elems(seg_len, n_seg);
    if (dp < 0) return DQO_ERR_INVALID_ARG;
    return dqo_quantize_range(seg_len, n_seg, grads, worker_stride, M, norms, b, seed, step,
                              worker_base, 0, dp, sign, level);
}

/* ------------------------------------------------------------------------------------------- */
/* O4: the message.  Sign plane: bit P of a little-endian bit array (byte P>>3, bit P&7).         */
/* Level plane: element P occupies bits [P*b, P*b+b), least significant level bit first.          */
/* ------------------------------------------------------------------------------------------- */
static void put_bits(uint8_t *plane, int64_t bit_pos, int width, uint32_t value)
{
    for (int k = 0; k < width; ++k) {
        int64_t q = bit_pos + k;
        if ((value >> k) & 1u) plane[q >> 3] |= (uint8_t)(1u << (q & 7));
    }
}

static uint32_t get_bits(const uint8_t *plane, int64_t bit_pos, int width)
{
    uint32_t value = 0;
    for (int k = 0; k < width; ++k) {
        int64_t q = bit_pos + k;
        value |= (uint32_t)((plane[q >> 3] >> (q & 7)) & 1u) << k;
    }
    return value;
}

/* one worker: codes (one byte each) -> message of dp/8 + dp*b/8 bytes */
int dqo_pack(const uint8_t *sign, const uint8_t *level, int64_t dp, int b, uint8_t *packed)
{
    if (!sign || !level || !packed || dp < 0 || dp % DQO_GRANULE || b < 1 || b > 8)
        return DQO_ERR_INVALID_ARG;
    uint8_t *sign_plane = packed;
    uint8_t *level_plane = packed + dp / 8;
    memset(packed, 0, (size_t)(dp / 8 + dp * b / 8));
    for (int64_t P = 0; P < dp; ++P) {
        put_bits(sign_plane, P, 1, sign[P]);
        put_bits(level_plane, P * b, b, level[P]);
    }
    return DQO_OK;
}

int dqo_unpack(const uint8_t *packed, int64_t dp, int b, uint8_t *sign, uint8_t *level)
{
    if (!sign || !level || !packed || dp < 0 || dp % DQO_GRANULE || b < 1 || b > 8)
        return DQO_ERR_INVALID_ARG;
    const uint8_t *sign_plane = packed;
    const uint8_t *level_plane = packed + dp / 8;
    for (int64_t P = 0; P < dp; ++P) {
        sign[P] = (uint8_t)get_bits(sign_plane, P, 1);
        level[P] = (uint8_t)get_bits(level_plane, P * b, b);
    }
    return DQO_OK;
}

/* ------------------------------------------------------------------------------------------- */
/* O5: dequantize and average (Algorithm 1, server side; Eq. (2) divides by W).                   */
/*   unit_{i,l} = N_{i,l} / s  (binary32; 0 on the zero-vector path)                              */
/*   v_{i,P} = level * unit, negated when the sign bit is set                                     */
/*   out_P = (float)( (sum_i (double)v_{i,P}) / M ); pads are +0.                                 */
/* ------------------------------------------------------------------------------------------- */
/* Range form: codes are [M][p_end - p_begin] for padded indices p_begin <= P < p_end (multiples
 * of 128); out has p_end - p_begin entries. */
static int dequant_reduce_range(const int64_t *seg_len, int32_t n_seg, const uint8_t *sign,
                                const uint8_t *level, int32_t M, const float *norms /* [M][n_seg] */,
                                int b, const int32_t *b_seg, int32_t b_worker_stride, int64_t p_begin,
                                int64_t p_end, float *out)
{
    if (!seg_len || !sign || !level || !norms || !out) return DQO_ERR_INVALID_ARG;
    if (n_seg < 1 || M < 1) return DQO_ERR_INVALID_ARG;
    if (!b_seg && (b < 1 || b > 8)) return DQO_ERR_INVALID_ARG;
    for (int32_t i = 0; b_seg && i < (b_worker_stride ? M : 1); ++i)
        if (!widths_ok(b_seg + (int64_t)i * b_worker_stride, n_seg)) return DQO_ERR_INVALID_ARG;
    int64_t dp = dqo_padded_elems(seg_len, n_seg);
    if (dp < 0 || p_begin < 0 || p_end > dp || p_begin > p_end) return DQO_ERR_INVALID_ARG;
    if (p_begin % DQO_GRANULE || p_end % DQO_GRANULE) return DQO_ERR_INVALID_ARG;
    const int64_t span = p_end - p_begin;
    for (int64_t q = 0; q < span; ++q) out[q] = 0.0f;
    int64_t start = 0;
    for (int32_t l = 0; l < n_seg; ++l) {
        /* the tensor's elements that lie in [p_begin, p_end) */
        const int64_t j_lo = p_begin > start ? p_begin - start : 0;
        const int64_t j_hi = p_end - start < seg_len[l] ? p_end - start : seg_len[l];
#pragma omp parallel for schedule(static)
        for (int64_t j = j_lo; j < j_hi; ++j) {
            const int64_t P = start + j;
            const int64_t q = P - p_begin;
            double acc = 0.0;
            for (int32_t i = 0; i < M; ++i) {
                const int width = b_seg ? b_seg[(int64_t)i * b_worker_stride + l] : b;
                const float s = (float)((1u << width) - 1u);
                const float N = norms[(int64_t)i * n_seg + l];
                const float unit = norm_is_usable(N) ? N / s : 0.0f;
                float v = (float)level[(int64_t)i * span + q] * unit;
                if (sign[(int64_t)i * span + q]) v = -v;
                acc += (double)v;
            }
            out[q] = (float)(acc / (double)M);
        }
        start += padded_len(seg_len[l]);
    }
    return DQO_OK;
}

int dqo_dequant_reduce_range(const int64_t *seg_len, int32_t n_seg, const uint8_t *sign,
                             const uint8_t *level, int32_t M, const float *norms /* [M][n_seg] */,
                             int b, int64_t p_begin, int64_t p_end, float *out)
{
    return dequant_reduce_range(seg_len, n_seg, sign, level, M, norms, b, NULL, 0, p_begin, p_end, out);
}

int dqo_dequant_reduce(const int64_t *seg_len, int32_t n_seg, const uint8_t *sign /* [M][D'] */,
                       const uint8_t *level /* [M][D'] */, int32_t M,
                       const float *norms /* [M][n_seg] */, int b, float *out /* [D'] */)
{
    int64_t dp = dqo_padded_elems(seg_len, n_seg);
    if (dp < 0) return DQO_ERR_INVALID_ARG;
    return dqo_dequant_reduce_range(seg_len, n_seg, sign, level, M, norms, b, 0, dp, out);
}

/* ------------------------------------------------------------------------------------------- */
/* Whole passes on messages, the shape the GPU library's entry points have.                       */
/* ------------------------------------------------------------------------------------------- */

/* quantize + pack for M workers; worker i's message starts at packed + i*packed_stride.
 * scratch must hold 2*D' bytes per worker: 2*M*D' in total. */
int dqo_quantize_pack(const int64_t *seg_len, int32_t n_seg, const float *grads,
                      int64_t worker_stride, int32_t M, const float *norms, int b, uint64_t seed,
                      uint32_t step, uint32_t worker_base, uint8_t *packed, int64_t packed_stride,
                      uint8_t *scratch)
{
    if (!packed || !scratch) return DQO_ERR_INVALID_ARG;
    int64_t dp = dqo_padded_elems(seg_len, n_seg);
    if (dp < 0 || b < 1 || b > 8 || packed_stride < dp / 8 + dp * b / 8) return DQO_ERR_INVALID_ARG;
    uint8_t *sign = scratch, *level = scratch + (int64_t)M * dp;
    int rc = dqo_quantize(seg_len, n_seg, grads, worker_stride, M, norms, b, seed, step,
                          worker_base, sign, level);
    if (rc != DQO_OK) return rc;
#pragma omp parallel for schedule(static)
    for (int32_t i = 0; i < M; ++i)
        dqo_pack(sign + (int64_t)i * dp, level + (int64_t)i * dp, dp, b,
                 packed + (int64_t)i * packed_stride);
    return DQO_OK;
}

/* unpack + dequantize + average; scratch as above */
int dqo_unpack_dequant_reduce(const int64_t *seg_len, int32_t n_seg, const uint8_t *packed,
                              int64_t packed_stride, int32_t M, const float *norms, int b,
                              float *out, uint8_t *scratch)
{
    if (!packed || !scratch) return DQO_ERR_INVALID_ARG;
    int64_t dp = dqo_padded_elems(seg_len, n_seg);
    if (dp < 0 || b < 1 || b > 8 || M < 1) return DQO_ERR_INVALID_ARG;
    uint8_t *sign = scratch, *level = scratch + (int64_t)M * dp;
#pragma omp parallel for schedule(static)
    for (int32_t i = 0; i < M; ++i)
        dqo_unpack(packed + (int64_t)i * packed_stride, dp, b, sign + (int64_t)i * dp,
                   level + (int64_t)i * dp);
    return dqo_dequant_reduce(seg_len, n_seg, sign, level, M, norms, b, out);
}

/* ------------------------------------------------------------------------------------------- */
/* One bit-width per tensor.                                                                      */
/*                                                                                                */
/* The paper's problem (the program before Eq. (17), solved in its appendix "Proof of Eq. (17)")  */
/* has one b_t per iteration.  With one scale and one level count s_l = 2^(b_l) - 1 per tensor,   */
/* Lemma 1's bound on the quantization variance of an iteration becomes                           */
/*     sum_l d_l Nbar_l^2 / (4 s_l^2),     Nbar_l^2 = (1/M) sum_i N_{i,l}^2,                      */
/* in place of d Gbar^2/(4 s^2), so the constraint reads                                          */
/*     sum_t alpha^(T-1-t) sum_l (d_l/d) Nbar_{t,l}^2 / s_{t,l}^2 = eps_hat                       */
/* and the cost is sum_t sum_l d_l b_{t,l}.  The same Lagrangian steps (stationarity in b_{t,l},  */
/* 2^(b-1) ~ s as in the appendix) give s_{t,l} proportional to alpha^((T-1-t)/2) Nbar_{t,l}      */
/* -- d_l cancels -- and the constraint fixes the factor at sqrt(T/eps_hat):                      */
/*     s*_{t,l} = sqrt(T/eps_hat) * alpha^((T-1-t)/2) * Nbar_{t,l},                               */
/* Eq. (17) with the tensor's own root-mean-square norm in place of Gbar_t.  Integer rounding and */
/* clamping as for the single width; an all-zero tensor gets b_min.                               */
/* ------------------------------------------------------------------------------------------- */
int dqo_select_bits_per_tensor(const float *norms /* [M][n_seg] */, int32_t M, int32_t n_seg,
                               int64_t t, int64_t T, double eps_hat_q, double alpha, int b_min,
                               int b_max, int32_t *b_out /* [n_seg] */,
                               double *nbar_out /* [n_seg] or NULL */)
{
    if (!norms || !b_out || M < 1 || n_seg < 1 || T < 1 || t < 0 || t >= T) return DQO_ERR_INVALID_ARG;
    if (!(eps_hat_q > 0.0) || !(alpha > 0.0) || !(alpha <= 1.0)) return DQO_ERR_INVALID_ARG;
    if (b_min < 1 || b_max > 8 || b_min > b_max) return DQO_ERR_INVALID_ARG;
    const double factor = sqrt((double)T / eps_hat_q) * pow(alpha, (double)(T - 1 - t) / 2.0);
    for (int32_t l = 0; l < n_seg; ++l) {
        double sum = 0.0;
        for (int32_t i = 0; i < M; ++i) {
            double n = (double)norms[(int64_t)i * n_seg + l];
            sum += n * n;
        }
        double nbar = sqrt(sum / (double)M);
        double s_star = factor * nbar;
        int b = b_max;
        for (int cand = b_min; cand <= b_max; ++cand) {
            double levels = (double)((1 << cand) - 1);
            if (levels >= s_star) { b = cand; break; }
        }
        b_out[l] = b;
        if (nbar_out) nbar_out[l] = nbar;
    }
    return DQO_OK;
}

/* message bytes with per-tensor widths: D'/8 sign bytes, then tensor l's pad_l * b_l / 8 level bytes */
int64_t dqo_packed_bytes_v(const int64_t *seg_len, int32_t n_seg, const int32_t *b_seg)
{
    int64_t dp = dqo_padded_elems(seg_len, n_seg);
    if (dp < 0 || !widths_ok(b_seg, n_seg)) return -1;
    int64_t bytes = dp / 8;
    for (int32_t l = 0; l < n_seg; ++l) bytes += padded_len(seg_len[l]) * b_seg[l] / 8;
    return bytes;
}

/* Codes with per-tensor widths: tensor l is quantized as by dqo_quantize with b = b_l (the      */
/* element's random number does not depend on b).  Range form as dqo_quantize_range.              */
int dqo_quantize_v_range(const int64_t *seg_len, int32_t n_seg, const float *grads, int64_t worker_stride,
                         int32_t M, const float *norms, const int32_t *b_seg, uint64_t seed, uint32_t step,
                         uint32_t worker_base, int64_t p_begin, int64_t p_end, uint8_t *sign, uint8_t *level)
{
    if (!b_seg) return DQO_ERR_INVALID_ARG;
    return quantize_range(seg_len, n_seg, grads, worker_stride, M, norms, 0, b_seg, 0, seed, step,
                          worker_base, p_begin, p_end, sign, level);
}

int dqo_quantize_v(const int64_t *seg_len, int32_t n_seg, const float *grads, int64_t worker_stride,
                   int32_t M, const float *norms, const int32_t *b_seg, uint64_t seed, uint32_t step,
                   uint32_t worker_base, uint8_t *sign /* [M][D'] */, uint8_t *level /* [M][D'] */)
{
    int64_t dp = dqo_padded_elems(seg_len, n_seg);
    if (dp < 0) return DQO_ERR_INVALID_ARG;
    return dqo_quantize_v_range(seg_len, n_seg, grads, worker_stride, M, norms, b_seg, seed, step,
                                worker_base, 0, dp, sign, level);
}

/* The message with per-tensor widths.  Sign plane as before.  Level plane: the tensors' level   */
/* fields follow one another, tensor l taking pad_l * b_l bits (a whole number of 16-byte pieces), */
/* its element j at bits [j*b_l, j*b_l + b_l) of that stretch, least significant bit first.  With */
/* all widths equal this is the layout of dqo_pack.                                               */
int dqo_pack_v(const uint8_t *sign, const uint8_t *level, const int64_t *seg_len, int32_t n_seg,
               const int32_t *b_seg, uint8_t *packed)
{
    int64_t dp = dqo_padded_elems(seg_len, n_seg);
    int64_t bytes = dqo_packed_bytes_v(seg_len, n_seg, b_seg);
    if (!sign || !level || !packed || dp < 0 || bytes < 0) return DQO_ERR_INVALID_ARG;
    memset(packed, 0, (size_t)bytes);
    uint8_t *level_plane = packed + dp / 8;
    int64_t start = 0, bit0 = 0;
    for (int32_t l = 0; l < n_seg; ++l) {
        const int64_t pad = padded_len(seg_len[l]);
        for (int64_t j = 0; j < pad; ++j) {
            put_bits(packed, start + j, 1, sign[start + j]);
            put_bits(level_plane, bit0 + j * b_seg[l], b_seg[l], level[start + j]);
        }
        start += pad;
        bit0 += pad * b_seg[l];
    }
    return DQO_OK;
}

int dqo_unpack_v(const uint8_t *packed, const int64_t *seg_len, int32_t n_seg, const int32_t *b_seg,
                 uint8_t *sign, uint8_t *level)
{
    int64_t dp = dqo_padded_elems(seg_len, n_seg);
    if (!sign || !level || !packed || dp < 0 || !widths_ok(b_seg, n_seg)) return DQO_ERR_INVALID_ARG;
    const uint8_t *level_plane = packed + dp / 8;
    int64_t start = 0, bit0 = 0;
    for (int32_t l = 0; l < n_seg; ++l) {
        const int64_t pad = padded_len(seg_len[l]);
        for (int64_t j = 0; j < pad; ++j) {
            sign[start + j] = (uint8_t)get_bits(packed, start + j, 1);
            level[start + j] = (uint8_t)get_bits(level_plane, bit0 + j * b_seg[l], b_seg[l]);
        }
        start += pad;
        bit0 += pad * b_seg[l];
    }
    return DQO_OK;
}

/* Average with per-tensor widths: tensor l dequantizes with unit N_{i,l} / (2^(b_l) - 1).       */
int dqo_dequant_reduce_v_range(const int64_t *seg_len, int32_t n_seg, const uint8_t *sign, const uint8_t *level,
                               int32_t M, const float *norms, const int32_t *b_seg, int64_t p_begin,
                               int64_t p_end, float *out)
{
    if (!b_seg) return DQO_ERR_INVALID_ARG;
    return dequant_reduce_range(seg_len, n_seg, sign, level, M, norms, 0, b_seg, 0, p_begin, p_end, out);
}

int dqo_dequant_reduce_v(const int64_t *seg_len, int32_t n_seg, const uint8_t *sign, const uint8_t *level,
                         int32_t M, const float *norms, const int32_t *b_seg, float *out /* [D'] */)
{
    int64_t dp = dqo_padded_elems(seg_len, n_seg);
    if (dp < 0) return DQO_ERR_INVALID_ARG;
    return dqo_dequant_reduce_v_range(seg_len, n_seg, sign, level, M, norms, b_seg, 0, dp, out);
}

/* whole passes on messages with per-tensor widths; scratch holds 2*M*D' bytes */
int dqo_quantize_pack_v(const int64_t *seg_len, int32_t n_seg, const float *grads, int64_t worker_stride,
                        int32_t M, const float *norms, const int32_t *b_seg, uint64_t seed, uint32_t step,
                        uint32_t worker_base, uint8_t *packed, int64_t packed_stride, uint8_t *scratch)
{
    if (!packed || !scratch) return DQO_ERR_INVALID_ARG;
    int64_t dp = dqo_padded_elems(seg_len, n_seg);
    int64_t bytes = dqo_packed_bytes_v(seg_len, n_seg, b_seg);
    if (dp < 0 || bytes < 0 || packed_stride < bytes) return DQO_ERR_INVALID_ARG;
    uint8_t *sign = scratch, *level = scratch + (int64_t)M * dp;
    int rc = dqo_quantize_v(seg_len, n_seg, grads, worker_stride, M, norms, b_seg, seed, step, worker_base,
                            sign, level);
    if (rc != DQO_OK) return rc;
#pragma omp parallel for schedule(static)
    for (int32_t i = 0; i < M; ++i)
        dqo_pack_v(sign + (int64_t)i * dp, level + (int64_t)i * dp, seg_len, n_seg, b_seg,
                   packed + (int64_t)i * packed_stride);
    return DQO_OK;
}

int dqo_unpack_dequant_reduce_v(const int64_t *seg_len, int32_t n_seg, const uint8_t *packed,
                                int64_t packed_stride, int32_t M, const float *norms, const int32_t *b_seg,
                                float *out, uint8_t *scratch)
{
    if (!packed || !scratch || M < 1) return DQO_ERR_INVALID_ARG;
    int64_t dp = dqo_padded_elems(seg_len, n_seg);
    if (dp < 0) return DQO_ERR_INVALID_ARG;
    uint8_t *sign = scratch, *level = scratch + (int64_t)M * dp;
    if (!widths_ok(b_seg, n_seg)) return DQO_ERR_INVALID_ARG;
#pragma omp parallel for schedule(static)
    for (int32_t i = 0; i < M; ++i)
        dqo_unpack_v(packed + (int64_t)i * packed_stride, seg_len, n_seg, b_seg, sign + (int64_t)i * dp,
                     level + (int64_t)i * dp);
    return dqo_dequant_reduce_v(seg_len, n_seg, sign, level, M, norms, b_seg, out);
}

/* ------------------------------------------------------------------------------------------- */
/* One bit-width per worker and tensor.                                                           */
/*                                                                                                */
/* Lemma 1 is written for workers that share b_t; with worker i using s_i levels the variance of  */
/* the average is (1/M^2) sum_i d N_i^2 / (4 s_i^2), so the constraint term Gbar^2/s^2 =          */
/* (1/M) sum_i N_i^2 / s^2 becomes (1/M) sum_i N_i^2 / s_i^2 and the cost d sum_i b_i.  The       */
/* Lagrangian steps of the appendix give s_i proportional to alpha^((T-1-t)/2) N_i, and the       */
/* constraint fixes the factor: s*_{t,i} = sqrt(T/eps_hat) alpha^((T-1-t)/2) N_{t,i} -- Eq. (17)  */
/* with the worker's own norm, which a worker can evaluate without the server.  With a level      */
/* count per worker AND tensor the same argument gives N_{t,i,l} in that place.                   */
/*   per_tensor = 0: b[i][l] = b_i from N_i = sqrt(sum_l N_{i,l}^2);  1: b[i][l] from N_{i,l}.    */
/* ------------------------------------------------------------------------------------------- */
int dqo_select_bits_per_worker(const float *norms /* [M][n_seg] */, int32_t M, int32_t n_seg, int64_t t,
                               int64_t T, double eps_hat_q, double alpha, int b_min, int b_max,
                               int per_tensor, int32_t *b_out /* [M][n_seg] */)
{
    if (!norms || !b_out || M < 1 || n_seg < 1 || T < 1 || t < 0 || t >= T) return DQO_ERR_INVALID_ARG;
    if (!(eps_hat_q > 0.0) || !(alpha > 0.0) || !(alpha <= 1.0)) return DQO_ERR_INVALID_ARG;
    if (b_min < 1 || b_max > 8 || b_min > b_max) return DQO_ERR_INVALID_ARG;
    const double factor = sqrt((double)T / eps_hat_q) * pow(alpha, (double)(T - 1 - t) / 2.0);
    for (int32_t i = 0; i < M; ++i) {
        double worker_sq = worker_squared_norm(norms + (int64_t)i * n_seg, n_seg);
        for (int32_t l = 0; l < n_seg; ++l) {
            double n = per_tensor ? (double)norms[(int64_t)i * n_seg + l] : sqrt(worker_sq);
            double s_star = factor * n;
            int b = b_max;
            for (int cand = b_min; cand <= b_max; ++cand) {
                double levels = (double)((1 << cand) - 1);
                if (levels >= s_star) { b = cand; break; }
            }
            b_out[(int64_t)i * n_seg + l] = b;
        }
    }
    return DQO_OK;
}

/* Messages with per-worker widths b[i][l]: worker i's message is the per-tensor message for its */
/* own widths, so the messages of one step can differ in length; each starts at i*packed_stride. */
int dqo_quantize_pack_w(const int64_t *seg_len, int32_t n_seg, const float *grads, int64_t worker_stride,
                        int32_t M, const float *norms, const int32_t *b /* [M][n_seg] */, uint64_t seed,
                        uint32_t step, uint32_t worker_base, uint8_t *packed, int64_t packed_stride,
                        uint8_t *scratch /* 2*D' bytes */)
{
    if (!grads || !norms || !b || !packed || !scratch || M < 1) return DQO_ERR_INVALID_ARG;
    for (int32_t i = 0; i < M; ++i) {
        const int32_t *bi = b + (int64_t)i * n_seg;
        int64_t bytes = dqo_packed_bytes_v(seg_len, n_seg, bi);
        if (bytes < 0 || packed_stride < bytes) return DQO_ERR_INVALID_ARG;
        int rc = dqo_quantize_pack_v(seg_len, n_seg, grads + (int64_t)i * worker_stride, worker_stride, 1,
                                     norms + (int64_t)i * n_seg, bi, seed, step, worker_base + (uint32_t)i,
                                     packed + (int64_t)i * packed_stride, packed_stride, scratch);
        if (rc != DQO_OK) return rc;
    }
    return DQO_OK;
}

/* Average of messages with per-worker widths: worker i's tensor l dequantizes with unit        */
/* N_{i,l} / (2^(b[i][l]) - 1).  scratch holds 2*M*D' bytes.                                      */
int dqo_unpack_dequant_reduce_w(const int64_t *seg_len, int32_t n_seg, const uint8_t *packed,
                                int64_t packed_stride, int32_t M, const float *norms,
                                const int32_t *b /* [M][n_seg] */, float *out, uint8_t *scratch)
{
    if (!packed || !scratch || !b || M < 1) return DQO_ERR_INVALID_ARG;
    int64_t dp = dqo_padded_elems(seg_len, n_seg);
    if (dp < 0) return DQO_ERR_INVALID_ARG;
    uint8_t *sign = scratch, *level = scratch + (int64_t)M * dp;
    for (int32_t i = 0; i < M; ++i) {
        int rc = dqo_unpack_v(packed + (int64_t)i * packed_stride, seg_len, n_seg, b + (int64_t)i * n_seg,
                              sign + (int64_t)i * dp, level + (int64_t)i * dp);
        if (rc != DQO_OK) return rc;
    }
    return dequant_reduce_range(seg_len, n_seg, sign, level, M, norms, 0, b, n_seg, 0, dp, out);
}

/* Eq. (7) with per-tensor widths, one iteration: W [ sum_l d_l (b_l + 1) + n_seg B_pre ] bits. */
int64_t dqo_comm_cost_bits_per_tensor(int W, const int64_t *seg_len, const int32_t *b_seg, int32_t n_seg,
                                      int B_pre)
{
    if (W < 1 || !seg_len || n_seg < 1 || B_pre < 0 || !widths_ok(b_seg, n_seg)) return -1;
    int64_t bits = 0;
    for (int32_t l = 0; l < n_seg; ++l) {
        if (seg_len[l] < 0) return -1;
        bits += seg_len[l] * (int64_t)(b_seg[l] + 1) + B_pre;
    }
    return (int64_t)W * bits;
}

/* ------------------------------------------------------------------------------------------- */
/* Sign-only messages: the 1-bit-per-element baseline of the paper's Table 2 ("SignSGD", cost     */
/* W*T*d bits -- Eq. (7) with b_paper = 1 and no norm).  A worker sends the sign plane alone.     */
/* The paper does not say what the server does with it; the two rules in use are both here:       */
/*   mean:      out_P = (1/M) sum_i c_{i,l} * sgn_{i,P}, with a per-worker, per-tensor scale c    */
/*              that travels beside the message (1 when scales == NULL);                          */
/*   majority:  out_P = sgn( sum_i sgn_{i,P} ) in {-1, 0, +1} (0 on a tie).                       */
/* sgn is -1 when the IEEE sign bit is set, else +1 (so +0.0 votes +1, as in the quantizer).      */
/* ------------------------------------------------------------------------------------------- */
int dqo_sign_pack(const int64_t *seg_len, int32_t n_seg, const float *grads, int64_t worker_stride,
                  int32_t M, uint8_t *packed, int64_t packed_stride)
{
    if (!seg_len || !grads || !packed || n_seg < 1 || M < 1) return DQO_ERR_INVALID_ARG;
    int64_t dp = dqo_padded_elems(seg_len, n_seg);
    if (dp < 0 || packed_stride < dp / 8) return DQO_ERR_INVALID_ARG;
    for (int32_t i = 0; i < M; ++i) {
        uint8_t *msg = packed + (int64_t)i * packed_stride;
        const float *g = grads + (int64_t)i * worker_stride;
        memset(msg, 0, (size_t)(dp / 8));
        int64_t start = 0;
        for (int32_t l = 0; l < n_seg; ++l) {
            for (int64_t j = 0; j < seg_len[l]; ++j) {
                uint32_t bits;
                memcpy(&bits, &g[start + j], 4);
                put_bits(msg, start + j, 1, bits >> 31);
            }
            start += padded_len(seg_len[l]);
        }
    }
    return DQO_OK;
}

int dqo_sign_reduce(const int64_t *seg_len, int32_t n_seg, const uint8_t *packed, int64_t packed_stride,
                    int32_t M, const float *scales /* [M][n_seg] or NULL */, int majority,
                    float *out /* [D'] */)
{
    if (!seg_len || !packed || !out || n_seg < 1 || M < 1) return DQO_ERR_INVALID_ARG;
    int64_t dp = dqo_padded_elems(seg_len, n_seg);
    if (dp < 0 || packed_stride < dp / 8) return DQO_ERR_INVALID_ARG;
    for (int64_t q = 0; q < dp; ++q) out[q] = 0.0f;
    int64_t start = 0;
    for (int32_t l = 0; l < n_seg; ++l) {
        for (int64_t j = 0; j < seg_len[l]; ++j) {
            const int64_t P = start + j;
            double acc = 0.0;
            int votes = 0;
            for (int32_t i = 0; i < M; ++i) {
                const int neg = (int)get_bits(packed + (int64_t)i * packed_stride, P, 1);
                const double c = scales ? (double)scales[(int64_t)i * n_seg + l] : 1.0;
                acc += neg ? -c : c;
                votes += neg ? -1 : 1;
            }
            if (majority)
                out[P] = votes > 0 ? 1.0f : (votes < 0 ? -1.0f : 0.0f);
            else
                out[P] = (float)(acc / (double)M);
        }
        start += padded_len(seg_len[l]);
    }
    return DQO_OK;
}

/* ------------------------------------------------------------------------------------------- */
/* Server update of Algorithm 1: x_{t+1} = x_t - eta * g_hat_t (also Eq. (2)).  The product and   */
/* the difference are formed in binary64 and rounded once to binary32.                            */
/* ------------------------------------------------------------------------------------------- */
int dqo_update(float *x, const float *ghat, int64_t n, float eta)
{
    if (!x || !ghat || n < 0) return DQO_ERR_INVALID_ARG;
    for (int64_t j = 0; j < n; ++j) x[j] = (float)((double)x[j] - (double)eta * (double)ghat[j]);
    return DQO_OK;
}

/* Eq. (24): alpha_est = [F(x_t)/F(x_0)]^(1/t); -1 when undefined */
double dqo_alpha_est(double F_t, double F_0, int64_t t)
{
    if (t < 1 || !(F_t > 0.0) || !(F_0 > 0.0)) return -1.0;
    return pow(F_t / F_0, 1.0 / (double)t);
}

/* Eq. (7), one iteration: W [ d b_paper + B_pre ] bits with b_paper = b + 1; n_norms norms of
 * B_pre bits per worker (the paper has one). */
int64_t dqo_comm_cost_bits(int W, int64_t d, int b, int32_t n_norms, int B_pre)
{
    if (W < 1 || d < 0 || b < 0 || b > 31 || n_norms < 0 || B_pre < 0) return -1;
    return (int64_t)W * (d * (int64_t)(b + 1) + (int64_t)n_norms * B_pre);
}

/* threads the parallel loops use (1 when built without OpenMP) */
#ifdef _OPENMP
#include <omp.h>
int dqo_num_threads(void) { return omp_get_max_threads(); }
void dqo_set_num_threads(int n) { if (n > 0) omp_set_num_threads(n); }
#else
int dqo_num_threads(void) { return 1; }
void dqo_set_num_threads(int n) { (void)n; }
#endif
