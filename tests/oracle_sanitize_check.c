/*
 * Host-only sanitizer run of the oracle (test infrastructure, like the rest of oracle/).
 * Built by tests/test_oracle_sanitizers.py together with dqo.c under
 * -fsanitize=address,undefined and executed on the CPU: drives every entry point of the oracle
 * over ragged layouts with buffers sized exactly, so that any out-of-bounds access, misaligned
 * access, signed overflow or invalid shift in the oracle aborts the run.  Prints "ok" on success.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int64_t dqo_padded_elems(const int64_t *, int32_t);
int64_t dqo_packed_bytes(const int64_t *, int32_t, int);
int64_t dqo_packed_bytes_v(const int64_t *, int32_t, const int32_t *);
int dqo_norm(const int64_t *, int32_t, const float *, int64_t, int32_t, float *);
int dqo_norm_linf(const int64_t *, int32_t, const float *, int64_t, int32_t, float *);
int dqo_select_bits(const float *, int32_t, int32_t, int64_t, int64_t, double, double, int, int, int *, double *);
int dqo_select_bits_linf(const float *, int32_t, int32_t, int64_t, int64_t, double, double, int, int, int *, double *);
int dqo_select_bits_per_tensor(const float *, int32_t, int32_t, int64_t, int64_t, double, double, int, int,
                               int32_t *, double *);
int dqo_quantize_pack(const int64_t *, int32_t, const float *, int64_t, int32_t, const float *, int, uint64_t,
                      uint32_t, uint32_t, uint8_t *, int64_t, uint8_t *);
int dqo_unpack_dequant_reduce(const int64_t *, int32_t, const uint8_t *, int64_t, int32_t, const float *, int,
                              float *, uint8_t *);
int dqo_quantize_pack_v(const int64_t *, int32_t, const float *, int64_t, int32_t, const float *, const int32_t *,
                        uint64_t, uint32_t, uint32_t, uint8_t *, int64_t, uint8_t *);
int dqo_unpack_dequant_reduce_v(const int64_t *, int32_t, const uint8_t *, int64_t, int32_t, const float *,
                                const int32_t *, float *, uint8_t *);
int dqo_sign_pack(const int64_t *, int32_t, const float *, int64_t, int32_t, uint8_t *, int64_t);
int dqo_sign_reduce(const int64_t *, int32_t, const uint8_t *, int64_t, int32_t, const float *, int, float *);
int dqo_update(float *, const float *, int64_t, float);
int64_t dqo_comm_cost_bits(int, int64_t, int, int32_t, int);
int64_t dqo_comm_cost_bits_per_tensor(int, const int64_t *, const int32_t *, int32_t, int);

static uint64_t state = 0x9E3779B97F4A7C15ull;
static uint32_t next_u32(void)
{
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (uint32_t)(state >> 32);
}
static float next_float(void) { return ((float)(next_u32() >> 8) * 0x1p-24f - 0.5f) * 0.02f; }

#define CHECK(x) do { if (!(x)) { fprintf(stderr, "check failed: %s (line %d)\n", #x, __LINE__); return 1; } } while (0)

int main(void)
{
    const int64_t layouts[][6] = { { 1, 0, 127, 128, 129, 300 }, { 4097, 5, 0, 0, 64, 2048 }, { 77, 0, 0, 0, 0, 0 } };
    for (int L = 0; L < 3; ++L) {
        const int32_t n_seg = 6;
        const int64_t *seg = layouts[L];
        const int64_t dp = dqo_padded_elems(seg, n_seg);
        CHECK(dp > 0 && dp % 128 == 0);
        for (int32_t M = 1; M <= 5; M += 2) {
            float *g = malloc(sizeof(float) * (size_t)(M * dp));
            float *norms = malloc(sizeof(float) * (size_t)(M * n_seg));
            float *out = malloc(sizeof(float) * (size_t)dp);
            float *x = calloc((size_t)dp, sizeof(float));
            uint8_t *scratch = malloc((size_t)(2 * M * dp));
            int32_t widths[6];
            double nbar[6], gbar;
            int b;
            CHECK(g && norms && out && x && scratch);
            for (int64_t k = 0; k < M * dp; ++k) g[k] = next_float();
            g[0] = -0.0f;
            if (dp > 200) { g[130] = NAN; g[131] = INFINITY; }      /* non-finite inputs must stay in bounds */
            CHECK(dqo_norm_linf(seg, n_seg, g, dp, M, norms) == 0);
            CHECK(dqo_select_bits_linf(norms, M, n_seg, 3, 10, 0.05, 0.9, 1, 8, &b, &gbar) == 0);
            CHECK(dqo_norm(seg, n_seg, g, dp, M, norms) == 0);
            CHECK(dqo_select_bits(norms, M, n_seg, 9, 10, 0.05, 0.9, 1, 8, &b, &gbar) == 0);
            CHECK(dqo_select_bits_per_tensor(norms, M, n_seg, 0, 10, 0.05, 0.9, 1, 8, widths, nbar) == 0);
            for (int bb = 1; bb <= 8; ++bb) {
                const int64_t nbytes = dqo_packed_bytes(seg, n_seg, bb);
                uint8_t *pk = malloc((size_t)(M * nbytes));
                CHECK(pk && nbytes == dp / 8 + dp * bb / 8);
                CHECK(dqo_quantize_pack(seg, n_seg, g, dp, M, norms, bb, 0xD05C6Dull << 20, 0xFFFFFFFFu, 0xFFFFFFF0u,
                                        pk, nbytes, scratch) == 0);
                CHECK(dqo_unpack_dequant_reduce(seg, n_seg, pk, nbytes, M, norms, bb, out, scratch) == 0);
                CHECK(dqo_update(x, out, dp, 0.1f) == 0);
                free(pk);
            }
            for (int k = 0; k < n_seg; ++k) widths[k] = 1 + (int32_t)(next_u32() % 8);
            {
                const int64_t nbytes = dqo_packed_bytes_v(seg, n_seg, widths);
                uint8_t *pk = malloc((size_t)(M * nbytes));
                CHECK(pk && nbytes > 0);
                CHECK(dqo_quantize_pack_v(seg, n_seg, g, dp, M, norms, widths, 7, 1, 0, pk, nbytes, scratch) == 0);
                CHECK(dqo_unpack_dequant_reduce_v(seg, n_seg, pk, nbytes, M, norms, widths, out, scratch) == 0);
                CHECK(dqo_comm_cost_bits_per_tensor(M, seg, widths, n_seg, 32) > 0);
                free(pk);
            }
            {
                uint8_t *pk = malloc((size_t)(M * dp / 8));
                CHECK(pk);
                CHECK(dqo_sign_pack(seg, n_seg, g, dp, M, pk, dp / 8) == 0);
                CHECK(dqo_sign_reduce(seg, n_seg, pk, dp / 8, M, NULL, 1, out) == 0);
                CHECK(dqo_sign_reduce(seg, n_seg, pk, dp / 8, M, norms, 0, out) == 0);
                free(pk);
            }
            CHECK(dqo_comm_cost_bits(8, 11173962, 31, 0, 32) == 8ll * 11173962 * 32);
            free(g); free(norms); free(out); free(x); free(scratch);
        }
    }
    /* rejected arguments must be rejected, not crash */
    {
        const int64_t seg[1] = { 100 };
        float g[128] = { 0 }, n[1] = { 1.0f };
        uint8_t pk[256], scratch[256];
        int b;
        CHECK(dqo_quantize_pack(seg, 1, g, 128, 1, n, 0, 1, 0, 0, pk, 256, scratch) != 0);
        CHECK(dqo_quantize_pack(seg, 1, g, 128, 1, n, 9, 1, 0, 0, pk, 256, scratch) != 0);
        CHECK(dqo_quantize_pack(seg, 1, g, 128, 1, n, 4, 1, 0, 0, pk, 16, scratch) != 0);
        CHECK(dqo_select_bits(n, 1, 1, 5, 5, 0.1, 0.9, 1, 8, &b, NULL) != 0);
        CHECK(dqo_packed_bytes(seg, 1, 0) < 0);
    }
    puts("ok");
    return 0;
}
