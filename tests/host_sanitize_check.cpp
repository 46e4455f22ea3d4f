// Host-only sanitizer run of the library's host code (not part of libdq.so): built by
// tests/test_library_sanitizers.py with the host pass under AddressSanitizer and
// UndefinedBehaviorSanitizer, and run on the CPU.  Exercises plan creation over ragged layouts,
// the size queries, the three bit rules, the cost accounting and the argument checks of the device
// entry points (which return before any launch).  Prints "ok" on success.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <vector>

#include "dq.h"

#define CHECK(x)                                                                 \
    do {                                                                         \
        if (!(x)) {                                                              \
            std::fprintf(stderr, "check failed: %s (line %d)\n", #x, __LINE__);  \
            return 1;                                                            \
        }                                                                        \
    } while (0)

int main()
{
    uint64_t state = 0x9E3779B97F4A7C15ull;
    auto next = [&]() {
        state ^= state << 13; state ^= state >> 7; state ^= state << 17;
        return static_cast<uint32_t>(state >> 32);
    };
    const int64_t choices[] = { 0, 1, 5, 127, 128, 129, 1000, 4096, 4097, 70001 };
    for (int round = 0; round < 40; ++round) {
        const int32_t n_seg = 1 + static_cast<int32_t>(next() % 40);
        std::vector<int64_t> seg(n_seg);
        for (auto& s : seg) s = choices[next() % 10];
        dq_plan_t* plan = nullptr;
        CHECK(dq_plan_create(seg.data(), n_seg, &plan) == DQ_OK && plan);
        CHECK(dq_plan_num_segments(plan) == n_seg);
        int64_t dp = 0;
        bool local = true;
        for (int32_t l = 0; l < n_seg; ++l) {
            CHECK(dq_plan_segment_start(plan, l) == dp);
            const int64_t pad = (seg[l] + 127) / 128 * 128;
            if (seg[l] > 0 && dp / 4096 != (dp + pad - 1) / 4096) local = false;
            dp += pad;
        }
        CHECK(dq_plan_padded_elems(plan) == dp && dq_plan_segment_start(plan, n_seg) == -1);
        CHECK((dq_plan_is_chunk_local(plan) != 0) == local);
        for (int b = 0; b <= 9; ++b) CHECK(dq_packed_bytes(plan, b) == (b >= 1 && b <= 8 ? dp / 8 + dp * b / 8 : -1));
        const int M = 1 + static_cast<int>(next() % 16);
        CHECK(dq_workspace_bytes(plan, M) >= 16 && dq_workspace_bytes(plan, 0) == -1);
        std::vector<float> norms(static_cast<size_t>(M) * n_seg);
        for (auto& v : norms) v = static_cast<float>(next() % 1000) * 1e-3f;
        std::vector<int32_t> widths(n_seg);
        std::vector<double> nbar(n_seg);
        int b = 0;
        double gbar = 0;
        CHECK(dq_select_bits(norms.data(), M, n_seg, 2, 7, 0.01, 0.95, 1, 8, &b, &gbar) == DQ_OK && b >= 1 && b <= 8);
        CHECK(dq_select_bits_linf(norms.data(), M, n_seg, 6, 7, 0.01, 0.95, 2, 6, &b, nullptr) == DQ_OK && b >= 2 && b <= 6);
        CHECK(dq_select_bits_per_tensor(norms.data(), M, n_seg, 0, 7, 0.01, 0.95, 1, 8, widths.data(), nbar.data()) == DQ_OK);
        CHECK(dq_packed_bytes_v(plan, widths.data()) >= dp / 8);
        CHECK(dq_comm_cost_bits_per_tensor(M, seg.data(), widths.data(), n_seg, 32) > 0);
        widths[0] = 9;
        CHECK(dq_packed_bytes_v(plan, widths.data()) == -1);
        // argument checks of the device entry points: nothing is launched
        float* fake = reinterpret_cast<float*>(0x1000);
        uint8_t* fake8 = reinterpret_cast<uint8_t*>(0x1000);
        CHECK(dq_norm(plan, nullptr, dp, M, fake, fake, nullptr) == DQ_ERR_INVALID_ARG);
        CHECK(dq_quantize_pack(plan, fake, dp, M, fake, 0, 1, 0, 0, fake8, 1 << 30, nullptr) == DQ_ERR_INVALID_ARG);
        CHECK(dq_unpack_dequant_reduce(plan, fake8, 16, M, fake, 4, fake, nullptr) == DQ_ERR_INVALID_ARG || dp == 0);
        CHECK(dq_sign_pack(plan, fake, dp, 0, fake8, 1 << 30, nullptr) == DQ_ERR_INVALID_ARG);
        CHECK(dq_quantize_pack_v(plan, nullptr, fake, dp, M, fake, 1, 0, 0, fake8, 1 << 30, nullptr) == DQ_ERR_INVALID_ARG);
        // one pass with bracketed norms: the workspace covers its four parts; bad arguments are refused
        CHECK(dq_bracketed_workspace_bytes(plan, M) >= (dp + 4095) / 4096 * 256 * M && dq_bracketed_workspace_bytes(plan, 0) == -1);
        CHECK(dq_bracketed_workspace_bytes(plan, M) % 256 == 0 && dq_bracketed_workspace_bytes(nullptr, M) == -1);
        CHECK(dq_norm_quantize_pack_bracketed(plan, fake, dp, M, 0, fake, fake, 9, 1, 0, 0, fake, fake8, 1 << 30, fake8, nullptr, nullptr) == DQ_ERR_INVALID_ARG);
        CHECK(dq_norm_quantize_pack_bracketed_v(plan, nullptr, fake, dp, M, 0, fake, fake, 1, 0, 0, fake, fake8, 1 << 30, fake8, nullptr, nullptr) == DQ_ERR_INVALID_ARG);
        CHECK(dq_norm_quantize_pack_bracketed(plan, fake, dp, M, 1, nullptr, fake, 4, 1, 0, 0, fake, fake8, 1 << 30, fake8, nullptr, nullptr) == DQ_ERR_INVALID_ARG);
        dq_plan_destroy(plan);
    }
    dq_plan_t* none = nullptr;
    const int64_t bad[2] = { 5, -1 };
    CHECK(dq_plan_create(bad, 2, &none) == DQ_ERR_INVALID_ARG && !none);
    CHECK(dq_comm_cost_bits(8, 11173962, 31, 0, 32) == INT64_C(8) * 11173962 * 32);
    CHECK(std::fabs(dq_alpha_est(0.5, 1.0, 10) - std::pow(0.5, 0.1)) < 1e-15 && dq_alpha_est(0.0, 1.0, 3) == -1.0);
    dq_plan_destroy(nullptr);
    dq_widths_destroy(nullptr);
    std::puts("ok");
    return 0;
}
