// Host-only driver for a sanitizer build of the library's host code (AddressSanitizer +
// UndefinedBehaviorSanitizer on the host pass; no GPU is touched): the scheduling round on random
// prefix-sharing request streams with store / evict events between rounds, the threshold
// routines, and the argument checks of every GPU entry point (which return before any launch).
// Exit status 0 = every call returned what it should and no sanitizer report was raised.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../include/moe_prefill.h"
#include "../../include/moe_sched.h"

#define CHECK(cond)                                                             \
    do {                                                                        \
        if (!(cond)) {                                                          \
            std::fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #cond); \
            return 1;                                                           \
        }                                                                       \
    } while (0)

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd() {
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return (uint32_t)(rng_state >> 32);
}

int main() {
    // ---- scheduling round
    const int N = 5, B = 16;
    moe_sched_t* s = nullptr;
    CHECK(moe_sched_create(0, B, &s) == MOE_ERR_BAD_SHAPE);
    CHECK(moe_sched_create(N, B, nullptr) == MOE_ERR_NULL_PTR);
    CHECK(moe_sched_create(N, B, &s) == MOE_OK);
    std::vector<std::vector<int32_t>> roots(3);
    for (auto& r : roots) {
        r.resize(100 + rnd() % 300);
        for (auto& t : r) t = (int32_t)(rnd() % 32000);
    }
    moe_cost_model_t cost{44000.0, 3.0};
    for (int round = 0; round < 6; ++round) {
        const int R = 40 + (int)(rnd() % 60);
        std::vector<std::vector<int32_t>> prefix(R);
        std::vector<uint64_t> hashes;
        std::vector<int64_t> offs(R + 1, 0), P(R), S(R);
        for (int r = 0; r < R; ++r) {
            prefix[r] = roots[rnd() % 3];
            const int tail = (int)(rnd() % 200);
            for (int i = 0; i < tail; ++i) prefix[r].push_back((int32_t)(rnd() % 32000));
            if (r % 7 == 0) prefix[r].resize(rnd() % B);              // shorter than one block
            P[r] = (int64_t)prefix[r].size();
            S[r] = 1 + rnd() % 300;
            std::vector<uint64_t> h(prefix[r].size() / B);
            CHECK(moe_sched_hash_blocks(prefix[r].data(), P[r], B, h.data()) == MOE_OK);
            hashes.insert(hashes.end(), h.begin(), h.end());
            offs[r + 1] = (int64_t)hashes.size();
        }
        std::vector<double> loads(N, 0.0), delta(R);
        std::vector<int32_t> assigned(R);
        std::vector<int64_t> matched(R);
        int64_t done = -1;
        CHECK(moe_sched_round(s, &cost, 3.0e8, R, hashes.data(), offs.data(), P.data(), S.data(), loads.data(),
                              assigned.data(), matched.data(), delta.data(), &done) == MOE_OK);
        CHECK(done >= 0 && done <= R);
        for (int r = 0; r < R; ++r) {
            CHECK(assigned[r] >= -1 && assigned[r] < N);
            CHECK(matched[r] >= 0 && matched[r] <= P[r] && matched[r] % B == 0);
            if (assigned[r] >= 0 && offs[r + 1] > offs[r])
                CHECK(moe_sched_blocks_stored(s, assigned[r], hashes.data() + offs[r], offs[r + 1] - offs[r]) == MOE_OK);
        }
        // optional outputs may be NULL
        std::vector<double> loads2(N, 1.0e9);
        CHECK(moe_sched_round(s, &cost, 3.0e8, R, hashes.data(), offs.data(), P.data(), S.data(), loads2.data(),
                              assigned.data(), nullptr, nullptr, &done) == MOE_OK);
        CHECK(done == 0);
        if (round % 2 == 1 && !hashes.empty())
            for (int w = 0; w < N; ++w)
                CHECK(moe_sched_blocks_evicted(s, w, hashes.data() + rnd() % hashes.size(), 1) == MOE_OK);
        int64_t c = -1, p = -1;
        CHECK(moe_sched_table_size(s, round % N, &c, &p) == MOE_OK && c >= 0 && p >= 0);
        CHECK(moe_sched_tokens_executed(s, loads.data(), round % N, 1000, 44000.0) == MOE_OK);
        CHECK(moe_sched_tokens_executed(s, loads.data(), N, 1, 1.0) != MOE_OK);
    }
    CHECK(moe_sched_round(s, &cost, 1.0, 0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                          nullptr) != MOE_OK);
    moe_sched_destroy(s);
    moe_sched_destroy(nullptr);

    // ---- thresholds
    CHECK(moe_saturation_threshold_flops(4e-3, 2.5e15, 1.2) > 1.19e13);
    CHECK(moe_calibrated_threshold_flops(0.0, 5.0, 3e14, 1.2) == 1.2 * 3e14);
    double t = 0.0;
    int32_t unit = -1;
    CHECK(moe_resolve_threshold(0.0, 1e-2, 2.5e-2, 0.0, 8192.0, 1.2, &t, &unit) == MOE_OK && unit == MOE_UNIT_TOKENS);
    CHECK(moe_resolve_threshold(0.0, 1e-2, 2.5e-2, 1.0, 8192.0, 1.2, nullptr, &unit) == MOE_ERR_NULL_PTR);

    // ---- argument checks of the GPU entry points: every call must fail on the host
    moe_config_t c{64, 128, 8, 2, 128, MOE_DTYPE_BF16, MOE_DTYPE_BF16, MOE_DTYPE_F32, 0};
    size_t n = 0;
    for (int call = 0; call < 5; ++call) CHECK(moe_workspace_bytes(&c, call, &n) == MOE_OK);
    CHECK(moe_workspace_bytes(&c, 9, &n) == MOE_ERR_UNSUPPORTED);
    CHECK(moe_workspace_bytes(nullptr, 0, &n) == MOE_ERR_NULL_PTR);
    moe_config_t bad = c;
    bad.K = 9;
    CHECK(moe_workspace_bytes(&bad, 0, &n) == MOE_ERR_BAD_SHAPE);
    void* fake = reinterpret_cast<void*>(0x1000);            // never dereferenced: validation fails first
    float* ff = static_cast<float*>(fake);
    int32_t* fi = static_cast<int32_t*>(fake);
    CHECK(moe_route(&c, nullptr, ff, nullptr, ff, fi, ff, nullptr, 0, nullptr) == MOE_ERR_NULL_PTR);
    CHECK(moe_route(&c, fake, ff, nullptr, nullptr, fi, ff, fake, 16, nullptr) == MOE_ERR_WORKSPACE_TOO_SMALL);
    CHECK(moe_permute(&c, fi, nullptr, fi, fi, fi, fi, nullptr, fake, 0, nullptr) == MOE_ERR_WORKSPACE_TOO_SMALL);
    CHECK(moe_grouped_ffn(&c, fake, fi, fi, fake, fake, fake, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, ff,
                          fake, 0, nullptr) == MOE_ERR_WORKSPACE_TOO_SMALL);
    CHECK(moe_combine(&c, ff, fi, nullptr, fake, nullptr) == MOE_ERR_NULL_PTR);
    CHECK(moe_prefill_layer(&c, fake, ff, nullptr, fake, fake, fake, nullptr, nullptr, nullptr, fake, nullptr, fake,
                            1024, nullptr) == MOE_ERR_WORKSPACE_TOO_SMALL);
    moe_config_t big{1 << 20, 256, 1024, 2, 256, MOE_DTYPE_BF16, MOE_DTYPE_BF16, MOE_DTYPE_F32, 0};
    CHECK(moe_permute_noalloc(&big, fi, nullptr, fi, fi, fi, fi, nullptr, nullptr) == MOE_ERR_TOO_LARGE);
    CHECK(moe_quantize_rows_e4m3(fake, 4, 12, static_cast<uint8_t*>(fake), ff, nullptr) == MOE_ERR_BAD_SHAPE);
    size_t wb = 0;
    CHECK(moe_layer_weight_bytes(&c, &wb) == MOE_OK && wb == 3u * 8 * 128 * 128 * 2);
    CHECK(moe_prefill_layers_streamed(&c, 1, nullptr, fake, nullptr, 1, 0, nullptr, nullptr, fake, 1 << 30, fake,
                                      nullptr) == MOE_ERR_NULL_PTR);
    for (int st = 0; st >= -9; --st) CHECK(moe_status_string(st) != nullptr);
    std::printf("sanitize_driver: ok\n");
    return 0;
}
