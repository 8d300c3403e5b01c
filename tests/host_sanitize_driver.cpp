// Exercises the host-only part of libcovap (planner, queries, policy, knobs)
// under AddressSanitizer and UBSan.  Built and run by tests/test_host_sanitize.py
// with g++; plan.cpp needs no HIP headers.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "covap.h"

#define CHECK(c)                                                        \
    do {                                                                \
        if (!(c)) {                                                     \
            std::fprintf(stderr, "CHECK failed: %s (line %d)\n", #c, __LINE__); \
            return 1;                                                   \
        }                                                               \
    } while (0)

static int exercise(const std::vector<int64_t> &numel, int32_t mode, int32_t dtype, int64_t S,
                    int64_t cap, int32_t K, int64_t ref)
{
    covap_plan_opts_t o = {dtype, mode, S, cap, ref, K, 0};
    covap_plan_t *p = nullptr;
    CHECK(covap_plan(numel.data(), (int32_t)numel.size(), &o, &p) == COVAP_OK);
    const int32_t ns = covap_plan_num_shards(p), nb = covap_plan_num_buckets(p);
    int64_t covered = 0, prev_end = 0;
    for (int32_t s = 0; s < ns; ++s) {
        int64_t off, len;
        int32_t b;
        CHECK(covap_plan_shard(p, s, &off, &len, &b) == COVAP_OK);
        CHECK(off >= prev_end && len > 0 && b >= 0 && b < nb);
        prev_end = off + len;
        covered += len;
    }
    CHECK(prev_end <= covap_plan_total_elems(p));
    int64_t sum = 0;
    for (int64_t n : numel) sum += n;
    CHECK(covered == sum);
    for (int32_t b = 0; b < nb; ++b) {
        int32_t lo, hi;
        CHECK(covap_plan_bucket(p, b, &lo, &hi) == COVAP_OK && lo < hi);
    }
    std::vector<int32_t> ids((size_t)ns + 1);
    for (uint64_t t = 0; t < (uint64_t)(2 * K + 1); ++t) {
        const int32_t n = covap_plan_selected(p, t, ids.data(), ns);
        CHECK(n >= 0 && n <= ns);
        for (int32_t i = 0; i < n; ++i) CHECK(covap_plan_is_selected(p, t, ids[i]) == 1);
        CHECK(covap_plan_packed_elems(p, t, -1) <= covap_plan_packed_elems_max(p));
        int64_t prev = 0;
        for (int32_t b = 0; b < nb; ++b) {
            const int64_t e = covap_plan_packed_elems(p, t, b), base = covap_plan_packed_base(p, t, b);
            CHECK(e >= 0 && base >= 0);
            if (e > 0) {
                CHECK(base >= prev);
                prev = base + e;
            }
        }
        CHECK(prev <= covap_plan_packed_elems(p, t, -1));
    }
    // replay of the launch geometry: the tiles of a call add up to the elements of its shards,
    // stay inside the arena, and the sent ones stay inside the step's payload
    const bool small = covap_plan_total_elems(p) < (1 << 20);
    for (uint64_t t = 0; t < (uint64_t)(small ? K + 1 : 2) && t < 5; ++t) {
        for (int32_t b = -1; b < (small ? nb : 0); ++b) {
            for (int32_t tile : {256, 8192}) {
                for (int32_t sent_only = 0; sent_only < 2; ++sent_only) {
                    int32_t launches = 0;
                    int64_t groups = 0;
                    const int64_t cnt = covap_plan_trace(p, t, b, tile, sent_only, 0, nullptr, nullptr, nullptr,
                                                         nullptr, &launches, &groups);
                    CHECK(cnt >= 0 && groups >= cnt);
                    std::vector<int64_t> off((size_t)cnt + 1), poff((size_t)cnt + 1);
                    std::vector<int32_t> n((size_t)cnt + 1);
                    std::vector<uint8_t> sel((size_t)cnt + 1);
                    CHECK(covap_plan_trace(p, t, b, tile, sent_only, cnt, off.data(), poff.data(), n.data(),
                                           sel.data(), nullptr, nullptr) == cnt);
                    int64_t elems = 0, sent = 0;
                    for (int64_t i = 0; i < cnt; ++i) {
                        CHECK(n[(size_t)i] >= 1 && n[(size_t)i] <= tile && off[(size_t)i] >= 0);
                        CHECK(off[(size_t)i] + n[(size_t)i] <= covap_plan_total_elems(p));
                        elems += n[(size_t)i];
                        if (sel[(size_t)i]) {
                            sent += n[(size_t)i];
                            CHECK(poff[(size_t)i] >= covap_plan_packed_base(p, t, b));
                            CHECK(poff[(size_t)i] + n[(size_t)i] <=
                                  covap_plan_packed_base(p, t, b) + covap_plan_packed_elems(p, t, b));
                        }
                    }
                    int64_t want = 0, want_sent = 0;
                    int32_t lo = 0, hi = ns;
                    if (b >= 0) CHECK(covap_plan_bucket(p, b, &lo, &hi) == COVAP_OK);
                    for (int32_t s = lo; s < hi; ++s) {
                        int64_t len;
                        CHECK(covap_plan_shard(p, s, nullptr, &len, nullptr) == COVAP_OK);
                        const bool is_sent = covap_plan_is_selected(p, t, s) == 1;
                        if (is_sent) want_sent += len;
                        if (is_sent || !sent_only) want += len;
                    }
                    CHECK(elems == want && sent == want_sent);
                }
            }
        }
    }
    CHECK(covap_plan_trace(p, 0, -1, 100, 0, 0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == -1);
    CHECK(covap_plan_shard(p, ns, nullptr, nullptr, nullptr) == COVAP_ERANGE);
    CHECK(covap_plan_packed_elems(p, 0, nb) == -1);
    CHECK(covap_plan_tensor_offset(p, (int32_t)numel.size()) == -1);
    covap_plan_free(p);
    return 0;
}

int main()
{
    const std::vector<int64_t> vgg = {4101096, 16781312, 107480576, 7079424, 7669760, 555072};
    const std::vector<int64_t> odd = {1003, 2001, 30007, 5, 4099, 17, 90001, 3, 0, 8};
    for (int32_t dtype = 0; dtype <= 2; ++dtype) {
        const int64_t epv = dtype == 0 ? 4 : 8;
        for (int32_t K : {1, 2, 3, 7, 16, 1000}) {
            if (exercise(vgg, COVAP_SHARD_FIXED, dtype, 1 << 20, 25 << 20, K, 0)) return 1;
            if (exercise(odd, COVAP_SHARD_FIXED, dtype, epv, 64, K, 0)) return 1;
            if (exercise(odd, COVAP_SHARD_FIXED, dtype, 1 << 30, 1, K, 0)) return 1;
            if (exercise(vgg, COVAP_SHARD_MEDIAN, dtype, 0, 4, K, 5590260)) return 1;
            if (exercise(vgg, COVAP_SHARD_MEDIAN, dtype, 0, 25 << 20, K, 0)) return 1;
            if (exercise(odd, COVAP_SHARD_MEDIAN, dtype, 0, 20000, K, 0)) return 1;
            if (exercise(odd, COVAP_SHARD_MEDIAN, dtype, 0, 1, K, 1)) return 1;
        }
    }
    covap_plan_t *p = nullptr;
    covap_plan_opts_t bad = {0, 0, 6, 100, 0, 2, 0};
    const int64_t one[1] = {100};
    CHECK(covap_plan(one, 1, &bad, &p) == COVAP_EINVAL && p == nullptr);
    CHECK(covap_plan(nullptr, 1, &bad, &p) == COVAP_EINVAL);
    int32_t K = 0;
    CHECK(covap_ratio_from_ccr(3.5, &K) == COVAP_OK && K == 4);
    CHECK(covap_ratio_from_times(842.0, 210.0, &K) == COVAP_OK && K == 5);
    CHECK(covap_ratio_from_ccr(-1.0, &K) == COVAP_EINVAL);
    float c = 0.f;
    CHECK(covap_ef_coeff(0.1f, 1000000, 100, 0.1f, &c) == COVAP_OK && c == 1.0f);
    CHECK(covap_ef_coeff(0.1f, 5, 0, 0.1f, &c) == COVAP_EINVAL);
    CHECK(covap_tune_set("compress_unroll", 2) == COVAP_OK && covap_tune_get("compress_unroll") == 2);
    CHECK(covap_tune_set("compress_unroll", 3) == COVAP_EINVAL);
    CHECK(covap_tune_set("compress_unroll", -1) == COVAP_OK && covap_tune_get("compress_unroll") == 1);
    CHECK(covap_tune_set(nullptr, 1) == COVAP_EINVAL && covap_tune_get("nope") == -1);
    CHECK(covap_last_error()[0] != 0);
    std::puts("host sanitize driver: ok");
    return 0;
}
