// Drives the host half of libkvswitch (kv_host.cpp, kv_lctru.cpp) under AddressSanitizer and
// UndefinedBehaviorSanitizer: valid calls, refused calls and a long random LCTRU sequence.
// Built and run by tests/test_host_sanitizers.py; exits 0 when every expectation holds.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cmath>
#include <vector>

#include "kvswitch.h"

#define EXPECT(cond)                                                        \
    do {                                                                    \
        if (!(cond)) {                                                      \
            std::printf("line %d: %s  [%s]\n", __LINE__, #cond, kv_last_error()); \
            return 1;                                                       \
        }                                                                   \
    } while (0)

static uint64_t rng_state = 88172645463325252ull;
static uint32_t rnd(uint32_t n) {
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return static_cast<uint32_t>(rng_state >> 11) % n;
}

int main() {
    kv_shape_t s = {32, 32, 32, 128, 4096, 16, 64, KV_FMT_F16_GROUPS};
    const int n = s.n_tokens / s.chunk_tokens;
    EXPECT(kv_record_bytes(&s, 8) == 4718592u);
    EXPECT(kv_record_bytes(&s, 3) == 0u);
    kv_shape_t bad = s;
    bad.n_tokens = 4001;
    EXPECT(kv_record_bytes(&bad, 8) == 0u);
    kv_shape_t i8 = s;
    i8.format = KV_FMT_I8_CHANNELS;
    EXPECT(kv_record_bytes(&i8, 1) == 2048u * (256 + 1024));

    std::vector<float> dens(n);
    for (auto& d : dens) d = static_cast<float>(rnd(50)) / 50.0f;       // many ties
    std::vector<uint8_t> bits(n);
    EXPECT(kv_bits_from_scores(dens.data(), n, 1, 1, 3, bits.data()) == KV_OK);
    EXPECT(kv_bits_from_scores(dens.data(), n, 2, 2, 3, bits.data()) == KV_EINVAL);
    int32_t counts[3];
    EXPECT(kv_bits_optimise(dens.data(), n, 1, 2, KV_OBJ_BITS_TO_DENSE, bits.data(), counts) == KV_OK);
    EXPECT(counts[0] + counts[1] + counts[2] == n);
    EXPECT(kv_bits_optimise(dens.data(), n, 1, 2, KV_OBJ_AS_PRINTED, bits.data(), nullptr) == KV_OK);
    EXPECT(kv_bits_optimise(dens.data(), n, 1, 8, KV_OBJ_BITS_TO_DENSE, bits.data(), counts) == KV_EINVAL);
    EXPECT(kv_bits_optimise(dens.data(), 0, 1, 2, KV_OBJ_BITS_TO_DENSE, bits.data(), counts) == KV_OK);

    std::vector<uint64_t> off(n + 1);
    EXPECT(kv_chunk_offsets(&s, bits.data(), off.data()) == KV_OK);
    EXPECT(off[0] == 0 && off[n] > 0);
    bits[5] = 7;
    EXPECT(kv_chunk_offsets(&s, bits.data(), off.data()) == KV_EBITS);
    bits[5] = 4;
    EXPECT(kv_chunk_offsets(&s, bits.data(), off.data()) == KV_OK);

    std::vector<int32_t> idx;
    for (int i = 0; i < n; i += 3) idx.push_back(i);
    std::vector<uint64_t> src(idx.size());
    std::vector<int32_t> dst(idx.size());
    std::vector<uint8_t> sb(idx.size());
    EXPECT(kv_build_gather(&s, off.data(), bits.data(), idx.data(), static_cast<int32_t>(idx.size()), src.data(),
                           dst.data(), sb.data()) == KV_OK);
    EXPECT(dst[1] == 3 * s.chunk_tokens && src[1] == off[3]);
    idx[2] = idx[1];
    EXPECT(kv_build_gather(&s, off.data(), bits.data(), idx.data(), static_cast<int32_t>(idx.size()), src.data(),
                           dst.data(), sb.data()) == KV_EINDEX);
    idx[2] = n;
    EXPECT(kv_build_gather(&s, off.data(), bits.data(), idx.data(), 3, src.data(), dst.data(), sb.data()) == KV_EINDEX);
    EXPECT(kv_build_gather(&s, off.data(), bits.data(), idx.data(), 0, src.data(), dst.data(), sb.data()) == KV_OK);

    const double xs[4] = {1, 2, 3, 4}, ts[4] = {3, 5, 7, 9};
    double a = 0, b = 0;
    EXPECT(kv_fit_line(xs, ts, 4, &a, &b) == KV_OK && a > 1.999 && a < 2.001 && b > 0.999 && b < 1.001);
    EXPECT(kv_fit_line(xs, ts, 1, &a, &b) == KV_EINVAL);
    const double same[2] = {2, 2};
    EXPECT(kv_fit_line(same, ts, 2, &a, &b) == KV_EINVAL);
    kv_pipeline_model_t m = {1e-4, 0.0, 1e-10, 1e-5};
    const int32_t missing[3] = {85, 85, 86};
    const uint64_t rec[3] = {4718592, 2621440, 1572864};
    int32_t re[3];
    double delay = -1;
    EXPECT(kv_plan_pipeline(&m, missing, rec, re, &delay) == KV_OK && delay > 0);
    EXPECT(re[0] >= 0 && re[0] <= 85 && re[1] >= 0 && re[2] >= 0);
    const uint64_t rec_bad[3] = {10, 20, 30};
    EXPECT(kv_plan_pipeline(&m, missing, rec_bad, re, &delay) == KV_EINVAL);
    // the split of a plan: counts per width add up, lists ascending, a plan that asks for too much is refused
    {
        EXPECT(kv_bits_from_scores(dens.data(), n, 1, 1, 3, bits.data()) == KV_OK);
        std::vector<int32_t> miss;
        for (int i = 1; i < n; i += 2) miss.push_back(i);
        int32_t have[3] = {0, 0, 0};
        for (int32_t i : miss) ++have[bits[i] == 8 ? 0 : bits[i] == 4 ? 1 : 2];
        const int32_t want[3] = {have[0] / 2, have[1], 0};
        std::vector<int32_t> ri(miss.size()), li(miss.size());
        int32_t nr = -1, nl = -1;
        EXPECT(kv_pipeline_split(&s, bits.data(), miss.data(), static_cast<int32_t>(miss.size()), want, ri.data(), &nr,
                                 li.data(), &nl) == KV_OK);
        EXPECT(nr == want[0] + want[1] && nr + nl == static_cast<int32_t>(miss.size()));
        for (int32_t k = 1; k < nr; ++k) EXPECT(ri[k] > ri[k - 1]);
        for (int32_t k = 1; k < nl; ++k) EXPECT(li[k] > li[k - 1]);
        const int32_t too_many[3] = {have[0] + 1, 0, 0};
        EXPECT(kv_pipeline_split(&s, bits.data(), miss.data(), static_cast<int32_t>(miss.size()), too_many, ri.data(), &nr,
                                 li.data(), &nl) == KV_EINVAL);
        miss[1] = miss[0];
        EXPECT(kv_pipeline_split(&s, bits.data(), miss.data(), static_cast<int32_t>(miss.size()), want, ri.data(), &nr,
                                 li.data(), &nl) == KV_EINDEX);
        EXPECT(kv_pipeline_split(&s, bits.data(), miss.data(), 0, too_many, ri.data(), &nr, li.data(), &nl) == KV_EINVAL ||
               (nr == 0 && nl == 0));
    }
    // densities that are not finite are refused before any sort sees them
    {
        std::vector<float> d2(dens);
        d2[3] = std::nanf("");
        EXPECT(kv_bits_from_scores(d2.data(), n, 1, 1, 3, bits.data()) == KV_EINVAL);
        EXPECT(kv_bits_optimise(d2.data(), n, 1, 2, KV_OBJ_BITS_TO_DENSE, bits.data(), counts) == KV_EINVAL);
        EXPECT(kv_bits_from_scores(dens.data(), n, 1, 1, 3, bits.data()) == KV_OK);
        EXPECT(kv_bits_optimise(dens.data(), n, 99, 100, KV_OBJ_BITS_TO_DENSE, bits.data(), counts) == KV_OK);
        EXPECT(counts[0] >= 0 && counts[1] >= 0 && counts[2] >= 0 && counts[0] + counts[1] + counts[2] == n);
    }

    // LCTRU: a long random sequence; sizes stay consistent, locked contexts are never evicted
    kv_lctru_t* q = kv_lctru_create();
    EXPECT(q != nullptr);
    std::vector<int32_t> oc(5000), ok(5000);
    const int width[4] = {16, 8, 4, 2};
    for (int step = 0; step < 20000; ++step) {
        const int ctx = static_cast<int>(rnd(12)), chunk = static_cast<int>(rnd(40));
        switch (rnd(8)) {
            case 0: case 1: case 2:
                kv_lctru_insert(q, ctx, chunk, width[rnd(4)], 1000 + rnd(5000), static_cast<uint64_t>(step));
                break;
            case 3: kv_lctru_touch_ctx(q, ctx, static_cast<uint64_t>(step)); break;
            case 4: kv_lctru_lock(q, ctx); break;
            case 5: kv_lctru_unlock(q, ctx); break;
            case 6: {
                int32_t got = 0;
                const int rc = kv_lctru_evict(q, rnd(20000), oc.data(), ok.data(), static_cast<int32_t>(oc.size()), &got);
                EXPECT(rc == KV_OK || rc == KV_ENOMEM);
                break;
            }
            default: if (rnd(10) == 0) kv_lctru_remove_ctx(q, ctx); break;
        }
        if (step % 997 == 0) {
            int32_t entries = 0, listed = 0;
            uint64_t bytes = 0;
            EXPECT(kv_lctru_size(q, &entries, &bytes) == KV_OK);
            EXPECT(kv_lctru_order(q, oc.data(), ok.data(), static_cast<int32_t>(oc.size()), &listed) == KV_OK);
            EXPECT(listed <= entries);
        }
    }
    EXPECT(kv_lctru_insert(q, 1, 1, 5, 10, 0) == KV_EBITS);
    EXPECT(kv_lctru_insert(nullptr, 1, 1, 8, 10, 0) == KV_EINVAL);
    kv_lctru_destroy(q);
    kv_lctru_destroy(nullptr);
    std::printf("host sanitizer drive ok\n");
    return 0;
}
