// Drives the host half of libkvswitch from several threads at once under ThreadSanitizer: the pure
// host functions keep no state between calls (the error text is per thread), and each thread may
// own a queue of its own.  Built and run by tests/test_host_sanitizers.py; exits 0 when every
// expectation holds and no data race is reported.
#include <atomic>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <thread>
#include <vector>

#include "kvswitch.h"

static std::atomic<int> failures{0};

#define EXPECT(cond)                                                                      \
    do {                                                                                  \
        if (!(cond)) {                                                                    \
            std::printf("thread %d line %d: %s  [%s]\n", id, __LINE__, #cond, kv_last_error()); \
            failures.fetch_add(1);                                                        \
            return;                                                                       \
        }                                                                                 \
    } while (0)

static void worker(int id) {
    uint64_t st = 0x9E3779B97F4A7C15ull * static_cast<uint64_t>(id + 1);
    auto rnd = [&](uint32_t n) {
        st ^= st << 13; st ^= st >> 7; st ^= st << 17;
        return static_cast<uint32_t>(st >> 11) % n;
    };
    kv_shape_t s = {4, 2, 2, 128, 2048, 16, 64, id % 2 ? KV_FMT_F16_GROUPS_H : KV_FMT_F16_GROUPS};
    const int n = s.n_tokens / s.chunk_tokens;
    kv_lctru_t* q = kv_lctru_create();
    EXPECT(q != nullptr);
    for (int round = 0; round < 200; ++round) {
        std::vector<float> dens(n);
        for (auto& d : dens) d = static_cast<float>(rnd(40)) / 40.0f;
        std::vector<uint8_t> bits(n);
        EXPECT(kv_bits_from_scores(dens.data(), n, 1, 1, 3, bits.data()) == KV_OK);
        std::vector<uint64_t> off(n + 1);
        EXPECT(kv_chunk_offsets(&s, bits.data(), off.data()) == KV_OK);
        uint64_t sum = 0;
        for (int i = 0; i < n; ++i) sum += kv_record_bytes(&s, bits[i]);
        EXPECT(off[n] == sum);
        int32_t idx[3] = {static_cast<int32_t>(rnd(40)), static_cast<int32_t>(40 + rnd(40)), static_cast<int32_t>(80 + rnd(40))};
        uint64_t src[3]; int32_t dst[3]; uint8_t sb[3];
        EXPECT(kv_build_gather(&s, off.data(), bits.data(), idx, 3, src, dst, sb) == KV_OK);
        EXPECT(src[1] == off[idx[1]] && dst[2] == idx[2] * s.chunk_tokens && sb[0] == bits[idx[0]]);
        // a refused call leaves its text with this thread only
        int32_t unsorted[2] = {5, 5};
        EXPECT(kv_build_gather(&s, off.data(), bits.data(), unsorted, 2, src, dst, sb) == KV_EINDEX);
        EXPECT(std::strlen(kv_last_error()) > 0);
        // a queue of this thread's own
        for (int c = 0; c < 8; ++c)
            EXPECT(kv_lctru_insert(q, id, round * 8 + c, bits[c], kv_record_bytes(&s, bits[c]), round) == KV_OK);
        int32_t ctx[16], chunk[16], n_out = 0;
        EXPECT(kv_lctru_evict(q, kv_record_bytes(&s, 2) * 4, ctx, chunk, 16, &n_out) == KV_OK);
        EXPECT(n_out >= 1 && ctx[0] == id);
    }
    kv_lctru_destroy(q);
}

int main() {
    std::vector<std::thread> pool;
    for (int id = 0; id < 6; ++id) pool.emplace_back(worker, id);
    for (auto& t : pool) t.join();
    if (failures.load()) return 1;
    std::printf("host threads drive ok\n");
    return 0;
}
