// LCTRU eviction queue and working-set lock (Sec. 3.4 ii): host bookkeeping
// only; it decides which resident chunks Reclaim hands out, it moves no data.
//
// One ordered set keyed by (more bits first, older last-access first, ctx,
// chunk) realises the concatenation of per-bit-width sub-queues, each in
// least-recently-used order.
#include <cstddef>
#include <map>
#include <new>
#include <set>
#include <tuple>
#include <unordered_set>
#include <vector>

#include "kv_internal.h"

using namespace kvs;

namespace {

struct Entry {
    int32_t bits;
    uint64_t bytes;
    uint64_t last;
};

// (-bits, last_access, ctx, chunk): ascending order == eviction order
using Key = std::tuple<int32_t, uint64_t, int32_t, int32_t>;

}  // namespace

struct kv_lctru {
    std::set<Key> queue;
    std::map<std::pair<int32_t, int32_t>, Entry> entries;   // (ctx, chunk) -> entry
    std::unordered_set<int32_t> locked;
    uint64_t total_bytes = 0;

    static Key key_of(int32_t ctx, int32_t chunk, const Entry& e) {
        return Key(-e.bits, e.last, ctx, chunk);
    }
};

extern "C" {

kv_lctru_t* kv_lctru_create(void) { return new (std::nothrow) kv_lctru(); }

void kv_lctru_destroy(kv_lctru_t* q) { delete q; }

int32_t kv_lctru_insert(kv_lctru_t* q, int32_t ctx, int32_t chunk, int32_t bits, uint64_t bytes,
                        uint64_t now) {
    if (!q) return fail(KV_EINVAL, "queue is NULL");
    if (ctx < 0 || chunk < 0) return fail(KV_EINVAL, "negative ctx/chunk id");
    if (bits != 16 && bits != 8 && bits != 4 && bits != 2 && bits != 1)
        return fail(KV_EBITS, "bits %d not in {16,8,4,2,1}", bits);
    try {
        const auto id = std::make_pair(ctx, chunk);
        if (q->entries.count(id)) return fail(KV_EINVAL, "(ctx %d, chunk %d) already resident", ctx, chunk);
        Entry e{bits, bytes, now};
        q->entries.emplace(id, e);
        q->queue.insert(kv_lctru::key_of(ctx, chunk, e));
        q->total_bytes += bytes;
    } catch (...) {
        return fail(KV_ENOMEM, "out of host memory");
    }
    return KV_OK;
}

int32_t kv_lctru_touch_ctx(kv_lctru_t* q, int32_t ctx, uint64_t now) {
    if (!q) return fail(KV_EINVAL, "queue is NULL");
    try {
        auto it = q->entries.lower_bound(std::make_pair(ctx, INT32_MIN));
        for (; it != q->entries.end() && it->first.first == ctx; ++it) {
            q->queue.erase(kv_lctru::key_of(ctx, it->first.second, it->second));
            it->second.last = now;
            q->queue.insert(kv_lctru::key_of(ctx, it->first.second, it->second));
        }
    } catch (...) {
        return fail(KV_ENOMEM, "out of host memory");
    }
    return KV_OK;
}

int32_t kv_lctru_lock(kv_lctru_t* q, int32_t ctx) {
    if (!q) return fail(KV_EINVAL, "queue is NULL");
    try {
        q->locked.insert(ctx);
    } catch (...) {
        return fail(KV_ENOMEM, "out of host memory");
    }
    return KV_OK;
}

int32_t kv_lctru_unlock(kv_lctru_t* q, int32_t ctx) {
    if (!q) return fail(KV_EINVAL, "queue is NULL");
    q->locked.erase(ctx);
    return KV_OK;
}

int32_t kv_lctru_evict(kv_lctru_t* q, uint64_t bytes_needed, int32_t* out_ctx, int32_t* out_chunk,
                       int32_t cap, int32_t* n_out) {
    if (!q || !n_out) return fail(KV_EINVAL, "queue/n_out is NULL");
    if (cap < 0 || (cap > 0 && (!out_ctx || !out_chunk))) return fail(KV_EINVAL, "bad output arrays");
    *n_out = 0;
    std::vector<std::set<Key>::iterator> picked;
    uint64_t got = 0;
    try {
        for (auto it = q->queue.begin(); it != q->queue.end() && got < bytes_needed; ++it) {
            const int32_t ctx = std::get<2>(*it);
            if (q->locked.count(ctx)) continue;
            picked.push_back(it);
            got += q->entries.at(std::make_pair(ctx, std::get<3>(*it))).bytes;
        }
    } catch (...) {
        return fail(KV_ENOMEM, "out of host memory");
    }
    if (got < bytes_needed)
        return fail(KV_ENOMEM, "only %llu evictable bytes, %llu needed",
                    static_cast<unsigned long long>(got), static_cast<unsigned long long>(bytes_needed));
    if (picked.size() > static_cast<size_t>(cap))
        return fail(KV_ENOMEM, "%zu entries needed, output capacity %d", picked.size(), cap);
    int32_t n = 0;
    for (auto it : picked) {
        const int32_t ctx = std::get<2>(*it), chunk = std::get<3>(*it);
        out_ctx[n] = ctx;
        out_chunk[n] = chunk;
        ++n;
        auto e = q->entries.find(std::make_pair(ctx, chunk));
        q->total_bytes -= e->second.bytes;
        q->entries.erase(e);
        q->queue.erase(it);
    }
    *n_out = n;
    return KV_OK;
}

int32_t kv_lctru_order(const kv_lctru_t* q, int32_t* out_ctx, int32_t* out_chunk, int32_t cap,
                       int32_t* n_out) {
    if (!q || !n_out) return fail(KV_EINVAL, "queue/n_out is NULL");
    if (cap < 0 || (cap > 0 && (!out_ctx || !out_chunk))) return fail(KV_EINVAL, "bad output arrays");
    int32_t n = 0;
    for (const Key& k : q->queue) {
        if (q->locked.count(std::get<2>(k))) continue;
        if (n >= cap) {
            *n_out = 0;
            return fail(KV_ENOMEM, "more than %d unlocked entries", cap);
        }
        out_ctx[n] = std::get<2>(k);
        out_chunk[n] = std::get<3>(k);
        ++n;
    }
    *n_out = n;
    return KV_OK;
}

int32_t kv_lctru_remove_ctx(kv_lctru_t* q, int32_t ctx) {
    if (!q) return fail(KV_EINVAL, "queue is NULL");
    auto it = q->entries.lower_bound(std::make_pair(ctx, INT32_MIN));
    while (it != q->entries.end() && it->first.first == ctx) {
        q->queue.erase(kv_lctru::key_of(ctx, it->first.second, it->second));
        q->total_bytes -= it->second.bytes;
        it = q->entries.erase(it);
    }
    q->locked.erase(ctx);
    return KV_OK;
}

int32_t kv_lctru_size(const kv_lctru_t* q, int32_t* n_entries, uint64_t* bytes) {
    if (!q) return fail(KV_EINVAL, "queue is NULL");
    if (n_entries) *n_entries = static_cast<int32_t>(q->entries.size());
    if (bytes) *bytes = q->total_bytes;
    return KV_OK;
}

}  // extern "C"
