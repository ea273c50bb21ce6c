// Host-side, GPU-free part of libkvswitch: error text, shape validation,
// record sizes and offsets, rank-based bit-width assignment (Sec. 3.2, Eq. 2)
// and the gather list of the Load primitive (Sec. 3.1).
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <numeric>
#include <vector>

#include "kv_internal.h"

namespace kvs {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

void clear_error() { g_err[0] = '\0'; }

int check_shape(const kv_shape_t* s) {
    if (!s) return fail(KV_EINVAL, "shape is NULL");
    if (s->n_layers <= 0 || s->n_kv_heads <= 0 || s->n_q_heads <= 0 || s->head_dim <= 0 ||
        s->n_tokens <= 0 || s->chunk_tokens <= 0 || s->group <= 0)
        return fail(KV_ESHAPE, "every shape field must be positive");
    if (s->n_tokens % s->chunk_tokens)
        return fail(KV_ESHAPE, "n_tokens %d is not a multiple of chunk_tokens %d", s->n_tokens,
                    s->chunk_tokens);
    if (!is_f16(*s) && !is_i8(*s))
        return fail(KV_ESHAPE, "format %d unknown", s->format);
    if (s->n_q_heads % s->n_kv_heads)
        return fail(KV_ESHAPE, "n_q_heads %d is not a multiple of n_kv_heads %d", s->n_q_heads,
                    s->n_kv_heads);
    if (s->head_dim > 1024 || s->chunk_tokens > 1024)
        return fail(KV_ESHAPE, "head_dim and chunk_tokens must be <= 1024");
    if (slabs_of(*s) * static_cast<uint64_t>(s->n_tokens) > (1ull << 31))
        return fail(KV_ESHAPE, "layers*2*kv_heads*tokens exceeds 2^31");
    if (is_i8(*s)) {
        if (s->head_dim < 64 || (s->head_dim & (s->head_dim - 1)))
            return fail(KV_ESHAPE, "int8 format needs head_dim a power of two in [64,1024], got %d", s->head_dim);
        const int64_t unit = static_cast<int64_t>(s->chunk_tokens) * s->head_dim;
        if (unit != 1024 && unit != 2048 && unit != 4096)
            return fail(KV_ESHAPE, "int8 format needs chunk_tokens*head_dim in {1024,2048,4096}, got %lld",
                        static_cast<long long>(unit));
        return KV_OK;
    }
    if (s->group != 64 && s->group != 128 && s->group != 256 && s->group != 512)
        return fail(KV_ESHAPE, "group %d not in {64,128,256,512}", s->group);
    if (s->head_dim % s->group)
        return fail(KV_ESHAPE, "head_dim %d is not a multiple of group %d", s->head_dim, s->group);
    if ((static_cast<int64_t>(s->chunk_tokens) * s->head_dim) % 512)
        return fail(KV_ESHAPE, "chunk_tokens*head_dim must be a multiple of 512");
    if ((s->chunk_tokens * s->head_dim / s->group) % 4)
        return fail(KV_ESHAPE, "chunk_tokens*head_dim/group must be a multiple of 4");
    return KV_OK;
}

}  // namespace kvs

using namespace kvs;

extern "C" {

const char* kv_last_error(void) { return g_err; }

uint64_t kv_record_bytes(const kv_shape_t* shape, int32_t bits) {
    if (check_shape(shape) != KV_OK) return 0;
    if (!valid_bits(*shape, bits)) {
        fail(KV_EBITS, "bits %d not in %s", bits, bits_set(*shape));
        return 0;
    }
    return record_bytes(*shape, bits);
}

int32_t kv_chunk_offsets(const kv_shape_t* shape, const uint8_t* bits, uint64_t* off) {
    if (int rc = check_shape(shape)) return rc;
    if (!bits || !off) return fail(KV_EINVAL, "bits/off is NULL");
    const int32_t n = shape->n_tokens / shape->chunk_tokens;
    for (int32_t i = 0; i < n; ++i)
        if (!valid_bits(*shape, bits[i]))
            return fail(KV_EBITS, "bits[%d] = %d not in %s", i, bits[i], bits_set(*shape));
    uint64_t acc = 0;
    for (int32_t i = 0; i < n; ++i) {
        off[i] = acc;
        acc += record_bytes(*shape, bits[i]);
    }
    off[n] = acc;
    return KV_OK;
}

// A NaN would make "denser than" no ordering at all (and the device planner, which counts ranks,
// would disagree with any sort): refused.
static int check_finite(const float* density, int32_t n) {
    for (int32_t i = 0; i < n; ++i)
        if (!std::isfinite(density[i])) return fail(KV_EINVAL, "density[%d] is not finite", i);
    return KV_OK;
}

int32_t kv_bits_from_scores(const float* density, int32_t n, int32_t num8, int32_t num4,
                            int32_t den, uint8_t* bits) {
    if (!density || !bits) return fail(KV_EINVAL, "density/bits is NULL");
    if (n < 0 || den <= 0 || num8 < 0 || num4 < 0 || num8 + num4 > den)
        return fail(KV_EINVAL, "need n >= 0, den > 0, 0 <= num8, 0 <= num4, num8+num4 <= den");
    if (int rc = check_finite(density, n)) return rc;
    std::vector<int32_t> order(static_cast<size_t>(n));
    std::iota(order.begin(), order.end(), 0);
    // densest first; equal densities keep index order
    std::stable_sort(order.begin(), order.end(),
                     [&](int32_t a, int32_t b) { return density[a] > density[b]; });
    const int64_t k8 = static_cast<int64_t>(n) * num8 / den;
    const int64_t k84 = static_cast<int64_t>(n) * (num8 + num4) / den;
    for (int64_t r = 0; r < n; ++r) bits[order[static_cast<size_t>(r)]] = r < k8 ? 8 : (r < k84 ? 4 : 2);
    return KV_OK;
}

int32_t kv_bits_optimise(const float* density, int32_t n, int32_t ratio_num, int32_t ratio_den,
                         int32_t objective, uint8_t* bits, int32_t* counts) {
    if (n < 0 || ratio_den <= 0 || ratio_num <= 0) return fail(KV_EINVAL, "need n >= 0 and a positive ratio");
    if (static_cast<int64_t>(ratio_num) * 4 < ratio_den || ratio_num > ratio_den)
        return fail(KV_EINVAL, "ratio %d/%d outside [1/4, 1]", ratio_num, ratio_den);
    if (objective != KV_OBJ_BITS_TO_DENSE && objective != KV_OBJ_AS_PRINTED)
        return fail(KV_EINVAL, "objective %d unknown", objective);
    if (n > 0 && (!density || !bits)) return fail(KV_EINVAL, "density/bits is NULL");
    if (int rc = check_finite(density, n)) return rc;
    std::vector<int32_t> order(static_cast<size_t>(n));
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(),
                     [&](int32_t a, int32_t b) { return density[a] > density[b]; });
    // prefix[k] = sum of the k densest, accumulated in rank order
    std::vector<double> prefix(static_cast<size_t>(n) + 1, 0.0);
    for (int32_t k = 0; k < n; ++k)
        prefix[static_cast<size_t>(k) + 1] = prefix[static_cast<size_t>(k)] +
                                             static_cast<double>(density[order[static_cast<size_t>(k)]]);
    const double w8 = 1.0;
    const double w4 = objective == KV_OBJ_BITS_TO_DENSE ? 0.5 : 2.0;
    const double w2 = objective == KV_OBJ_BITS_TO_DENSE ? 0.25 : 4.0;
    int64_t M = static_cast<int64_t>(n) * (4LL * ratio_num - ratio_den) / ratio_den;
    // 3*k8 + k4 = 3n - 1 is the one total that no split of n chunks reaches (it needs k4 = 2 with
    // a single chunk left): the largest reachable average below the target is then 3n - 2
    if (n > 0 && M == 3LL * n - 1) --M;
    const int64_t k8_lo = std::max<int64_t>(0, (M - n + 1) / 2);   // k2 = n - M + 2*k8 >= 0
    const int64_t k8_hi = M / 3;                                   // k4 = M - 3*k8 >= 0
    int64_t best_k8 = k8_lo;
    double best = 0.0;
    for (int64_t k8 = k8_lo; k8 <= k8_hi; ++k8) {
        const int64_t k4 = M - 3 * k8;
        const double s8 = prefix[static_cast<size_t>(k8)];
        const double s4 = prefix[static_cast<size_t>(k8 + k4)] - prefix[static_cast<size_t>(k8)];
        const double s2 = prefix[static_cast<size_t>(n)] - prefix[static_cast<size_t>(k8 + k4)];
        const double info = w8 * s8 + w4 * s4 + w2 * s2;
        if (k8 == k8_lo || info > best) {
            best = info;
            best_k8 = k8;
        }
    }
    const int64_t k4 = M - 3 * best_k8;
    for (int64_t r = 0; r < n; ++r)
        bits[order[static_cast<size_t>(r)]] = r < best_k8 ? 8 : (r < best_k8 + k4 ? 4 : 2);
    if (counts) {
        counts[0] = static_cast<int32_t>(best_k8);
        counts[1] = static_cast<int32_t>(k4);
        counts[2] = static_cast<int32_t>(n - best_k8 - k4);
    }
    return KV_OK;
}

int32_t kv_fit_line(const double* x, const double* t, int32_t n, double* slope, double* intercept) {
    if (!x || !t || !slope || !intercept) return fail(KV_EINVAL, "NULL pointer");
    if (n < 2) return fail(KV_EINVAL, "need at least two points");
    double sx = 0.0, st = 0.0;
    for (int32_t i = 0; i < n; ++i) {
        sx += x[i];
        st += t[i];
    }
    const double mx = sx / n, mt = st / n;
    double sxx = 0.0, sxt = 0.0;
    for (int32_t i = 0; i < n; ++i) {
        sxx += (x[i] - mx) * (x[i] - mx);
        sxt += (x[i] - mx) * (t[i] - mt);
    }
    if (!(sxx > 0.0)) return fail(KV_EINVAL, "all x are equal");
    *slope = sxt / sxx;
    *intercept = mt - *slope * mx;
    return KV_OK;
}

int32_t kv_plan_pipeline(const kv_pipeline_model_t* model, const int32_t* missing,
                         const uint64_t* rec_bytes, int32_t* recompute, double* delay) {
    if (!model || !missing || !rec_bytes || !recompute) return fail(KV_EINVAL, "NULL pointer");
    if (!(model->re_per_chunk >= 0.0) || !(model->re_fixed >= 0.0) || !(model->io_per_byte >= 0.0) ||
        !(model->io_fixed >= 0.0))
        return fail(KV_EINVAL, "model coefficients must be non-negative");
    if (missing[0] < 0 || missing[1] < 0 || missing[2] < 0) return fail(KV_EINVAL, "negative chunk count");
    if (!(rec_bytes[0] > rec_bytes[1] && rec_bytes[1] > rec_bytes[2] && rec_bytes[2] > 0))
        return fail(KV_EINVAL, "record sizes must be positive and strictly decreasing (8, 4, 2 bits)");
    const int64_t total = static_cast<int64_t>(missing[0]) + missing[1] + missing[2];
    const double all_bytes = static_cast<double>(missing[0]) * static_cast<double>(rec_bytes[0]) +
                             static_cast<double>(missing[1]) * static_cast<double>(rec_bytes[1]) +
                             static_cast<double>(missing[2]) * static_cast<double>(rec_bytes[2]);
    double best = 0.0;
    int64_t best_x = 0;
    for (int64_t x = 0; x <= total; ++x) {
        // heaviest records leave the IO first
        const int64_t r8 = std::min<int64_t>(x, missing[0]);
        const int64_t r4 = std::min<int64_t>(x - r8, missing[1]);
        const int64_t r2 = x - r8 - r4;
        const double removed = static_cast<double>(r8) * static_cast<double>(rec_bytes[0]) +
                               static_cast<double>(r4) * static_cast<double>(rec_bytes[1]) +
                               static_cast<double>(r2) * static_cast<double>(rec_bytes[2]);
        const double io_b = all_bytes - removed;
        const double t_re = x > 0 ? model->re_per_chunk * static_cast<double>(x) + model->re_fixed : 0.0;
        const double t_io = (x < total) ? model->io_per_byte * io_b + model->io_fixed : 0.0;
        const double d = std::max(t_re, t_io);
        if (x == 0 || d < best) {
            best = d;
            best_x = x;
        }
    }
    const int64_t r8 = std::min<int64_t>(best_x, missing[0]);
    const int64_t r4 = std::min<int64_t>(best_x - r8, missing[1]);
    recompute[0] = static_cast<int32_t>(r8);
    recompute[1] = static_cast<int32_t>(r4);
    recompute[2] = static_cast<int32_t>(best_x - r8 - r4);
    if (delay) *delay = best;
    return KV_OK;
}

int32_t kv_pipeline_split(const kv_shape_t* shape, const uint8_t* bits, const int32_t* missing_idx,
                          int32_t n_missing, const int32_t* recompute, int32_t* recompute_idx,
                          int32_t* n_recompute, int32_t* load_idx, int32_t* n_load) {
    if (int rc = check_shape(shape)) return rc;
    if (n_missing < 0) return fail(KV_EINVAL, "n_missing %d < 0", n_missing);
    if (!recompute || !n_recompute || !n_load) return fail(KV_EINVAL, "NULL pointer");
    if (n_missing > 0 && (!bits || !missing_idx || !recompute_idx || !load_idx)) return fail(KV_EINVAL, "NULL list pointer");
    if (recompute[0] < 0 || recompute[1] < 0 || recompute[2] < 0) return fail(KV_EINVAL, "negative chunk count");
    const int32_t n = shape->n_tokens / shape->chunk_tokens;
    int64_t have[3] = {0, 0, 0};
    for (int32_t j = 0; j < n_missing; ++j) {
        const int32_t i = missing_idx[j];
        if (i < 0 || i >= n) return fail(KV_EINDEX, "missing_idx[%d] = %d outside [0,%d)", j, i, n);
        if (j && i <= missing_idx[j - 1]) return fail(KV_EINDEX, "missing_idx not strictly ascending at position %d", j);
        if (!valid_bits(*shape, bits[i])) return fail(KV_EBITS, "bits[%d] = %d not in %s", i, bits[i], bits_set(*shape));
        if (bits[i] == 8) ++have[0];
        else if (bits[i] == 4) ++have[1];
        else if (bits[i] == 2) ++have[2];
    }
    for (int w = 0; w < 3; ++w)
        if (recompute[w] > have[w])
            return fail(KV_EINVAL, "plan recomputes %d chunks of %d bits, %lld are missing", recompute[w], 8 >> w,
                        static_cast<long long>(have[w]));
    int32_t left[3] = {recompute[0], recompute[1], recompute[2]};
    int32_t n_re = 0, n_io = 0;
    for (int32_t j = 0; j < n_missing; ++j) {
        const int32_t i = missing_idx[j];
        const int w = bits[i] == 8 ? 0 : (bits[i] == 4 ? 1 : (bits[i] == 2 ? 2 : -1));
        if (w >= 0 && left[w] > 0) {
            --left[w];
            recompute_idx[n_re++] = i;
        } else {
            load_idx[n_io++] = i;
        }
    }
    *n_recompute = n_re;
    *n_load = n_io;
    return KV_OK;
}

int32_t kv_build_gather(const kv_shape_t* shape, const uint64_t* off, const uint8_t* bits,
                        const int32_t* chunk_idx, int32_t n_sel, uint64_t* src_off,
                        int32_t* dst_tok, uint8_t* sel_bits) {
    if (int rc = check_shape(shape)) return rc;
    if (n_sel < 0) return fail(KV_EINVAL, "n_sel %d < 0", n_sel);
    if (n_sel == 0) return KV_OK;
    if (!off || !bits || !chunk_idx || !src_off || !dst_tok || !sel_bits)
        return fail(KV_EINVAL, "NULL list pointer");
    const int32_t n = shape->n_tokens / shape->chunk_tokens;
    for (int32_t j = 0; j < n_sel; ++j) {
        const int32_t i = chunk_idx[j];
        if (i < 0 || i >= n) return fail(KV_EINDEX, "chunk_idx[%d] = %d outside [0,%d)", j, i, n);
        if (j && i <= chunk_idx[j - 1])
            return fail(KV_EINDEX, "chunk_idx not strictly ascending at position %d", j);
        if (!valid_bits(*shape, bits[i]))
            return fail(KV_EBITS, "bits[%d] = %d not in %s", i, bits[i], bits_set(*shape));
    }
    for (int32_t j = 0; j < n_sel; ++j) {
        const int32_t i = chunk_idx[j];
        src_off[j] = off[i];
        dst_tok[j] = i * shape->chunk_tokens;
        sel_bits[j] = bits[i];
    }
    return KV_OK;
}

}  // extern "C"
