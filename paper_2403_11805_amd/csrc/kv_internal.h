// Internal helpers shared by the translation units of libkvswitch.
#pragma once

#include <cstdint>

#include "kvswitch.h"

namespace kvs {

// Records code + formatted text as the calling thread's last error; returns code.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

// KV_OK, or KV_EINVAL / KV_ESHAPE with the error text set.
int check_shape(const kv_shape_t* s);

// The fp16 group formats (parameters in fp32 or in binary16).
inline bool is_f16(const kv_shape_t& s) {
    return s.format == KV_FMT_F16_GROUPS || s.format == KV_FMT_F16_GROUPS_H;
}

// The int8 cache formats (channel-wise parameters in fp32 or in binary16).
inline bool is_i8(const kv_shape_t& s) {
    return s.format == KV_FMT_I8_CHANNELS || s.format == KV_FMT_I8_CHANNELS_H;
}

// Widths a chunk may have: {16,8,4,2} for the fp16 format, {8,4,2,1} for the int8 formats.
inline bool valid_bits(const kv_shape_t& s, int b) {
    if (is_i8(s)) return b == 8 || b == 4 || b == 2 || b == 1;
    return b == 16 || b == 8 || b == 4 || b == 2;
}
inline const char* bits_set(const kv_shape_t& s) {
    return is_i8(s) ? "{8,4,2,1}" : "{16,8,4,2}";
}

inline uint64_t slabs_of(const kv_shape_t& s) {
    return static_cast<uint64_t>(s.n_layers) * 2u * static_cast<uint64_t>(s.n_kv_heads);
}

// Bytes of one chunk's record; shape and bits already validated.
inline uint64_t record_bytes(const kv_shape_t& s, int bits) {
    const uint64_t rows = slabs_of(s) * static_cast<uint64_t>(s.chunk_tokens);
    if (is_i8(s)) {
        if (bits == 8) return rows * static_cast<uint64_t>(s.head_dim);
        const uint64_t meta = s.format == KV_FMT_I8_CHANNELS ? 8u : 4u;   // (scale, minimum) per channel
        return rows * static_cast<uint64_t>(s.head_dim) * bits / 8u +
               slabs_of(s) * meta * static_cast<uint64_t>(s.head_dim);
    }
    if (bits == 16) return rows * static_cast<uint64_t>(s.head_dim) * 2u;
    const uint64_t meta = s.format == KV_FMT_F16_GROUPS_H ? 4u : 8u;      // (scale, minimum) per group
    return rows * (static_cast<uint64_t>(s.head_dim) * bits / 8u +
                   meta * static_cast<uint64_t>(s.head_dim / s.group));
}

inline bool aligned(const void* p, uintptr_t a) {
    return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0;
}

}  // namespace kvs
