// gfx950 kernels for chunk compression (quantise + bit-pack) and swap-in
// (gather + unpack + dequantise).  Sec. 3.2 "Compressing chunks", Sec. 4
// (bit-shift packing), Load primitive of Sec. 3.1.
//
// Work unit: one (chunk, slab) pair = chunk_tokens x head_dim contiguous fp16
// on the cache side and one contiguous run of code bytes on the record side.
// One 64-lane wavefront handles one unit; a lane owns "pieces" of 8
// consecutive elements (one 16-byte cache access), so a quantisation group of
// G elements is spread over G/8 neighbouring lanes and its min/max is a short
// DPP butterfly.  Both sides stream: the kernels are HBM-bound, the arithmetic
// is kept to a few VALU operations per element.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kvs {

typedef _Float16 h2_t __attribute__((ext_vector_type(2)));
typedef _Float16 h8_t __attribute__((ext_vector_type(8)));

struct QuantGeom {
    int32_t n_tokens;      // N
    int32_t chunk_tokens;  // T
    int32_t slabs;         // layers * 2 * kv_heads
    int32_t pieces;        // T * D / 8: 16-byte pieces per unit (multiple of 64)
    int32_t row_pieces;    // D / 8
    int32_t lpg_log2;      // log2(G / 8): lanes per quantisation group (3..6)
};

// DPP lane exchange inside a row of 16 lanes.  CTRL: 0xB1 = swap neighbours,
// 0x4E = swap lane pairs, 0x141 = mirror inside 8 lanes, 0x140 = mirror inside 16.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
    return static_cast<uint32_t>(
        __builtin_amdgcn_update_dpp(0, static_cast<int>(v), CTRL, 0xF, 0xF, false));
}

__device__ __forceinline__ h2_t h2_from_u32(uint32_t u) { return __builtin_bit_cast(h2_t, u); }
__device__ __forceinline__ uint32_t u32_from_h2(h2_t h) { return __builtin_bit_cast(uint32_t, h); }

template <int CTRL>
__device__ __forceinline__ h2_t pkmin_dpp(h2_t m) {
    return __builtin_elementwise_min(m, h2_from_u32(dpp_u32<CTRL>(u32_from_h2(m))));
}

// (min, -max) of the 8 halfs of a piece, reduced over the 2^lpg_log2 lanes of
// the quantisation group; every lane of the group ends with the same pair.
__device__ __forceinline__ h2_t group_min_negmax(const h8_t& x, int lpg_log2) {
    h2_t a = {x[0], x[1]}, b = {x[2], x[3]}, c = {x[4], x[5]}, d = {x[6], x[7]};
    h2_t lo = __builtin_elementwise_min(__builtin_elementwise_min(a, b),
                                        __builtin_elementwise_min(c, d));
    h2_t hi = __builtin_elementwise_max(__builtin_elementwise_max(a, b),
                                        __builtin_elementwise_max(c, d));
    _Float16 mn = lo[0] < lo[1] ? lo[0] : lo[1];
    _Float16 mx = hi[0] > hi[1] ? hi[0] : hi[1];
    h2_t m = {mn, static_cast<_Float16>(-mx)};
    m = pkmin_dpp<0xB1>(m);
    m = pkmin_dpp<0x4E>(m);
    m = pkmin_dpp<0x141>(m);
    if (lpg_log2 >= 4) m = pkmin_dpp<0x140>(m);
    if (lpg_log2 >= 5) {
        uint32_t o = static_cast<uint32_t>(__shfl_xor(static_cast<int>(u32_from_h2(m)), 16));
        m = __builtin_elementwise_min(m, h2_from_u32(o));
    }
    if (lpg_log2 >= 6) {
        uint32_t o = static_cast<uint32_t>(__shfl_xor(static_cast<int>(u32_from_h2(m)), 32));
        m = __builtin_elementwise_min(m, h2_from_u32(o));
    }
    return m;
}

// x + 0.0f of the format definition: -0 becomes +0, everything else is kept.
// Done on the bit pattern so that no floating-point simplification can drop it.
__device__ __forceinline__ float positive_zero(float x) {
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    return __builtin_bit_cast(float, (u << 1) ? u : 0u);
}

// Quantise the 8 elements of one piece to BITS-bit codes (as exact small
// floats in r[]).  The contract is code = rint((x - mn) / scale) with a true
// binary32 division.  The fast path multiplies by an approximate reciprocal;
// its result q' differs from the true rounded quotient by less than
// 8 * 2^-24 * q, so rint(q') can only differ when q' lies within that distance
// of a half-integer.  Lanes that see such a value redo the piece with the
// exact division, which keeps every code bit-identical to the definition.
template <int BITS>
__device__ __forceinline__ void quantise_piece(const h8_t& x, float mn, float scale, float r[8]) {
    constexpr float kLevels = static_cast<float>((1 << BITS) - 1);
    // 0.5 - 2^BITS * 2^-20: a half-integer closer than 16 * 2^-24 * q_max is "dangerous"
    constexpr float kSafe = 0.5f - static_cast<float>(1 << BITS) * 9.5367431640625e-07f;
    const float inv = (scale != 0.0f) ? __builtin_amdgcn_rcpf(scale) : 0.0f;
    bool danger = false;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const float d = static_cast<float>(x[k]) - mn;
        const float q = d * inv;
        const float c = __builtin_rintf(q);
        danger |= (__builtin_fabsf(q - c) >= kSafe);
        r[k] = c;
    }
    if (danger) {
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const float d = static_cast<float>(x[k]) - mn;
            float c = __builtin_rintf(d / scale);
            c = __builtin_fminf(__builtin_fmaxf(c, 0.0f), kLevels);
            r[k] = c;
        }
    }
}

// One (chunk, slab) unit -> codes, scale and mn of its record.
template <int BITS>
__device__ __forceinline__ void compress_unit(const uint4* __restrict__ src,
                                              uint8_t* __restrict__ codes,
                                              float* __restrict__ scale_out,
                                              float* __restrict__ mn_out, const QuantGeom& g,
                                              int lane) {
    constexpr float kLevels = static_cast<float>((1 << BITS) - 1);
    const int lpg_mask = (1 << g.lpg_log2) - 1;
    for (int p0 = 0; p0 < g.pieces; p0 += 256) {
        uint4 raw[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (p0 + u * 64 < g.pieces) raw[u] = src[p0 + u * 64 + lane];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (p0 + u * 64 >= g.pieces) break;
            const int p = p0 + u * 64 + lane;
            const h8_t x = __builtin_bit_cast(h8_t, raw[u]);
            const h2_t m = group_min_negmax(x, g.lpg_log2);
            const float mn = positive_zero(static_cast<float>(m[0]));
            const float mx = positive_zero(static_cast<float>(static_cast<_Float16>(-m[1])));
            const float scale = (mx - mn) / kLevels;
            float r[8];
            quantise_piece<BITS>(x, mn, scale, r);
            if constexpr (BITS == 8) {
                uint32_t w0 = 0, w1 = 0;
                w0 = __builtin_amdgcn_cvt_pk_u8_f32(r[0], 0, w0);
                w0 = __builtin_amdgcn_cvt_pk_u8_f32(r[1], 1, w0);
                w0 = __builtin_amdgcn_cvt_pk_u8_f32(r[2], 2, w0);
                w0 = __builtin_amdgcn_cvt_pk_u8_f32(r[3], 3, w0);
                w1 = __builtin_amdgcn_cvt_pk_u8_f32(r[4], 0, w1);
                w1 = __builtin_amdgcn_cvt_pk_u8_f32(r[5], 1, w1);
                w1 = __builtin_amdgcn_cvt_pk_u8_f32(r[6], 2, w1);
                w1 = __builtin_amdgcn_cvt_pk_u8_f32(r[7], 3, w1);
                reinterpret_cast<uint2*>(codes)[p] = make_uint2(w0, w1);
            } else if constexpr (BITS == 4) {
                // four 4-bit codes = 16 bits: exact as a float sum
                const float lo = __builtin_fmaf(r[3], 4096.0f,
                                 __builtin_fmaf(r[2], 256.0f, __builtin_fmaf(r[1], 16.0f, r[0])));
                const float hi = __builtin_fmaf(r[7], 4096.0f,
                                 __builtin_fmaf(r[6], 256.0f, __builtin_fmaf(r[5], 16.0f, r[4])));
                reinterpret_cast<uint32_t*>(codes)[p] =
                    static_cast<uint32_t>(lo) | (static_cast<uint32_t>(hi) << 16);
            } else {
                // eight 2-bit codes = 16 bits
                float acc = r[7];
#pragma unroll
                for (int k = 6; k >= 0; --k) acc = __builtin_fmaf(acc, 4.0f, r[k]);
                reinterpret_cast<uint16_t*>(codes)[p] =
                    static_cast<uint16_t>(static_cast<uint32_t>(acc));
            }
            if ((lane & lpg_mask) == 0) {
                scale_out[p >> g.lpg_log2] = scale;
                mn_out[p >> g.lpg_log2] = mn;
            }
        }
    }
}

__device__ __forceinline__ void copy_unit(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                          int pieces, int lane) {
    for (int p0 = 0; p0 < pieces; p0 += 256) {
        uint4 raw[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (p0 + u * 64 < pieces) raw[u] = src[p0 + u * 64 + lane];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (p0 + u * 64 < pieces) dst[p0 + u * 64 + lane] = raw[u];
    }
}

// Grid: ceil(n_chunks * slabs / 4) blocks of 256 threads.  Units are numbered
// slab-major (consecutive units walk the token axis of one slab) so that the
// cache side is read as one forward stream.
__global__ __launch_bounds__(256) void compress_kernel(const uint4* __restrict__ kv,
                                                       const uint8_t* __restrict__ bits,
                                                       const uint64_t* __restrict__ off,
                                                       uint8_t* __restrict__ packed,
                                                       QuantGeom g, int32_t n_chunks) {
    const int lane = threadIdx.x & 63;
    const int64_t unit = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (unit >= static_cast<int64_t>(n_chunks) * g.slabs) return;
    const int slab = static_cast<int>(unit / n_chunks);
    const int chunk = static_cast<int>(unit - static_cast<int64_t>(slab) * n_chunks);
    const int b = __builtin_amdgcn_readfirstlane(static_cast<int>(bits[chunk]));
    const uint64_t rec = off[chunk];
    const uint4* src = kv + (static_cast<uint64_t>(slab) * g.n_tokens +
                             static_cast<uint64_t>(chunk) * g.chunk_tokens) * g.row_pieces;
    uint8_t* base = packed + rec;
    if (b == 16) {
        copy_unit(src, reinterpret_cast<uint4*>(base) + static_cast<uint64_t>(slab) * g.pieces,
                  g.pieces, lane);
        return;
    }
    const uint64_t code_bytes = static_cast<uint64_t>(g.pieces) * b;      // per unit
    const uint32_t groups = static_cast<uint32_t>(g.pieces) >> g.lpg_log2;  // per unit
    uint8_t* codes = base + slab * code_bytes;
    float* scale = reinterpret_cast<float*>(base + g.slabs * code_bytes) +
                   static_cast<uint64_t>(slab) * groups;
    float* mn = scale + static_cast<uint64_t>(g.slabs) * groups;
    if (b == 8) compress_unit<8>(src, codes, scale, mn, g, lane);
    else if (b == 4) compress_unit<4>(src, codes, scale, mn, g, lane);
    else compress_unit<2>(src, codes, scale, mn, g, lane);
}

// ------------------------------------------------------------------ swap-in

template <int BITS>
__device__ __forceinline__ void swapin_unit(const uint8_t* __restrict__ codes,
                                            const float* __restrict__ scale_in,
                                            const float* __restrict__ mn_in,
                                            uint4* __restrict__ dst, const QuantGeom& g,
                                            int lane) {
    constexpr uint32_t kMask = (1u << BITS) - 1u;
    for (int p0 = 0; p0 < g.pieces; p0 += 64) {
        const int p = p0 + lane;
        uint32_t w0, w1 = 0;
        if constexpr (BITS == 8) {
            const uint2 w = reinterpret_cast<const uint2*>(codes)[p];
            w0 = w.x;
            w1 = w.y;
        } else if constexpr (BITS == 4) {
            w0 = reinterpret_cast<const uint32_t*>(codes)[p];
        } else {
            w0 = reinterpret_cast<const uint16_t*>(codes)[p];
        }
        const float sc = scale_in[p >> g.lpg_log2];
        const float mn = mn_in[p >> g.lpg_log2];
        h8_t out;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            uint32_t c;
            if constexpr (BITS == 8) c = ((k < 4 ? w0 : w1) >> ((k & 3) * 8)) & kMask;
            else c = (w0 >> (k * BITS)) & kMask;
            const float prod = static_cast<float>(c) * sc;   // rounded product, then rounded sum
            out[k] = static_cast<_Float16>(prod + mn);
        }
        dst[p] = __builtin_bit_cast(uint4, out);
    }
}

// One (selected record, slab) unit of the Load primitive.
__device__ __forceinline__ void swapin_dispatch(const uint8_t* __restrict__ base, int b, int slab,
                                                uint4* __restrict__ dst, const QuantGeom& g,
                                                int lane) {
    if (b == 16) {
        copy_unit(reinterpret_cast<const uint4*>(base) + static_cast<uint64_t>(slab) * g.pieces,
                  dst, g.pieces, lane);
        return;
    }
    const uint64_t code_bytes = static_cast<uint64_t>(g.pieces) * b;
    const uint32_t groups = static_cast<uint32_t>(g.pieces) >> g.lpg_log2;
    const uint8_t* codes = base + slab * code_bytes;
    const float* scale = reinterpret_cast<const float*>(base + g.slabs * code_bytes) +
                         static_cast<uint64_t>(slab) * groups;
    const float* mn = scale + static_cast<uint64_t>(g.slabs) * groups;
    if (b == 8) swapin_unit<8>(codes, scale, mn, dst, g, lane);
    else if (b == 4) swapin_unit<4>(codes, scale, mn, dst, g, lane);
    else swapin_unit<2>(codes, scale, mn, dst, g, lane);
}

// Grid: ceil(n_sel * slabs / 4) blocks of 256 threads; units slab-major so the
// cache side is written as forward streams.  Gather lists in device memory.
__global__ __launch_bounds__(256) void swapin_kernel(const uint8_t* __restrict__ packed,
                                                     const uint64_t* __restrict__ src_off,
                                                     const int32_t* __restrict__ dst_tok,
                                                     const uint8_t* __restrict__ sel_bits,
                                                     uint4* __restrict__ kv_out, QuantGeom g,
                                                     int32_t n_sel) {
    const int lane = threadIdx.x & 63;
    const int64_t unit = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (unit >= static_cast<int64_t>(n_sel) * g.slabs) return;
    const int slab = static_cast<int>(unit / n_sel);
    const int j = static_cast<int>(unit - static_cast<int64_t>(slab) * n_sel);
    const int b = __builtin_amdgcn_readfirstlane(static_cast<int>(sel_bits[j]));
    uint4* dst = kv_out + (static_cast<uint64_t>(slab) * g.n_tokens +
                           static_cast<uint64_t>(dst_tok[j])) * g.row_pieces;
    swapin_dispatch(packed + src_off[j], b, slab, dst, g, lane);
}

// Same work for one staged batch of the streaming Load: the (short) gather
// list travels in the kernel arguments, offsets are relative to the staging slot.
constexpr int kBatchMax = 64;
struct SwapinBatch {
    uint64_t src_off[kBatchMax];
    int32_t dst_tok[kBatchMax];
    uint8_t bits[kBatchMax];
    int32_t n;
};

__global__ __launch_bounds__(256) void swapin_batch_kernel(const uint8_t* __restrict__ staged,
                                                           SwapinBatch list,
                                                           uint4* __restrict__ kv_out,
                                                           QuantGeom g) {
    const int lane = threadIdx.x & 63;
    const int64_t unit = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (unit >= static_cast<int64_t>(list.n) * g.slabs) return;
    const int slab = static_cast<int>(unit / list.n);
    const int j = static_cast<int>(unit - static_cast<int64_t>(slab) * list.n);
    const int b = list.bits[j];
    uint4* dst = kv_out + (static_cast<uint64_t>(slab) * g.n_tokens +
                           static_cast<uint64_t>(list.dst_tok[j])) * g.row_pieces;
    swapin_dispatch(staged + list.src_off[j], b, slab, dst, g, lane);
}

}  // namespace kvs
