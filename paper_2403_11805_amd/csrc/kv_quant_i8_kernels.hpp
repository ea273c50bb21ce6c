// gfx950 kernels for the int8, channel-wise record format: the paper's own
// quantiser setting (Sec. 3.2 "Compressing chunks", Sec. 4): the cache is held
// as 8-bit integers and a chunk is quantised further to 4, 2 or 1 bits with one
// (scale, minimum) pair per head_dim channel of a slab, taken over the slab's
// chunk_tokens tokens.
//
// One wavefront holds one (chunk, slab) unit of chunk_tokens x head_dim bytes
// (1, 2 or 4 KiB) in registers: a lane owns PPL pieces of 16 consecutive bytes,
// piece u * 64 + lane, so all of a lane's pieces carry the same 16 channels
// (64 is a multiple of the head_dim / 16 pieces of a token row).  The
// per-channel min/max is an in-lane reduction over the lane's pieces followed
// by an exchange between the lanes that hold the same channels.  Values are
// handled as x + 128 (0..255), exact in binary32; the differences x - mn the
// format defines are unchanged by the offset.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kv_lane_ops.hpp"
#include "kv_quant_kernels.hpp"

namespace kvs {

// 16 bytes (as four words) -> 16 floats 0..255
__device__ __forceinline__ void unpack16(const u4_t& w, float f[16]) {
    const uint32_t d[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        f[4 * j + 0] = static_cast<float>(d[j] & 0xffu);
        f[4 * j + 1] = static_cast<float>((d[j] >> 8) & 0xffu);
        f[4 * j + 2] = static_cast<float>((d[j] >> 16) & 0xffu);
        f[4 * j + 3] = static_cast<float>(d[j] >> 24);
    }
}

// rotate by N lanes inside each row of 16 lanes
template <int N>
__device__ __forceinline__ float row_ror(float v) {
    const int u = __builtin_bit_cast(int, v);
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(u, u, 0x120 + N, 0xF, 0xF, false));
}

// min (or max) over all lanes that hold the same channels: lanes l + j * rp,
// rp = 2^rp_log2 pieces per token row (4..64).
template <bool IS_MIN>
__device__ __forceinline__ float same_channel_reduce(float v, int rp_log2) {
    auto op = [](float a, float b) { return IS_MIN ? fminf(a, b) : fmaxf(a, b); };
    if (rp_log2 <= 2) v = op(v, row_ror<4>(v));
    if (rp_log2 <= 3) v = op(v, row_ror<8>(v));
    if (rp_log2 <= 4) v = op(v, __shfl_xor(v, 16));
    if (rp_log2 <= 5) v = IS_MIN ? xhalf_min(v) : xhalf_max(v);
    return v;
}

// Codes of 16 elements (exact small floats) -> BITS*2 bytes in up to two words.
template <int BITS>
__device__ __forceinline__ u2_t pack16(const float r[16]) {
    u2_t w = {0u, 0u};
    if constexpr (BITS == 4) {
        // four 4-bit codes = 16 bits: exact as a float sum
        float h[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            h[j] = __builtin_fmaf(r[4 * j + 3], 4096.0f,
                   __builtin_fmaf(r[4 * j + 2], 256.0f, __builtin_fmaf(r[4 * j + 1], 16.0f, r[4 * j])));
        w.x = static_cast<uint32_t>(h[0]) | (static_cast<uint32_t>(h[1]) << 16);
        w.y = static_cast<uint32_t>(h[2]) | (static_cast<uint32_t>(h[3]) << 16);
    } else if constexpr (BITS == 2) {
        float lo = r[7], hi = r[15];
#pragma unroll
        for (int k = 6; k >= 0; --k) {
            lo = __builtin_fmaf(lo, 4.0f, r[k]);
            hi = __builtin_fmaf(hi, 4.0f, r[8 + k]);
        }
        w.x = static_cast<uint32_t>(lo) | (static_cast<uint32_t>(hi) << 16);
    } else {
        float a = r[15];
#pragma unroll
        for (int k = 14; k >= 0; --k) a = __builtin_fmaf(a, 2.0f, r[k]);
        w.x = static_cast<uint32_t>(a);
    }
    return w;
}

template <int BITS, int PPL>
__device__ __forceinline__ void compress_i8_unit(const u4_t raw[PPL], uint8_t* __restrict__ codes,
                                                 float* __restrict__ scale_out,
                                                 float* __restrict__ mn_out, int rp_log2, int lane) {
    constexpr float kLevels = static_cast<float>((1 << BITS) - 1);
    constexpr float kSafe = 0.5f - static_cast<float>(1 << BITS) * 9.5367431640625e-07f;
    float f[PPL][16];
#pragma unroll
    for (int u = 0; u < PPL; ++u) {
        const u4_t biased = raw[u] ^ 0x80808080u;      // int8 -> x + 128, order preserved
        unpack16(biased, f[u]);
    }
    float scale[16], inv[16], mn[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        float lo = f[0][k], hi = f[0][k];
#pragma unroll
        for (int u = 1; u < PPL; ++u) {
            lo = fminf(lo, f[u][k]);
            hi = fmaxf(hi, f[u][k]);
        }
        lo = same_channel_reduce<true>(lo, rp_log2);
        hi = same_channel_reduce<false>(hi, rp_log2);
        mn[k] = lo;
        scale[k] = (hi - lo) / kLevels;
        inv[k] = (scale[k] != 0.0f) ? __builtin_amdgcn_rcpf(scale[k]) : 0.0f;
    }
#pragma unroll
    for (int u = 0; u < PPL; ++u) {
        float r[16];
        float emax = 0.0f;
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const float q = (f[u][k] - mn[k]) * inv[k];
            r[k] = __builtin_rintf(q);
            emax = fmaxf(emax, __builtin_fabsf(q - r[k]));
        }
        // integer data meet exact ties often: those lanes redo the piece with the true division
        if (emax >= kSafe) {
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                float c = 0.0f;
                if (scale[k] != 0.0f) {
                    c = __builtin_rintf((f[u][k] - mn[k]) / scale[k]);
                    c = __builtin_fminf(__builtin_fmaxf(c, 0.0f), kLevels);
                }
                r[k] = c;
            }
        }
        const u2_t w = pack16<BITS>(r);
        const int p = u * 64 + lane;
        if constexpr (BITS == 4) stream_store<KVS_NT_CODE_STORE>(w, reinterpret_cast<u2_t*>(codes) + p);
        else if constexpr (BITS == 2) stream_store<KVS_NT_CODE_STORE>(w.x, reinterpret_cast<uint32_t*>(codes) + p);
        else stream_store<KVS_NT_CODE_STORE>(static_cast<uint16_t>(w.x), reinterpret_cast<uint16_t*>(codes) + p);
    }
    // the first token row's lanes write their 16 channels' parameters
    if (lane < (1 << rp_log2)) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const u4_t sv = {__builtin_bit_cast(uint32_t, scale[4 * j]), __builtin_bit_cast(uint32_t, scale[4 * j + 1]),
                             __builtin_bit_cast(uint32_t, scale[4 * j + 2]), __builtin_bit_cast(uint32_t, scale[4 * j + 3])};
            const float m0 = mn[4 * j] - 128.0f, m1 = mn[4 * j + 1] - 128.0f, m2 = mn[4 * j + 2] - 128.0f,
                        m3 = mn[4 * j + 3] - 128.0f;
            const u4_t mv = {__builtin_bit_cast(uint32_t, m0), __builtin_bit_cast(uint32_t, m1),
                             __builtin_bit_cast(uint32_t, m2), __builtin_bit_cast(uint32_t, m3)};
            reinterpret_cast<u4_t*>(scale_out)[lane * 4 + j] = sv;
            reinterpret_cast<u4_t*>(mn_out)[lane * 4 + j] = mv;
        }
    }
}

// Grid as compress_kernel with one task per unit (g.tpu = 1); g.pieces = T * D / 16,
// g.row_pieces = D / 16, g.lpg_log2 = log2(row_pieces).
template <int PPL>
__global__ __launch_bounds__(256) void compress_i8_kernel(const u4_t* __restrict__ kv,
                                                          const uint8_t* __restrict__ bits,
                                                          const uint64_t* __restrict__ off,
                                                          uint8_t* __restrict__ packed, QuantGeom g,
                                                          int32_t n_chunks) {
    const int lane = threadIdx.x & 63;
    int chunk, slab, p0;
    if (!wave_task(g, n_chunks, PPL, chunk, slab, p0)) return;
    const u4_t* src = kv + (static_cast<uint64_t>(slab) * g.n_tokens +
                            static_cast<uint64_t>(chunk) * g.chunk_tokens) * g.row_pieces;
    u4_t raw[PPL];
#pragma unroll
    for (int u = 0; u < PPL; ++u) raw[u] = stream_load<KVS_NT_CACHE_LOAD>(src + u * 64 + lane);
    const int b = uniform_byte(bits, chunk);
    uint8_t* base = packed + off[chunk];
    if (b == 8) {
#pragma unroll
        for (int u = 0; u < PPL; ++u)
            stream_store<KVS_NT_CODE_STORE>(raw[u], reinterpret_cast<u4_t*>(base) +
                                            static_cast<uint64_t>(slab) * g.pieces + u * 64 + lane);
        return;
    }
    const uint64_t code_bytes = static_cast<uint64_t>(g.pieces) * 2 * b;   // T * D * b / 8 per unit
    const uint32_t channels = static_cast<uint32_t>(g.row_pieces) * 16;
    uint8_t* codes = base + slab * code_bytes;
    float* scale = reinterpret_cast<float*>(base + g.slabs * code_bytes) +
                   static_cast<uint64_t>(slab) * channels;
    float* mn = scale + static_cast<uint64_t>(g.slabs) * channels;
    if (b == 4) compress_i8_unit<4, PPL>(raw, codes, scale, mn, g.lpg_log2, lane);
    else if (b == 2) compress_i8_unit<2, PPL>(raw, codes, scale, mn, g.lpg_log2, lane);
    else compress_i8_unit<1, PPL>(raw, codes, scale, mn, g.lpg_log2, lane);
}

// ------------------------------------------------------------------ swap-in

template <int BITS, int PPL>
__device__ __forceinline__ void swapin_i8_unit(const uint8_t* __restrict__ codes,
                                               const float* __restrict__ scale_in,
                                               const float* __restrict__ mn_in,
                                               u4_t* __restrict__ dst, int rp_log2, int lane) {
    constexpr uint32_t kMask = (1u << BITS) - 1u;
    u2_t w[PPL];
#pragma unroll
    for (int u = 0; u < PPL; ++u) {
        const int p = u * 64 + lane;
        w[u] = u2_t{0u, 0u};
        if constexpr (BITS == 4) w[u] = stream_load<KVS_NT_CODE_LOAD>(reinterpret_cast<const u2_t*>(codes) + p);
        else if constexpr (BITS == 2) w[u].x = stream_load<KVS_NT_CODE_LOAD>(reinterpret_cast<const uint32_t*>(codes) + p);
        else w[u].x = stream_load<KVS_NT_CODE_LOAD>(reinterpret_cast<const uint16_t*>(codes) + p);
    }
    const int cb = lane & ((1 << rp_log2) - 1);        // which 16 channels this lane holds
    float sc[16], mn[16];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const u4_t sv = reinterpret_cast<const u4_t*>(scale_in)[cb * 4 + j];
        const u4_t mv = reinterpret_cast<const u4_t*>(mn_in)[cb * 4 + j];
        const uint32_t s4[4] = {sv.x, sv.y, sv.z, sv.w}, m4[4] = {mv.x, mv.y, mv.z, mv.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            sc[4 * j + k] = __builtin_bit_cast(float, s4[k]);
            mn[4 * j + k] = __builtin_bit_cast(float, m4[k]);
        }
    }
#pragma unroll
    for (int u = 0; u < PPL; ++u) {
        uint32_t out[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t word = 0;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int e = 4 * j + k;                  // element of the piece
                const int bitpos = e * BITS;
                const uint32_t c = ((bitpos < 32 ? w[u].x : w[u].y) >> (bitpos & 31)) & kMask;
                const float prod = static_cast<float>(c) * sc[e];    // rounded product, then rounded sum
                float v = __builtin_rintf(prod + mn[e]);
                v = __builtin_fminf(__builtin_fmaxf(v, -128.0f), 127.0f);
                word = __builtin_amdgcn_cvt_pk_u8_f32(v + 128.0f, k, word);
            }
            out[j] = word ^ 0x80808080u;                 // back to two's complement bytes
        }
        const u4_t v4 = {out[0], out[1], out[2], out[3]};
        stream_store<KVS_NT_CACHE_STORE>(v4, dst + u * 64 + lane);
    }
}

template <int PPL>
__device__ __forceinline__ void swapin_i8_task(const uint8_t* __restrict__ base, int b, int slab,
                                               u4_t* __restrict__ dst, const QuantGeom& g, int lane) {
    if (b == 8) {
        const u4_t* src = reinterpret_cast<const u4_t*>(base) + static_cast<uint64_t>(slab) * g.pieces;
        u4_t raw[PPL];
#pragma unroll
        for (int u = 0; u < PPL; ++u) raw[u] = stream_load<KVS_NT_CODE_LOAD>(src + u * 64 + lane);
#pragma unroll
        for (int u = 0; u < PPL; ++u) stream_store<KVS_NT_CACHE_STORE>(raw[u], dst + u * 64 + lane);
        return;
    }
    const uint64_t code_bytes = static_cast<uint64_t>(g.pieces) * 2 * b;
    const uint32_t channels = static_cast<uint32_t>(g.row_pieces) * 16;
    const uint8_t* codes = base + slab * code_bytes;
    const float* scale = reinterpret_cast<const float*>(base + g.slabs * code_bytes) +
                         static_cast<uint64_t>(slab) * channels;
    const float* mn = scale + static_cast<uint64_t>(g.slabs) * channels;
    if (b == 4) swapin_i8_unit<4, PPL>(codes, scale, mn, dst, g.lpg_log2, lane);
    else if (b == 2) swapin_i8_unit<2, PPL>(codes, scale, mn, dst, g.lpg_log2, lane);
    else swapin_i8_unit<1, PPL>(codes, scale, mn, dst, g.lpg_log2, lane);
}

template <int PPL>
__global__ __launch_bounds__(256) void swapin_i8_kernel(const uint8_t* __restrict__ packed,
                                                        const uint64_t* __restrict__ src_off,
                                                        const int32_t* __restrict__ dst_tok,
                                                        const uint8_t* __restrict__ sel_bits,
                                                        u4_t* __restrict__ kv_out, QuantGeom g,
                                                        int32_t n_sel) {
    const int lane = threadIdx.x & 63;
    int j, slab, p0;
    if (!wave_task(g, n_sel, PPL, j, slab, p0)) return;
    u4_t* dst = kv_out + (static_cast<uint64_t>(slab) * g.n_tokens +
                          static_cast<uint64_t>(dst_tok[j])) * g.row_pieces;
    swapin_i8_task<PPL>(packed + src_off[j], uniform_byte(sel_bits, j), slab, dst, g, lane);
}

template <int PPL>
__global__ __launch_bounds__(256) void swapin_i8_batch_kernel(const uint8_t* __restrict__ staged,
                                                              SwapinBatch list,
                                                              u4_t* __restrict__ kv_out, QuantGeom g) {
    const int lane = threadIdx.x & 63;
    int j, slab, p0;
    if (!wave_task(g, list.n, PPL, j, slab, p0)) return;
    u4_t* dst = kv_out + (static_cast<uint64_t>(slab) * g.n_tokens +
                          static_cast<uint64_t>(list.dst_tok[j])) * g.row_pieces;
    swapin_i8_task<PPL>(staged + list.src_off[j], list.bits[j], slab, dst, g, lane);
}

}  // namespace kvs
