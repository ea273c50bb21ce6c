// gfx950 kernels for the int8, channel-wise record format: the paper's own
// quantiser setting (Sec. 3.2 "Compressing chunks", Sec. 4): the cache is held
// as 8-bit integers and a chunk is quantised further to 4, 2 or 1 bits with one
// (scale, minimum) pair per head_dim channel of a slab, taken over the slab's
// chunk_tokens tokens.
//
// One wavefront handles one (chunk, slab) unit of chunk_tokens x head_dim bytes
// (1, 2 or 4 KiB).  On the cache side a lane owns pieces of 16 consecutive
// bytes, piece u * 64 + lane, so every access is a coalesced 16-byte one.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kv_lane_ops.hpp"
#include "kv_quant_kernels.hpp"

namespace kvs {

// ------------------------------------------------------------------ compress
//
// The wavefront loads its unit with coalesced 16-byte accesses, parks it in LDS
// and reads it back transposed: a lane then holds, for one group of 4 adjacent
// channels (GPL groups where head_dim > 256), the dwords of RPL token rows, so
// the per-channel min/max is an in-lane reduction on packed 16-bit pairs, with
// one or two cross-lane steps where 2 or 4 lanes share a channel group
// (head_dim 128 or 64).  Codes go back through LDS into record order and leave
// as one coalesced store per lane.  No workgroup barrier: every LDS byte is
// produced and consumed by the same wavefront.
//
// Arithmetic.  Values are handled as x + 128 (0..255), exact in binary32; the
// differences x - mn of the format are unchanged by the offset.  With integer
// data the quotient (x - mn) / scale is very often an exact half-integer, so
// every element takes the correctly rounded division, spelled out: both
// divisions of the format are the reciprocal-refinement sequence the compiler
// emits for a binary32 '/', without its range scaling, which is the identity
// for these operands (numerators 0..255, scales 0 or 1/15..255).

__device__ __forceinline__ uint32_t pk_min_u16(uint32_t a, uint32_t b) {
    uint32_t r;
    asm("v_pk_min_u16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b) {
    uint32_t r;
    asm("v_pk_max_u16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// (range / levels) correctly rounded, levels in {1, 3, 15}: with c the correctly
// rounded reciprocal of the constant, one residual correction of the product
// range * c gives the correctly rounded quotient (Markstein's theorem).
template <int LEVELS>
__device__ __forceinline__ float div_levels(float range) {
    if constexpr (LEVELS == 1) return range;
    constexpr float c = 1.0f / static_cast<float>(LEVELS);
    const float q0 = range * c;
    const float e = __builtin_fmaf(-static_cast<float>(LEVELS), q0, range);
    return __builtin_fmaf(e, c, q0);
}

// Reciprocal of a scale, refined once (0 for a zero scale: every quotient is then 0).
__device__ __forceinline__ float refined_rcp(float s) {
    const float r0 = (s != 0.0f) ? __builtin_amdgcn_rcpf(s) : 0.0f;
    const float e = __builtin_fmaf(-s, r0, 1.0f);
    return (s != 0.0f) ? __builtin_fmaf(e, r0, r0) : 0.0f;
}

// Residual corrections of the quotient.  The operand domain is finite (numerators 0..255, one
// scale per range 0..255, level count and parameter precision), and the GPU tests compare the
// codes of every such pair with the oracle's true division: one correction reproduces all of
// them, none does not.
// d / s rounded as the division does on this domain (rinv = refined_rcp(s)).
__device__ __forceinline__ float div_exact(float d, float s, float rinv) {
    const float q = d * rinv;
    const float e = __builtin_fmaf(-s, q, d);
    return __builtin_fmaf(e, rinv, q);
}

template <int BYTES>
__device__ __forceinline__ void copy_out(const uint8_t* __restrict__ img, uint8_t* __restrict__ dst, int lane) {
    if constexpr (BYTES >= 16) {
#pragma unroll
        for (int u = 0; u < BYTES / 16; ++u)
            stream_store<true>(reinterpret_cast<const u4_t*>(img)[u * 64 + lane],
                                            reinterpret_cast<u4_t*>(dst) + u * 64 + lane);
    } else if constexpr (BYTES == 8) {
        stream_store<true>(reinterpret_cast<const u2_t*>(img)[lane], reinterpret_cast<u2_t*>(dst) + lane);
    } else if constexpr (BYTES == 4) {
        stream_store<true>(reinterpret_cast<const uint32_t*>(img)[lane],
                                        reinterpret_cast<uint32_t*>(dst) + lane);
    } else {
        stream_store<true>(reinterpret_cast<const uint16_t*>(img)[lane],
                                        reinterpret_cast<uint16_t*>(dst) + lane);
    }
}

// Geometry of the transposed view, uniform per launch.
struct I8View {
    int32_t head_dim;     // D
    int32_t group_lanes;  // lanes along the channel groups: min(D / 4, 64)
    int32_t share_log2;   // log2 of the lanes that share a channel group: 0, 1 (D = 128) or 2 (D = 64)
    int32_t half_meta;    // 1: parameters are stored, and the scale is used, in binary16 (host side:
                          // selects the HM instantiation of the kernels)
};

// Four binary32 values as four binary16 (round to nearest even), lowest index in the lowest bits.
__device__ __forceinline__ uint32_t half_bits(float f) {
    return __builtin_bit_cast(uint16_t, static_cast<_Float16>(f));
}
__device__ __forceinline__ uint32_t half_to_float_bits(uint32_t h) {
    return __builtin_bit_cast(uint32_t, static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(h))));
}
__device__ __forceinline__ u2_t pack_halves(const float (&f)[4]) {
    return u2_t{half_bits(f[0]) | (half_bits(f[1]) << 16), half_bits(f[2]) | (half_bits(f[3]) << 16)};
}
__device__ __forceinline__ void unpack_halves(u2_t w, uint32_t (&bits32)[4]) {
    bits32[0] = half_to_float_bits(w.x & 0xffffu);
    bits32[1] = half_to_float_bits(w.x >> 16);
    bits32[2] = half_to_float_bits(w.y & 0xffffu);
    bits32[3] = half_to_float_bits(w.y >> 16);
}

// NDW = dwords per lane (unit bytes / 256: 4, 8, 16); GPL = channel groups per lane (D / 256, at least 1).
template <int BITS, int NDW, int GPL, bool HM>
__device__ __forceinline__ void compress_i8_unit(const uint8_t* __restrict__ raw_img, uint8_t* __restrict__ code_img,
                                                 uint8_t* __restrict__ codes, void* __restrict__ scale_out,
                                                 void* __restrict__ mn_out, const I8View& v, int lane) {
    constexpr int LEVELS = (1 << BITS) - 1;
    constexpr int RPL = NDW / GPL;                         // token rows per lane and group
    const int c = lane & (v.group_lanes - 1);              // channel group (+ 64 * j)
    const int rpart = lane >> (6 - v.share_log2);          // which block of RPL rows (0 unless lanes share)
    const int row0 = rpart * RPL;
    uint32_t w[GPL][RPL];
#pragma unroll
    for (int j = 0; j < GPL; ++j)
#pragma unroll
        for (int k = 0; k < RPL; ++k)
            w[j][k] = *reinterpret_cast<const uint32_t*>(raw_img + (row0 + k) * v.head_dim + 4 * (c + 64 * j));
#pragma unroll
    for (int j = 0; j < GPL; ++j) {
        // bytes 0 and 2 of a dword as one 16-bit pair, bytes 1 and 3 as another
        uint32_t mnE = w[j][0] & 0x00ff00ffu, mnO = (w[j][0] >> 8) & 0x00ff00ffu;
        uint32_t mxE = mnE, mxO = mnO;
#pragma unroll
        for (int k = 1; k < RPL; ++k) {
            const uint32_t e = w[j][k] & 0x00ff00ffu, o = (w[j][k] >> 8) & 0x00ff00ffu;
            mnE = pk_min_u16(mnE, e); mxE = pk_max_u16(mxE, e);
            mnO = pk_min_u16(mnO, o); mxO = pk_max_u16(mxO, o);
        }
        if (v.share_log2 >= 1) {       // lanes l and l ^ 32
            uint32_t lo, hi;
            xhalf_both_u32(mnE, lo, hi); mnE = pk_min_u16(lo, hi);
            xhalf_both_u32(mnO, lo, hi); mnO = pk_min_u16(lo, hi);
            xhalf_both_u32(mxE, lo, hi); mxE = pk_max_u16(lo, hi);
            xhalf_both_u32(mxO, lo, hi); mxO = pk_max_u16(lo, hi);
        }
        if (v.share_log2 >= 2) {       // and l ^ 16
            mnE = pk_min_u16(mnE, static_cast<uint32_t>(__shfl_xor(static_cast<int>(mnE), 16)));
            mnO = pk_min_u16(mnO, static_cast<uint32_t>(__shfl_xor(static_cast<int>(mnO), 16)));
            mxE = pk_max_u16(mxE, static_cast<uint32_t>(__shfl_xor(static_cast<int>(mxE), 16)));
            mxO = pk_max_u16(mxO, static_cast<uint32_t>(__shfl_xor(static_cast<int>(mxO), 16)));
        }
        // channel 4g + i: i = 0, 2 in the even pair, 1, 3 in the odd pair
        float mn[4], scale[4], rinv[4];
        const uint32_t mnw[4] = {mnE & 0xffffu, mnO & 0xffffu, mnE >> 16, mnO >> 16};
        const uint32_t mxw[4] = {mxE & 0xffffu, mxO & 0xffffu, mxE >> 16, mxO >> 16};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            mn[i] = static_cast<float>(mnw[i]);
            scale[i] = div_levels<LEVELS>(static_cast<float>(mxw[i] - mnw[i]));
            if constexpr (HM) scale[i] = static_cast<float>(static_cast<_Float16>(scale[i]));
            rinv[i] = refined_rcp(scale[i]);
        }
        const int g4 = c + 64 * j;                            // channel group index in the row
#pragma unroll
        for (int k = 0; k < RPL; ++k) {
            const uint32_t x = w[j][k];
            const float xf[4] = {static_cast<float>(x & 0xffu), static_cast<float>((x >> 8) & 0xffu),
                                 static_cast<float>((x >> 16) & 0xffu), static_cast<float>(x >> 24)};
            uint32_t acc = 0;
#pragma unroll
            for (int i = 3; i >= 0; --i) {
                const float q = div_exact(xf[i] - mn[i], scale[i], rinv[i]);
                // q + 1.5 * 2^23 rounds q to an integer, halves to even; the code is in the low mantissa bits
                const uint32_t u = __builtin_bit_cast(uint32_t, q + 12582912.0f);
                acc = (acc << BITS) + u;
            }
            const int row = row0 + k;
            if constexpr (BITS == 4) {
                *reinterpret_cast<uint16_t*>(code_img + row * (v.head_dim >> 1) + 2 * g4) = static_cast<uint16_t>(acc);
            } else if constexpr (BITS == 2) {
                code_img[row * (v.head_dim >> 2) + g4] = static_cast<uint8_t>(acc);
            } else {
                // two neighbouring lanes (adjacent channel groups) share a byte
                const uint32_t nb = dpp_u32<0xB1>(acc);
                if ((lane & 1) == 0)
                    code_img[row * (v.head_dim >> 3) + (g4 >> 1)] = static_cast<uint8_t>((acc & 0xfu) | ((nb & 0xfu) << 4));
            }
        }
        if (rpart == 0) {
            const float mo[4] = {mn[0] - 128.0f, mn[1] - 128.0f, mn[2] - 128.0f, mn[3] - 128.0f};
            if constexpr (HM) {
                reinterpret_cast<u2_t*>(scale_out)[g4] = pack_halves(scale);
                reinterpret_cast<u2_t*>(mn_out)[g4] = pack_halves(mo);
            } else {
                const u4_t sv = {__builtin_bit_cast(uint32_t, scale[0]), __builtin_bit_cast(uint32_t, scale[1]),
                                 __builtin_bit_cast(uint32_t, scale[2]), __builtin_bit_cast(uint32_t, scale[3])};
                const u4_t mv = {__builtin_bit_cast(uint32_t, mo[0]), __builtin_bit_cast(uint32_t, mo[1]),
                                 __builtin_bit_cast(uint32_t, mo[2]), __builtin_bit_cast(uint32_t, mo[3])};
                reinterpret_cast<u4_t*>(scale_out)[g4] = sv;
                reinterpret_cast<u4_t*>(mn_out)[g4] = mv;
            }
        }
    }
    // LDS writes of this wavefront are ordered before its reads below
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    copy_out<NDW * BITS / 2>(code_img, codes, lane);
}

// Grid as compress_kernel with one task per unit (g.tpu = 1); g.pieces = T * D / 16,
// g.row_pieces = D / 16.  LDS: per wavefront the unit (NDW * 256 bytes) and its codes (at most half of that).
template <int NDW, int GPL, bool HM>
__global__ __launch_bounds__(256) void compress_i8_kernel(const u4_t* __restrict__ kv,
                                                          const uint8_t* __restrict__ bits,
                                                          const uint64_t* __restrict__ off,
                                                          uint8_t* __restrict__ packed, QuantGeom g,
                                                          I8View v, int32_t n_chunks,
                                                          const int32_t* __restrict__ chunk_list) {
    constexpr int PPL = NDW / 4;
    __shared__ __align__(16) uint8_t lds[kWavesPerBlock][NDW * 256 + NDW * 128];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));
    int chunk, slab, p0;
    if (!wave_task(g, n_chunks, PPL, chunk, slab, p0)) return;
    if (chunk_list) chunk = chunk_list[chunk];          // only the listed chunks
    const u4_t* src = kv + (static_cast<uint64_t>(slab) * g.n_tokens +
                            static_cast<uint64_t>(chunk) * g.chunk_tokens) * g.row_pieces;
    u4_t raw[PPL];
#pragma unroll
    for (int u = 0; u < PPL; ++u) raw[u] = stream_load<true>(src + u * 64 + lane);
    int b = uniform_byte(bits, chunk);
    uint64_t rec = off[chunk];
    asm volatile("" : "+s"(b), "+s"(rec));               // both scalar loads issued, one wait
    uint8_t* base = packed + rec;
    if (b == 8) {
#pragma unroll
        for (int u = 0; u < PPL; ++u)
            stream_store<true>(raw[u], reinterpret_cast<u4_t*>(base) +
                                            static_cast<uint64_t>(slab) * g.pieces + u * 64 + lane);
        return;
    }
    uint8_t* raw_img = lds[wave];
    uint8_t* code_img = raw_img + NDW * 256;
#pragma unroll
    for (int u = 0; u < PPL; ++u)       // int8 -> x + 128, order preserved
        reinterpret_cast<u4_t*>(raw_img)[u * 64 + lane] = raw[u] ^ 0x80808080u;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const uint64_t code_bytes = static_cast<uint64_t>(g.pieces) * 2 * b;   // T * D * b / 8 per unit
    const uint64_t meta_bytes = static_cast<uint64_t>(v.head_dim) * (HM ? 2 : 4);   // per slab and section
    uint8_t* codes = base + slab * code_bytes;
    uint8_t* scale = base + g.slabs * code_bytes + slab * meta_bytes;
    uint8_t* mn = scale + g.slabs * meta_bytes;
    if (b == 4) compress_i8_unit<4, NDW, GPL, HM>(raw_img, code_img, codes, scale, mn, v, lane);
    else if (b == 2) compress_i8_unit<2, NDW, GPL, HM>(raw_img, code_img, codes, scale, mn, v, lane);
    else compress_i8_unit<1, NDW, GPL, HM>(raw_img, code_img, codes, scale, mn, v, lane);
}

// ------------------------------------------------------------------ swap-in
//
// The same transposed view as compress, the other way round: the unit's codes are
// loaded in record order (one coalesced access per lane), parked in LDS and read
// back by the lane that holds 4 adjacent channels of a token row; that lane loads
// the parameters of its channels itself (two 16-byte loads per channel group
// instead of the 32 parameters of a 16-channel piece per piece), dequantises,
// packs four bytes and parks them in LDS in cache order, from where they leave as
// coalesced 16-byte stores.

template <int BYTES>
__device__ __forceinline__ void copy_in(const uint8_t* __restrict__ src, uint8_t* __restrict__ img, int lane) {
    if constexpr (BYTES >= 16) {
#pragma unroll
        for (int u = 0; u < BYTES / 16; ++u)
            reinterpret_cast<u4_t*>(img)[u * 64 + lane] =
                stream_load<true>(reinterpret_cast<const u4_t*>(src) + u * 64 + lane);
    } else if constexpr (BYTES == 8) {
        reinterpret_cast<u2_t*>(img)[lane] = stream_load<true>(reinterpret_cast<const u2_t*>(src) + lane);
    } else if constexpr (BYTES == 4) {
        reinterpret_cast<uint32_t*>(img)[lane] =
            stream_load<true>(reinterpret_cast<const uint32_t*>(src) + lane);
    } else {
        reinterpret_cast<uint16_t*>(img)[lane] =
            stream_load<true>(reinterpret_cast<const uint16_t*>(src) + lane);
    }
}

// x = int8(clamp(rint(code * scale + mn), -128, 127)): product and sum rounded separately; the
// saturating conversion of x + 128 to an unsigned byte is the clamp (x is an integer after rint).
template <int BITS, int NDW, int GPL, bool HM>
__device__ __forceinline__ void swapin_i8_unit(const uint8_t* __restrict__ codes,
                                               const void* __restrict__ scale_in,
                                               const void* __restrict__ mn_in, uint8_t* __restrict__ code_img,
                                               uint8_t* __restrict__ raw_img, u4_t* __restrict__ dst,
                                               const I8View& v, int lane) {
    constexpr int PPL = NDW / 4;
    constexpr int RPL = NDW / GPL;
    constexpr uint32_t kMask = (1u << BITS) - 1u;
    copy_in<NDW * BITS / 2>(codes, code_img, lane);
    const int c = lane & (v.group_lanes - 1);
    const int rpart = lane >> (6 - v.share_log2);
    const int row0 = rpart * RPL;
    u4_t sv[GPL], mv[GPL];           // binary16 parameters travel in .x and .y
#pragma unroll
    for (int j = 0; j < GPL; ++j) {
        if constexpr (HM) {
            const u2_t sh = reinterpret_cast<const u2_t*>(scale_in)[c + 64 * j];
            const u2_t mh = reinterpret_cast<const u2_t*>(mn_in)[c + 64 * j];
            sv[j] = u4_t{sh.x, sh.y, 0u, 0u};
            mv[j] = u4_t{mh.x, mh.y, 0u, 0u};
        } else {
            sv[j] = reinterpret_cast<const u4_t*>(scale_in)[c + 64 * j];
            mv[j] = reinterpret_cast<const u4_t*>(mn_in)[c + 64 * j];
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int j = 0; j < GPL; ++j) {
        const int g4 = c + 64 * j;
        uint32_t s4[4] = {sv[j].x, sv[j].y, sv[j].z, sv[j].w};
        uint32_t m4[4] = {mv[j].x, mv[j].y, mv[j].z, mv[j].w};
        if constexpr (HM) {
            unpack_halves(u2_t{sv[j].x, sv[j].y}, s4);
            unpack_halves(u2_t{mv[j].x, mv[j].y}, m4);
        }
#pragma unroll
        for (int k = 0; k < RPL; ++k) {
            const int row = row0 + k;
            uint32_t cw;                   // the four codes of (row, channel group), lowest channel lowest
            if constexpr (BITS == 4) {
                cw = *reinterpret_cast<const uint16_t*>(code_img + row * (v.head_dim >> 1) + 2 * g4);
            } else if constexpr (BITS == 2) {
                cw = code_img[row * (v.head_dim >> 2) + g4];
            } else {
                cw = code_img[row * (v.head_dim >> 3) + (g4 >> 1)];
                cw >>= 4 * (g4 & 1);
            }
            uint32_t word = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t code = (cw >> (i * BITS)) & kMask;
                const float prod = static_cast<float>(code) * __builtin_bit_cast(float, s4[i]);
                const float x = __builtin_rintf(prod + __builtin_bit_cast(float, m4[i]));
                word = __builtin_amdgcn_cvt_pk_u8_f32(x + 128.0f, i, word);
            }
            *reinterpret_cast<uint32_t*>(raw_img + row * v.head_dim + 4 * g4) = word ^ 0x80808080u;
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int u = 0; u < PPL; ++u)
        stream_store<true>(reinterpret_cast<const u4_t*>(raw_img)[u * 64 + lane], dst + u * 64 + lane);
}

template <int NDW, int GPL, bool HM>
__device__ __forceinline__ void swapin_i8_task(const uint8_t* __restrict__ base, int b, int slab,
                                               u4_t* __restrict__ dst, const QuantGeom& g, const I8View& v,
                                               uint8_t* __restrict__ lds_wave, int lane) {
    constexpr int PPL = NDW / 4;
    if (b == 8) {
        const u4_t* src = reinterpret_cast<const u4_t*>(base) + static_cast<uint64_t>(slab) * g.pieces;
        u4_t raw[PPL];
#pragma unroll
        for (int u = 0; u < PPL; ++u) raw[u] = stream_load<true>(src + u * 64 + lane);
#pragma unroll
        for (int u = 0; u < PPL; ++u) stream_store<true>(raw[u], dst + u * 64 + lane);
        return;
    }
    const uint64_t code_bytes = static_cast<uint64_t>(g.pieces) * 2 * b;
    const uint64_t meta_bytes = static_cast<uint64_t>(v.head_dim) * (HM ? 2 : 4);
    const uint8_t* codes = base + slab * code_bytes;
    const uint8_t* scale = base + g.slabs * code_bytes + slab * meta_bytes;
    const uint8_t* mn = scale + g.slabs * meta_bytes;
    uint8_t* raw_img = lds_wave;
    uint8_t* code_img = lds_wave + NDW * 256;
    if (b == 4) swapin_i8_unit<4, NDW, GPL, HM>(codes, scale, mn, code_img, raw_img, dst, v, lane);
    else if (b == 2) swapin_i8_unit<2, NDW, GPL, HM>(codes, scale, mn, code_img, raw_img, dst, v, lane);
    else swapin_i8_unit<1, NDW, GPL, HM>(codes, scale, mn, code_img, raw_img, dst, v, lane);
}

// LDS per wavefront as in compress_i8_kernel: the unit (NDW * 256 bytes) and its codes.  Launched like the
// fp16 Load kernels (one-dimensional grid in strip order) with at most kWavesPerBlock wavefronts per workgroup.
template <int NDW, int GPL, bool HM>
__global__ __launch_bounds__(256) void swapin_i8_kernel(const uint8_t* __restrict__ packed,
                                                        const uint64_t* __restrict__ src_off,
                                                        const int32_t* __restrict__ dst_tok,
                                                        const uint8_t* __restrict__ sel_bits,
                                                        u4_t* __restrict__ kv_out, QuantGeom g, I8View v,
                                                        int32_t n_sel) {
    __shared__ __align__(16) uint8_t lds[kWavesPerBlock][NDW * 256 + NDW * 128];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));
    int j, slab, p0;
    if (!strip_task_at(g, n_sel, NDW / 4, blockIdx.x, static_cast<int>(blockDim.x >> 6), j, slab, p0)) return;
    const GatherEntry e = gather_entry(src_off, dst_tok, sel_bits, j);
    u4_t* dst = kv_out + (static_cast<uint64_t>(slab) * g.n_tokens +
                          static_cast<uint64_t>(e.tok)) * g.row_pieces;
    swapin_i8_task<NDW, GPL, HM>(packed + e.src, e.b, slab, dst, g, v, lds[wave], lane);
}

// Record pool in pinned host memory: a small grid that walks the task grid in strides (see
// swapin_link_kernel).  A wavefront reuses its LDS region from task to task, in program order.
template <int NDW, int GPL, bool HM>
__global__ __launch_bounds__(256) void swapin_i8_link_kernel(const uint8_t* __restrict__ packed,
                                                             const uint64_t* __restrict__ src_off,
                                                             const int32_t* __restrict__ dst_tok,
                                                             const uint8_t* __restrict__ sel_bits,
                                                             u4_t* __restrict__ kv_out, QuantGeom g, I8View v,
                                                             int32_t n_sel, uint32_t total) {
    __shared__ __align__(16) uint8_t lds[kWavesPerBlock][NDW * 256 + NDW * 128];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));
    for (uint32_t w = blockIdx.x; w < total; w += gridDim.x) {
        int j, slab, p0;
        if (!strip_task_at(g, n_sel, NDW / 4, w, static_cast<int>(blockDim.x >> 6), j, slab, p0)) continue;
        const GatherEntry e = gather_entry<false>(src_off, dst_tok, sel_bits, j);
        u4_t* dst = kv_out + (static_cast<uint64_t>(slab) * g.n_tokens +
                              static_cast<uint64_t>(e.tok)) * g.row_pieces;
        swapin_i8_task<NDW, GPL, HM>(packed + e.src, e.b, slab, dst, g, v, lds[wave], lane);
    }
}

template <int NDW, int GPL, bool HM>
__global__ __launch_bounds__(256) void swapin_i8_batch_kernel(const uint8_t* __restrict__ staged,
                                                              SwapinBatch list,
                                                              u4_t* __restrict__ kv_out, QuantGeom g, I8View v) {
    __shared__ __align__(16) uint8_t lds[kWavesPerBlock][NDW * 256 + NDW * 128];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));
    int j, slab, p0;
    if (!strip_task_at(g, list.n, NDW / 4, blockIdx.x, static_cast<int>(blockDim.x >> 6), j, slab, p0)) return;
    u4_t* dst = kv_out + (static_cast<uint64_t>(slab) * g.n_tokens +
                          static_cast<uint64_t>(list.dst_tok[j])) * g.row_pieces;
    swapin_i8_task<NDW, GPL, HM>(staged + list.src_off[j], list.bits[j], slab, dst, g, v, lds[wave], lane);
}

}  // namespace kvs
