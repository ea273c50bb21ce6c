// gfx950 kernels for chunk compression (quantise + bit-pack) and swap-in
// (gather + unpack + dequantise).  Sec. 3.2 "Compressing chunks", Sec. 4
// (bit-shift packing), Load primitive of Sec. 3.1.
//
// Work unit: one (chunk, slab) pair = chunk_tokens x head_dim contiguous fp16
// on the cache side and one contiguous run of code bytes on the record side.
// A lane owns "pieces" of 8 consecutive elements (one 16-byte cache access); a
// wavefront instruction touches 64 consecutive pieces (1 KiB of cache), fully
// coalesced.  A quantisation group of G elements is spread over G/8
// neighbouring lanes, so its min/max is a short DPP butterfly.  A wavefront
// task is PPL * 64 pieces of one unit, all loads issued before any arithmetic:
// measured on MI355X, one piece per lane streams best for a plain copy, but
// the quantising paths need 4 to amortise the dependent scalar loads of the
// per-chunk lists and to hide their arithmetic.  The chunk index of a task is
// wave-uniform, so the bit-width and the record offset are scalar loads and
// the branch on the width is uniform.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kvs {

typedef _Float16 h8_t __attribute__((ext_vector_type(8)));
typedef unsigned int u4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u2_t __attribute__((ext_vector_type(2)));

struct QuantGeom {
    int32_t n_tokens;      // N
    int32_t chunk_tokens;  // T
    int32_t slabs;         // layers * 2 * kv_heads (fixes the record layout)
    int32_t slab0;         // the launch covers slabs [slab0, slab0 + slab_count): all of them, or
    int32_t slab_count;    // those of a range of layers (layer-wise Load, Sec. 3.3)
    int32_t pieces;        // T * D / 8: 16-byte pieces per unit (multiple of 64)
    int32_t row_pieces;    // D / 8
    int32_t lpg_log2;      // log2(G / 8): lanes per quantisation group (3..6)
    int32_t tpu;           // wavefront tasks per unit = pieces / (64 * pieces-per-lane)
    int32_t tpu_shift;     // log2(tpu) if tpu is a power of two, else -1
    int32_t record_major;  // task order: 0 = walk the chunks of one slab (cache side is one
                           // stream), 1 = walk the slabs of one chunk (record side is one stream)
    int32_t strip;         // Load kernels (fp16 formats): slabs written side by side, one per XCD (kStripSlabs)
    int32_t groups;        // Load kernels: workgroups per slab = ceil(listed chunks * tpu / waves per workgroup)
};

constexpr int kWavesPerBlock = 4;

// Entry i of a byte list at a wave-uniform index, read through the aligned
// 32-bit word that contains it so that it can be a scalar load.  The word's address is
// formed by pointer arithmetic on `list` itself (never through an integer), so that the
// compiler still knows it points to global memory: a pointer rebuilt from an integer is a
// generic one, whose load is a vector instruction, and the width it returns then lives in a
// vector register - every branch on it and every address derived from it with it.
__device__ __forceinline__ int uniform_byte(const uint8_t* __restrict__ list, int i) {
    const int skew = static_cast<int>(reinterpret_cast<uintptr_t>(list) & 3);
    const int k = i + skew;                                     // index from the aligned word before `list`
    const uint32_t* words = reinterpret_cast<const uint32_t*>(list - skew);
    const uint32_t w = words[k >> 2];
    return static_cast<int>((w >> ((k & 3) * 8)) & 0xffu);
}

// The list entries of gather task j (wave-uniform): three scalar loads issued together and waited for
// once.  Left to the compiler they are issued one by one, each in front of its first use, and a
// wavefront that has a single task spends three trips to the scalar cache before its first vector load.
struct GatherEntry {
    uint64_t src;
    int32_t tok;
    int b;
};
template <bool TOGETHER = true, bool SCALAR_WIDTH = true>
__device__ __forceinline__ GatherEntry gather_entry(const uint64_t* __restrict__ src_off,
                                                    const int32_t* __restrict__ dst_tok,
                                                    const uint8_t* __restrict__ sel_bits, int j) {
    GatherEntry e;
    e.tok = dst_tok[j];
    e.src = src_off[j];
    if constexpr (SCALAR_WIDTH) e.b = uniform_byte(sel_bits, j);
    else e.b = sel_bits[j];          // a byte load is a vector load: the width stays in a vector register
    // all of them are needed here (not in the kernels that walk tasks in a loop, where the compiler
    // does not keep the entries in scalar registers)
    if constexpr (TOGETHER && SCALAR_WIDTH) asm volatile("" : "+s"(e.tok), "+s"(e.src), "+s"(e.b));
    else if constexpr (TOGETHER) asm volatile("" : "+s"(e.tok), "+s"(e.src));
    return e;
}

// Wavefront task -> (chunk or list index, slab, first piece).  Task ids are uniform
// per wavefront; readfirstlane keeps everything derived from them in SGPRs, so
// the per-chunk list entries become scalar loads and the width branch is uniform.
__device__ __forceinline__ bool wave_task_at(const QuantGeom& g, int n_chunks, int ppl, uint32_t bx,
                                             uint32_t by, int& chunk, int& slab, int& piece0) {
    const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));
    const int t = static_cast<int>(bx) * kWavesPerBlock + wave;
    int unit, sub;
    if (g.tpu_shift >= 0) {
        unit = t >> g.tpu_shift;
        sub = t & (g.tpu - 1);
    } else {
        unit = t / g.tpu;
        sub = t - unit * g.tpu;
    }
    piece0 = sub * 64 * ppl;
    if (g.record_major) {
        slab = g.slab0 + unit;
        chunk = static_cast<int>(by);
        return unit < g.slab_count;
    }
    chunk = unit;
    slab = g.slab0 + static_cast<int>(by);
    return unit < n_chunks;
}

// Task order of the Load kernels of the fp16 formats.  The launch is one-dimensional; a workgroup of
// `wpb` wavefronts takes wpb consecutive tasks of ONE slab (consecutive chunks of the list: their
// tokens are adjacent in the cache where the chunks are), and consecutive workgroup ids walk a strip
// of kStripSlabs slabs before they move on along the token axis.  Workgroup ids are dealt to the
// eight XCDs in turn, so with a strip of eight every XCD writes ONE plane of the cache as a forward
// stream through its own L2, and the eight planes of a strip are neighbours in memory.  Measured on
// MI355X (4096-token multi-head cache, stores only): 7.4 TB/s, against 6.0 TB/s when consecutive
// workgroups write consecutive 8 KiB blocks of one plane (each XCD then sees every eighth block) -
// and the whole kernel 0.485 against 0.517 ms.
constexpr int kStripSlabs = 8;
constexpr int kLoadWavesMax = 8;      // wavefronts per workgroup of the Load kernels at most

__device__ __forceinline__ bool strip_task_at(const QuantGeom& g, int n_units, int ppl, uint32_t id, int wpb,
                                              int& unit, int& slab, int& piece0) {
    const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));
    const uint32_t per_strip = static_cast<uint32_t>(g.groups) * static_cast<uint32_t>(g.strip);
    const uint32_t s = id / per_strip;                      // strip (the last one may be narrower)
    const uint32_t local = id - s * per_strip;
    const int first = static_cast<int>(s) * g.strip;
    const int width = min(g.strip, g.slab_count - first);
    const uint32_t grp = local / static_cast<uint32_t>(width);
    slab = g.slab0 + first + static_cast<int>(local - grp * static_cast<uint32_t>(width));
    const int t = static_cast<int>(grp) * wpb + wave;       // task inside the slab
    int sub;
    if (g.tpu_shift >= 0) {
        unit = t >> g.tpu_shift;
        sub = t & (g.tpu - 1);
    } else {
        unit = t / g.tpu;
        sub = t - unit * g.tpu;
    }
    piece0 = sub * 64 * ppl;
    return unit < n_units;
}

__device__ __forceinline__ bool wave_task(const QuantGeom& g, int n_chunks, int ppl, int& chunk,
                                          int& slab, int& piece0) {
    return wave_task_at(g, n_chunks, ppl, blockIdx.x, blockIdx.y, chunk, slab, piece0);
}

// Streaming accesses: every byte is touched once, so cache loads, code loads, code stores and cache
// stores are all marked non-temporal (measured per access on MI355X: each of the four gains, ~4 % together).
template <bool NT, typename T>
__device__ __forceinline__ T stream_load(const T* p) {
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}
template <bool NT, typename T>
__device__ __forceinline__ void stream_store(T v, T* p) {
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// Packed fp16 min/max on raw registers.  Written as instructions so that no
// NaN-quieting copies are inserted in front of them (inputs are finite).
__device__ __forceinline__ uint32_t pk_min_f16(uint32_t a, uint32_t b) {
    uint32_t r;
    asm("v_pk_min_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ uint32_t pk_max_f16(uint32_t a, uint32_t b) {
    uint32_t r;
    asm("v_pk_max_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// DPP lane exchange inside a row of 16 lanes.  CTRL: 0xB1 = swap neighbours,
// 0x4E = swap lane pairs, 0x141 = mirror inside 8 lanes, 0x140 = mirror inside 16.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
    return static_cast<uint32_t>(
        __builtin_amdgcn_update_dpp(static_cast<int>(v), static_cast<int>(v), CTRL, 0xF, 0xF, false));
}

// x + 0.0f of the format definition (-0 becomes +0, everything else is kept),
// as an instruction so that no floating-point simplification can drop it.
__device__ __forceinline__ float plus_zero(float x) {
    float r;
    asm("v_add_f32 %0, 0, %1" : "=v"(r) : "v"(x));
    return r;
}

// min and max of the quantisation group this lane's piece belongs to
// (2^lpg_log2 neighbouring lanes), as binary32 with -0 canonicalised to +0.
__device__ __forceinline__ void group_min_max(const u4_t& raw, int lpg_log2, float& mn, float& mx) {
    uint32_t lo = pk_min_f16(pk_min_f16(raw.x, raw.y), pk_min_f16(raw.z, raw.w));
    uint32_t hi = pk_max_f16(pk_max_f16(raw.x, raw.y), pk_max_f16(raw.z, raw.w));
    // lo = (min of the even elements, min of the odd ones), hi the same for the maxima.  With the maxima
    // negated, one packed min of (lo.even, -hi.odd) and (lo.odd, -hi.even) leaves (min, -max) of the eight
    // elements in one register, and every later packed min reduces both at once.
    const uint32_t nh = hi ^ 0x80008000u;
    uint32_t m = pk_min_f16((lo & 0xffffu) | (nh & 0xffff0000u), __builtin_amdgcn_alignbit(nh, lo, 16));
    m = pk_min_f16(m, dpp_u32<0xB1>(m));
    m = pk_min_f16(m, dpp_u32<0x4E>(m));
    m = pk_min_f16(m, dpp_u32<0x141>(m));
    if (lpg_log2 >= 4) m = pk_min_f16(m, dpp_u32<0x140>(m));
    if (lpg_log2 >= 5) m = pk_min_f16(m, static_cast<uint32_t>(__shfl_xor(static_cast<int>(m), 16)));
    if (lpg_log2 >= 6) m = pk_min_f16(m, static_cast<uint32_t>(__shfl_xor(static_cast<int>(m), 32)));
    const _Float16 hmin = __builtin_bit_cast(_Float16, static_cast<uint16_t>(m & 0xffffu));
    const _Float16 hneg = __builtin_bit_cast(_Float16, static_cast<uint16_t>(m >> 16));
    mn = plus_zero(static_cast<float>(hmin));
    mx = plus_zero(-static_cast<float>(hneg));
}

// Quantise the 8 elements of one piece to BITS-bit codes (exact small floats
// in r[]).  The contract is code = rint((x - mn) / scale) with a true binary32
// division.  The fast path takes q' = fma(x, inv, c) with inv = rcp(scale) (1 ulp)
// and c = -mn * inv rounded once; the fp16 element enters the FMA as it is
// (v_fma_mix_f32), so an element costs one instruction where conversion,
// subtraction and product cost three.  With q the exact quotient,
//   |q' - q| <= q * (2^-23 + 2^-24) + |c| * 2^-24 * (1 + 2^-22)
// (the reciprocal's ulp, the rounding of the sum, the rounding of c), so rint(q')
// can only differ from the defined code when q' lies within that distance of a
// half-integer.  A lane that sees |q' - rint(q')| >= 0.5 - (2^BITS * 2^-22 +
// |c| * 2^-23) redoes its piece with the exact division, which keeps every code
// bit-identical to the definition (a group far from zero against its range, e.g.
// values 1000..1001, has a large |c| and takes the exact path more often).
// CLAMP: the scale may fall short of range / levels (a scale rounded to binary16), so the quotient can
// pass the top level and is cut there; with an exact scale it cannot, and 8-bit codes saturate when
// they are packed.
template <int BITS, bool CLAMP>
__device__ __forceinline__ void quantise_piece(const h8_t& x, float mn, float scale, float r[8]) {
    constexpr float kLevels = static_cast<float>((1 << BITS) - 1);
    const float inv = (scale != 0.0f) ? __builtin_amdgcn_rcpf(scale) : 0.0f;
    const float c = -mn * inv;
    const float safe = 0.5f - __builtin_fmaf(__builtin_fabsf(c), 1.1920928955078125e-07f,
                                             static_cast<float>(1 << BITS) * 2.384185791015625e-07f);
    float e[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const float q = __builtin_fmaf(static_cast<float>(x[k]), inv, c);
        r[k] = __builtin_rintf(q);
        e[k] = __builtin_fabsf(q - r[k]);
        if constexpr (CLAMP) r[k] = __builtin_fminf(r[k], kLevels);
    }
    const float e01 = __builtin_fmaxf(__builtin_fmaxf(e[0], e[1]), e[2]);
    const float e02 = __builtin_fmaxf(__builtin_fmaxf(e[3], e[4]), e[5]);
    const float emax = __builtin_fmaxf(__builtin_fmaxf(e01, e02), __builtin_fmaxf(e[6], e[7]));
    if (!(emax < safe)) {
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const float d = static_cast<float>(x[k]) - mn;
            float c2 = __builtin_rintf(d / scale);
            c2 = __builtin_fminf(__builtin_fmaxf(c2, 0.0f), kLevels);
            r[k] = c2;
        }
    }
}

// One piece -> its codes (and, from the first lane of each group, scale and mn).
// HP: the parameters are kept in binary16 (format KV_FMT_F16_GROUPS_H): the scale is rounded to
// binary16 before the codes are computed, the minimum is one of the inputs and exact.
template <int BITS, bool HP>
__device__ __forceinline__ void compress_piece(const u4_t& raw, uint8_t* __restrict__ codes,
                                               void* __restrict__ scale_out,
                                               void* __restrict__ mn_out, int p, int lpg_log2,
                                               int lane) {
    constexpr float kLevels = static_cast<float>((1 << BITS) - 1);
    float mn, mx;
    group_min_max(raw, lpg_log2, mn, mx);
    // scale = (mx - mn) / levels, correctly rounded, without the division sequence: with y the binary32
    // nearest to 1 / levels and q0 = range * y, one correction step q0 + (range - levels * q0) * y (the
    // residual is exact in an FMA) gives the correctly rounded quotient; for levels 3, 15 and 255 this
    // holds for every binary32 numerator in [0, 2^17] (tests/scale_division_check.c goes through them one by one).
    constexpr float kInvLevels = 1.0f / kLevels;
    const float range = mx - mn;
    const float q0 = range * kInvLevels;
    float scale = __builtin_fmaf(__builtin_fmaf(-kLevels, q0, range), kInvLevels, q0);
    if constexpr (HP) {
        // two roundings, as the format defines them: the quotient to binary32, that value to binary16.  The
        // register barrier keeps the compiler from folding the last FMA and the conversion into one
        // instruction that rounds the exact sum to binary16 once (which differs for about one range in 6000).
        asm volatile("" : "+v"(scale));
        scale = static_cast<float>(static_cast<_Float16>(scale));
    }
    const h8_t x = __builtin_bit_cast(h8_t, raw);
    float r[8];
    quantise_piece<BITS, HP && BITS != 8>(x, mn, scale, r);
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
        u2_t w = {w0, w1};
        stream_store<true>(w, reinterpret_cast<u2_t*>(codes) + p);
    } else if constexpr (BITS == 4) {
        // four 4-bit codes = 16 bits: exact as a float sum
        const float lo = __builtin_fmaf(r[3], 4096.0f,
                         __builtin_fmaf(r[2], 256.0f, __builtin_fmaf(r[1], 16.0f, r[0])));
        const float hi = __builtin_fmaf(r[7], 4096.0f,
                         __builtin_fmaf(r[6], 256.0f, __builtin_fmaf(r[5], 16.0f, r[4])));
        stream_store<true>(static_cast<uint32_t>(lo) | (static_cast<uint32_t>(hi) << 16),
                     reinterpret_cast<uint32_t*>(codes) + p);
    } else {
        // eight 2-bit codes = 16 bits
        float acc = r[7];
#pragma unroll
        for (int k = 6; k >= 0; --k) acc = __builtin_fmaf(acc, 4.0f, r[k]);
        stream_store<true>(static_cast<uint16_t>(static_cast<uint32_t>(acc)),
                     reinterpret_cast<uint16_t*>(codes) + p);
    }
    if ((lane & ((1 << lpg_log2) - 1)) == 0) {
        if constexpr (HP) {
            static_cast<_Float16*>(scale_out)[p >> lpg_log2] = static_cast<_Float16>(scale);
            static_cast<_Float16*>(mn_out)[p >> lpg_log2] = static_cast<_Float16>(mn);
        } else {
            static_cast<float*>(scale_out)[p >> lpg_log2] = scale;
            static_cast<float*>(mn_out)[p >> lpg_log2] = mn;
        }
    }
}

// Grid (ceil(n_chunks * tpu / 4), slabs) or, record-major, (ceil(slabs * tpu / 4),
// n_chunks); block 256 threads = 4 wavefront tasks of PPL * 64 pieces each.
// chunk_list (may be NULL): the n_chunks chunk indices to compress instead of 0..n_chunks-1.
template <int PPL, bool HP>
__global__ __launch_bounds__(64 * kWavesPerBlock) void compress_kernel(const u4_t* __restrict__ kv,
                                                       const uint8_t* __restrict__ bits,
                                                       const uint64_t* __restrict__ off,
                                                       uint8_t* __restrict__ packed, QuantGeom g,
                                                       int32_t n_chunks,
                                                       const int32_t* __restrict__ chunk_list) {
    const int lane = threadIdx.x & 63;
    int chunk, slab, p0;
    if (!wave_task(g, n_chunks, PPL, chunk, slab, p0)) return;
    if (chunk_list) chunk = chunk_list[chunk];          // only the listed chunks (uniform: a scalar load)
    const u4_t* src = kv + (static_cast<uint64_t>(slab) * g.n_tokens +
                            static_cast<uint64_t>(chunk) * g.chunk_tokens) * g.row_pieces;
    u4_t raw[PPL];
#pragma unroll
    for (int u = 0; u < PPL; ++u) raw[u] = stream_load<true>(src + p0 + u * 64 + lane);
    int b = uniform_byte(bits, chunk);
    uint64_t rec = off[chunk];
    asm volatile("" : "+s"(b), "+s"(rec));               // both scalar loads issued, one wait
    uint8_t* base = packed + rec;
    if (b == 16) {
#pragma unroll
        for (int u = 0; u < PPL; ++u)
            stream_store<true>(raw[u], reinterpret_cast<u4_t*>(base) +
                                            static_cast<uint64_t>(slab) * g.pieces + p0 + u * 64 + lane);
        return;
    }
    const uint64_t code_bytes = static_cast<uint64_t>(g.pieces) * b;        // per unit
    const uint32_t groups = static_cast<uint32_t>(g.pieces) >> g.lpg_log2;  // per unit
    uint8_t* codes = base + slab * code_bytes;
    constexpr uint64_t kParam = HP ? 2 : 4;                               // bytes per stored parameter
    uint8_t* scale = base + g.slabs * code_bytes + static_cast<uint64_t>(slab) * groups * kParam;
    uint8_t* mn = scale + static_cast<uint64_t>(g.slabs) * groups * kParam;
    if (b == 8) {
#pragma unroll
        for (int u = 0; u < PPL; ++u)
            compress_piece<8, HP>(raw[u], codes, scale, mn, p0 + u * 64 + lane, g.lpg_log2, lane);
    } else if (b == 4) {
#pragma unroll
        for (int u = 0; u < PPL; ++u)
            compress_piece<4, HP>(raw[u], codes, scale, mn, p0 + u * 64 + lane, g.lpg_log2, lane);
    } else {
#pragma unroll
        for (int u = 0; u < PPL; ++u)
            compress_piece<2, HP>(raw[u], codes, scale, mn, p0 + u * 64 + lane, g.lpg_log2, lane);
    }
}

// ------------------------------------------------------------------ swap-in

// Codes of one piece as loaded from the record (8, 4 or 2 bytes).
template <int BITS>
__device__ __forceinline__ u2_t load_codes(const uint8_t* __restrict__ codes, int p) {
    u2_t w = {0u, 0u};
    if constexpr (BITS == 8) w = stream_load<true>(reinterpret_cast<const u2_t*>(codes) + p);
    else if constexpr (BITS == 4) w.x = stream_load<true>(reinterpret_cast<const uint32_t*>(codes) + p);
    else w.x = stream_load<true>(reinterpret_cast<const uint16_t*>(codes) + p);
    return w;
}

template <int BITS>
__device__ __forceinline__ u4_t dequantise_piece(u2_t w, float sc, float mn) {
    constexpr uint32_t kMask = (1u << BITS) - 1u;
    h8_t out;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        uint32_t c;
        if constexpr (BITS == 8) c = ((k < 4 ? w.x : w.y) >> ((k & 3) * 8)) & kMask;
        else c = (w.x >> (k * BITS)) & kMask;
        const float prod = static_cast<float>(c) * sc;   // rounded product, then rounded sum
        out[k] = static_cast<_Float16>(prod + mn);
    }
    return __builtin_bit_cast(u4_t, out);
}

template <int BITS, int PPL, bool HP>
__device__ __forceinline__ void swapin_pieces(const uint8_t* __restrict__ codes,
                                              const void* __restrict__ scale,
                                              const void* __restrict__ mn, u4_t* __restrict__ dst,
                                              int p0, int lane, int lpg_log2) {
    u2_t w[PPL];
    float sc[PPL], m[PPL];
#pragma unroll
    for (int u = 0; u < PPL; ++u) {
        const int p = p0 + u * 64 + lane;
        w[u] = load_codes<BITS>(codes, p);
        if constexpr (HP) {
            sc[u] = static_cast<float>(static_cast<const _Float16*>(scale)[p >> lpg_log2]);
            m[u] = static_cast<float>(static_cast<const _Float16*>(mn)[p >> lpg_log2]);
        } else {
            sc[u] = static_cast<const float*>(scale)[p >> lpg_log2];
            m[u] = static_cast<const float*>(mn)[p >> lpg_log2];
        }
    }
#pragma unroll
    for (int u = 0; u < PPL; ++u)
        stream_store<true>(dequantise_piece<BITS>(w[u], sc[u], m[u]),
                                         dst + p0 + u * 64 + lane);
}

// PPL * 64 pieces of one (selected record, slab) unit of the Load primitive.
template <int PPL, bool HP>
__device__ __forceinline__ void swapin_task(const uint8_t* __restrict__ base, int b, int slab,
                                            u4_t* __restrict__ dst, const QuantGeom& g, int p0,
                                            int lane) {
    if (b == 16) {
        const u4_t* src = reinterpret_cast<const u4_t*>(base) + static_cast<uint64_t>(slab) * g.pieces;
        u4_t raw[PPL];
#pragma unroll
        for (int u = 0; u < PPL; ++u) raw[u] = stream_load<true>(src + p0 + u * 64 + lane);
#pragma unroll
        for (int u = 0; u < PPL; ++u) stream_store<true>(raw[u], dst + p0 + u * 64 + lane);
        return;
    }
    const uint64_t code_bytes = static_cast<uint64_t>(g.pieces) * b;
    const uint32_t groups = static_cast<uint32_t>(g.pieces) >> g.lpg_log2;
    const uint8_t* codes = base + slab * code_bytes;
    constexpr uint64_t kParam = HP ? 2 : 4;                               // bytes per stored parameter
    const uint8_t* scale = base + g.slabs * code_bytes + static_cast<uint64_t>(slab) * groups * kParam;
    const uint8_t* mn = scale + static_cast<uint64_t>(g.slabs) * groups * kParam;
    if (b == 8) swapin_pieces<8, PPL, HP>(codes, scale, mn, dst, p0, lane, g.lpg_log2);
    else if (b == 4) swapin_pieces<4, PPL, HP>(codes, scale, mn, dst, p0, lane, g.lpg_log2);
    else swapin_pieces<2, PPL, HP>(codes, scale, mn, dst, p0, lane, g.lpg_log2);
}

// One-dimensional grid of g.groups * g.slab_count workgroups of up to kLoadWavesMax wavefronts in
// strip order (strip_task_at); gather lists in device memory.
template <int PPL, bool HP>
__global__ __launch_bounds__(64 * kLoadWavesMax) void swapin_kernel(const uint8_t* __restrict__ packed,
                                                     const uint64_t* __restrict__ src_off,
                                                     const int32_t* __restrict__ dst_tok,
                                                     const uint8_t* __restrict__ sel_bits,
                                                     u4_t* __restrict__ kv_out, QuantGeom g,
                                                     int32_t n_sel) {
    const int lane = threadIdx.x & 63;
    int j, slab, p0;
    if (!strip_task_at(g, n_sel, PPL, blockIdx.x, static_cast<int>(blockDim.x >> 6), j, slab, p0)) return;
    const GatherEntry e = gather_entry<true, false>(src_off, dst_tok, sel_bits, j);
    u4_t* dst = kv_out + (static_cast<uint64_t>(slab) * g.n_tokens +
                          static_cast<uint64_t>(e.tok)) * g.row_pieces;
    swapin_task<PPL, HP>(packed + e.src, e.b, slab, dst, g, p0, lane);
}

// The same Load for a record pool that stays in pinned host memory.  A wavefront of this
// launch spends its time waiting for the host link, and a few hundred of them keep the link
// full (measured on MI355X: 32 workgroups reach 60 % of the link's rate, 64 reach 96 %, 128 and
// more all of it); so the launch is a small one-dimensional grid whose workgroups walk the task
// grid (gx x gy workgroups of swapin_kernel) in strides, and most of the compute units' wavefront
// slots stay free for kernels of other streams.
constexpr uint32_t kLinkBlocks = 128;

template <int PPL, bool HP>
__global__ __launch_bounds__(64 * kLoadWavesMax) void swapin_link_kernel(const uint8_t* __restrict__ packed,
                                                          const uint64_t* __restrict__ src_off,
                                                          const int32_t* __restrict__ dst_tok,
                                                          const uint8_t* __restrict__ sel_bits,
                                                          u4_t* __restrict__ kv_out, QuantGeom g,
                                                          int32_t n_sel, uint32_t total) {
    const int lane = threadIdx.x & 63;
    for (uint32_t w = blockIdx.x; w < total; w += gridDim.x) {
        int j, slab, p0;
        if (!strip_task_at(g, n_sel, PPL, w, static_cast<int>(blockDim.x >> 6), j, slab, p0)) continue;
        const GatherEntry e = gather_entry<false>(src_off, dst_tok, sel_bits, j);
        u4_t* dst = kv_out + (static_cast<uint64_t>(slab) * g.n_tokens +
                              static_cast<uint64_t>(e.tok)) * g.row_pieces;
        swapin_task<PPL, HP>(packed + e.src, e.b, slab, dst, g, p0, lane);
    }
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

template <int PPL, bool HP>
__global__ __launch_bounds__(64 * kLoadWavesMax) void swapin_batch_kernel(const uint8_t* __restrict__ staged,
                                                           SwapinBatch list,
                                                           u4_t* __restrict__ kv_out, QuantGeom g) {
    const int lane = threadIdx.x & 63;
    int j, slab, p0;
    if (!strip_task_at(g, list.n, PPL, blockIdx.x, static_cast<int>(blockDim.x >> 6), j, slab, p0)) return;
    u4_t* dst = kv_out + (static_cast<uint64_t>(slab) * g.n_tokens +
                          static_cast<uint64_t>(list.dst_tok[j])) * g.row_pieces;
    swapin_task<PPL, HP>(staged + list.src_off[j], list.bits[j], slab, dst, g, p0, lane);
}

}  // namespace kvs
