// gfx950 kernels for the recompute of interleaved chunks (Sec. 3.3, "Making
// interleaved chunks recomputable"): the tokens of the missing chunks go through
// one Llama-style block; q and k are encoded with the tokens' GLOBAL positions,
// the recomputed K/V are inserted between the resident K/V of the cache, and the
// recomputed queries attend to the recovered K/V under a causal mask by global
// position.  The dense projections are library GEMMs; everything else is here.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kv_lane_ops.hpp"

namespace kvs {

typedef _Float16 rv8h_t __attribute__((ext_vector_type(8)));
typedef _Float16 rv4h_t __attribute__((ext_vector_type(4)));
typedef short rv4s_t __attribute__((ext_vector_type(4)));
typedef float rv16f_t __attribute__((ext_vector_type(16)));
typedef float rv4f_t __attribute__((ext_vector_type(4)));
typedef unsigned int ru4_t __attribute__((ext_vector_type(4)));

// Global position of recomputed token m: chunks of T tokens, chunk_idx ascending.
__device__ __forceinline__ int global_position(const int32_t* __restrict__ chunk_idx, int T, int m) {
    return chunk_idx[m / T] * T + m % T;
}

// xn[m][:] = x[m][:] / sqrt(mean(x[m][:]^2) + eps) * w[:]      (fp16 in/out, binary32 inside)
// One wavefront per row; d_model % 8 == 0.
__global__ __launch_bounds__(256) void rmsnorm_kernel(const _Float16* __restrict__ x,
                                                      const _Float16* __restrict__ w,
                                                      _Float16* __restrict__ xn, int32_t M,
                                                      int32_t d_model, float eps) {
    const int lane = threadIdx.x & 63;
    const int m = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (m >= M) return;
    const rv8h_t* row = reinterpret_cast<const rv8h_t*>(x + static_cast<int64_t>(m) * d_model);
    const int pieces = d_model / 8;
    float ss = 0.0f;
    for (int p = lane; p < pieces; p += 64) {
        const rv8h_t v = row[p];
#pragma unroll
        for (int k = 0; k < 8; ++k) ss += static_cast<float>(v[k]) * static_cast<float>(v[k]);
    }
#pragma unroll
    for (int o = 16; o >= 1; o >>= 1) ss += __shfl_xor(ss, o);
    ss = xhalf_sum(ss);
    const float r = 1.0f / sqrtf(ss / static_cast<float>(d_model) + eps);
    const rv8h_t* wp = reinterpret_cast<const rv8h_t*>(w);
    rv8h_t* out = reinterpret_cast<rv8h_t*>(xn + static_cast<int64_t>(m) * d_model);
    for (int p = lane; p < pieces; p += 64) {
        const rv8h_t v = row[p], g = wp[p];
        rv8h_t o;
#pragma unroll
        for (int k = 0; k < 8; ++k)
            o[k] = static_cast<_Float16>(static_cast<float>(v[k]) * r * static_cast<float>(g[k]));
        out[p] = o;
    }
}

// The same norm over a row that a projection left as `splits` binary32 partial products
// [splits][M][d_model]:  x[m][:] = fp16(part[0][m][:] + part[1][m][:] + ... + resid[m][:])  (split order,
// rounded once) is stored - it is the next residual - and normed.  One workgroup per row: with few rows
// the partial products are most of what a layer reads here, and a wavefront per row would leave the
// memory system idle.
__global__ __launch_bounds__(256) void rmsnorm_sum_kernel(const float* __restrict__ part, int32_t splits,
                                                          const _Float16* __restrict__ resid,
                                                          _Float16* __restrict__ x,
                                                          const _Float16* __restrict__ w,
                                                          _Float16* __restrict__ xn, int32_t M,
                                                          int32_t d_model, float eps) {
    __shared__ float wave_ss[4];
    const int m = blockIdx.x;
    const int pieces = d_model / 8;
    const int64_t plane4 = static_cast<int64_t>(M) * d_model / 4;
    const rv4f_t* src = reinterpret_cast<const rv4f_t*>(part) + static_cast<int64_t>(m) * d_model / 4;
    const rv8h_t* res = reinterpret_cast<const rv8h_t*>(resid + static_cast<int64_t>(m) * d_model);
    rv8h_t* row = reinterpret_cast<rv8h_t*>(x + static_cast<int64_t>(m) * d_model);
    float ss = 0.0f;
    for (int p = threadIdx.x; p < pieces; p += 256) {
        rv4f_t lo = src[2 * p], hi = src[2 * p + 1];
#pragma unroll 4
        for (int sp = 1; sp < splits; ++sp) {
            lo += src[sp * plane4 + 2 * p];
            hi += src[sp * plane4 + 2 * p + 1];
        }
        const rv8h_t r = res[p];
        rv8h_t v;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            v[k] = static_cast<_Float16>(lo[k] + static_cast<float>(r[k]));
            v[k + 4] = static_cast<_Float16>(hi[k] + static_cast<float>(r[k + 4]));
        }
        row[p] = v;                                  // read again below by this same thread
#pragma unroll
        for (int k = 0; k < 8; ++k) ss += static_cast<float>(v[k]) * static_cast<float>(v[k]);
    }
#pragma unroll
    for (int o = 16; o >= 1; o >>= 1) ss += __shfl_xor(ss, o);
    ss = xhalf_sum(ss);
    if ((threadIdx.x & 63) == 0) wave_ss[threadIdx.x >> 6] = ss;
    __syncthreads();
    ss = (wave_ss[0] + wave_ss[1]) + (wave_ss[2] + wave_ss[3]);
    const float r = 1.0f / sqrtf(ss / static_cast<float>(d_model) + eps);
    const rv8h_t* wp = reinterpret_cast<const rv8h_t*>(w);
    rv8h_t* out = reinterpret_cast<rv8h_t*>(xn + static_cast<int64_t>(m) * d_model);
    for (int p = threadIdx.x; p < pieces; p += 256) {
        const rv8h_t v = row[p], g = wp[p];
        rv8h_t o;
#pragma unroll
        for (int k = 0; k < 8; ++k)
            o[k] = static_cast<_Float16>(static_cast<float>(v[k]) * r * static_cast<float>(g[k]));
        out[p] = o;
    }
}

// Rotary angles: theta[i] = base^(-2i/D) in double, computed on the host.
struct RopeTable {
    double theta[128];      // head_dim / 2 <= 128
};

// Four workgroups per recomputed token m at global position p (grid (M, 4): q, k and the two halves of v;
// with some hundred tokens a workgroup per token leaves half the CUs idle and walks its row in eight
// dependent trips to memory):
//   q16[m][h][:]            = rope(q32[m][h][:], p)                       (fp16)
//   K plane [g][p][:]       = rope(k32[m][g][:], p)   V plane [g][p][:] = v32[m][g][:]   (fp16 cache)
// The pair (i, i + D/2) is rotated by p * theta[i]; sine and cosine are taken in
// double (positions reach tens of thousands of radians).  q32, k32 and v32 may be `splits` partial
// products each ([splits][M][heads * D], M = the grid size), which are added in split order as they
// are read.
__global__ __launch_bounds__(256) void rope_scatter_kernel(const float* __restrict__ q32,
                                                           const float* __restrict__ k32,
                                                           const float* __restrict__ v32,
                                                           const int32_t* __restrict__ chunk_idx,
                                                           _Float16* __restrict__ q16,
                                                           _Float16* __restrict__ k_plane,
                                                           _Float16* __restrict__ v_plane,
                                                           RopeTable tab, int32_t T, int32_t N,
                                                           int32_t Hq, int32_t Hkv, int32_t D, int32_t splits) {
    __shared__ __attribute__((aligned(16))) float cs[2][128];
    const int64_t plane_q = static_cast<int64_t>(gridDim.x) * Hq * D, plane_kv = static_cast<int64_t>(gridDim.x) * Hkv * D;
    // four adjacent elements, the partial products added in split order
    auto sum4 = [&](const float* at, int64_t plane) {
        rv4f_t a = *reinterpret_cast<const rv4f_t*>(at);
#pragma unroll 4
        for (int sp = 1; sp < splits; ++sp) a += *reinterpret_cast<const rv4f_t*>(at + sp * plane);
        return a;
    };
    auto to_half4 = [](rv4f_t a) {
        return rv4h_t{static_cast<_Float16>(a[0]), static_cast<_Float16>(a[1]), static_cast<_Float16>(a[2]),
                      static_cast<_Float16>(a[3])};
    };
    const int m = blockIdx.x;
    const int part = blockIdx.y;            // 0: q, 1: k, 2 and 3: the halves of v (uniform per workgroup)
    const int p = global_position(chunk_idx, T, m);
    const int half = D / 2, half4 = D / 8;
    if (part >= 2) {
        const float* vrow = v32 + static_cast<int64_t>(m) * Hkv * D;
        const int n4 = Hkv * D / 4, mid = n4 / 2;
        for (int e = (part == 2 ? 0 : mid) + threadIdx.x; e < (part == 2 ? mid : n4); e += blockDim.x) {
            const int g = e / (D / 4), d = (e % (D / 4)) * 4;
            *reinterpret_cast<rv4h_t*>(v_plane + (static_cast<int64_t>(g) * N + p) * D + d) = to_half4(sum4(vrow + e * 4, plane_kv));
        }
        return;
    }
    for (int i = threadIdx.x; i < half; i += blockDim.x) {
        double s, c;
        sincos(static_cast<double>(p) * tab.theta[i], &s, &c);
        cs[0][i] = static_cast<float>(c);
        cs[1][i] = static_cast<float>(s);
    }
    __syncthreads();
    if (part == 0) {
        const float* qrow = q32 + static_cast<int64_t>(m) * Hq * D;
        _Float16* qout = q16 + static_cast<int64_t>(m) * Hq * D;
        for (int e = threadIdx.x; e < Hq * half4; e += blockDim.x) {
            const int h = e / half4, i = (e % half4) * 4;
            const rv4f_t a = sum4(qrow + h * D + i, plane_q), b = sum4(qrow + h * D + i + half, plane_q);
            const rv4f_t c = *reinterpret_cast<const rv4f_t*>(&cs[0][i]), s = *reinterpret_cast<const rv4f_t*>(&cs[1][i]);
            *reinterpret_cast<rv4h_t*>(qout + h * D + i) = to_half4(a * c - b * s);
            *reinterpret_cast<rv4h_t*>(qout + h * D + i + half) = to_half4(b * c + a * s);
        }
        return;
    }
    const float* krow = k32 + static_cast<int64_t>(m) * Hkv * D;
    for (int e = threadIdx.x; e < Hkv * half4; e += blockDim.x) {
        const int g = e / half4, i = (e % half4) * 4;
        const rv4f_t a = sum4(krow + g * D + i, plane_kv), b = sum4(krow + g * D + i + half, plane_kv);
        const rv4f_t c = *reinterpret_cast<const rv4f_t*>(&cs[0][i]), s = *reinterpret_cast<const rv4f_t*>(&cs[1][i]);
        _Float16* dst = k_plane + (static_cast<int64_t>(g) * N + p) * D;
        *reinterpret_cast<rv4h_t*>(dst + i) = to_half4(a * c - b * s);
        *reinterpret_cast<rv4h_t*>(dst + i + half) = to_half4(b * c + a * s);
    }
}

// act = silu(gate) * up, elementwise, 8 elements per thread (n % 8 == 0).
// (act may be gate: each thread reads its elements before it writes them)
// With `part_gate` the two operands are first made from projections left as `splits` binary32 partial
// products of n8 * 8 elements each: gate = fp16(sum in split order), up likewise.
__global__ __launch_bounds__(256) void silu_mul_kernel(const _Float16* gate, const _Float16* up,
                                                       _Float16* act, int64_t n8,
                                                       const float* __restrict__ part_gate,
                                                       const float* __restrict__ part_up, int32_t splits) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i >= n8) return;
    rv8h_t g, u;
    if (part_gate) {
        const rv4f_t* pg = reinterpret_cast<const rv4f_t*>(part_gate);
        const rv4f_t* pu = reinterpret_cast<const rv4f_t*>(part_up);
        rv4f_t g0 = pg[2 * i], g1 = pg[2 * i + 1], u0 = pu[2 * i], u1 = pu[2 * i + 1];
        for (int sp = 1; sp < splits; ++sp) {
            const int64_t at = (sp * n8 + i) * 2;
            g0 += pg[at]; g1 += pg[at + 1];
            u0 += pu[at]; u1 += pu[at + 1];
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            g[k] = static_cast<_Float16>(g0[k]); g[k + 4] = static_cast<_Float16>(g1[k]);
            u[k] = static_cast<_Float16>(u0[k]); u[k + 4] = static_cast<_Float16>(u1[k]);
        }
    } else {
        g = reinterpret_cast<const rv8h_t*>(gate)[i];
        u = reinterpret_cast<const rv8h_t*>(up)[i];
    }
    rv8h_t o;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const float x = static_cast<float>(g[k]);
        o[k] = static_cast<_Float16>(x / (1.0f + __expf(-x)) * static_cast<float>(u[k]));
    }
    reinterpret_cast<rv8h_t*>(act)[i] = o;
}

// Stand-in operands for timing GEMM kernels: every 16-bit half is a binary16 of magnitude
// [0.5, 1) with a hashed mantissa and sign (timings with constant operands mislead: they draw
// less power, and the clock, hence the ranking of kernels, follows the power).
__global__ __launch_bounds__(256) void fill_noise_kernel(uint32_t* __restrict__ words, int64_t n) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i >= n) return;
    uint32_t h = static_cast<uint32_t>(i) * 2654435761u + 0x9e3779b9u;
    h ^= h >> 15; h *= 0x85ebca6bu; h ^= h >> 13; h *= 0xc2b2ae35u; h ^= h >> 16;
    words[i] = (h & 0x83ff83ffu) | 0x38003800u;
}

struct AttnGeom {
    int32_t M;        // recomputed tokens
    int32_t T;        // chunk tokens
    int32_t N;        // cache tokens
    int32_t Hq, Hkv;
    int32_t n_rb;     // ceil(M / 32): blocks of 32 query rows
    int32_t pairs;    // (Hq / Hkv) * n_rb: (row block, query head) pairs per kv head
    float scale_log2e;
};

// Causal attention of the recomputed queries over the recovered K/V of one layer.
// A wavefront owns one (block of 32 query rows, query head) pair: S^T = K_tile Q^T
// with mfma_f32_32x32x16_f16 (a lane owns one query row and 16 of the tile's 32
// tokens), online softmax per row, O^T += V_tile^T P^T with the probabilities
// rounded to fp16 as the B operand straight from the registers (the contraction
// index is permuted the same way on both operands).  The eight wavefronts of a
// workgroup take eight consecutive pairs of ONE kv head, so K and V tiles are
// fetched once per workgroup (coalesced 16-byte loads, two tiles ahead) and shared
// through LDS: K with its row pieces permuted by the row number, V in cache order and
// read through the LDS transpose read.  Tokens after a row's global position
// are masked; a wavefront skips the tiles that lie entirely behind its last row,
// and the output accumulators are rescaled only when some row's maximum moved.
constexpr int kAttnWaves = 8;
constexpr int kMaxSplits = 16;     // workgroups that may share the key range of a row block

//
// SPLIT: with few recomputed rows there are too few workgroups to fill the chip and each walks
// the whole key range alone.  The key tiles are then divided among gridDim.z workgroups per
// (pairs, kv head); each writes the unnormalised output, running maximum and denominator of its
// share (part_o [split][row][head][D], part_ml [split][row][head][2], binary32) and
// attention_combine_kernel merges the shares in a fixed order.
template <int D, bool SPLIT>
__global__ __launch_bounds__(64 * kAttnWaves) void recompute_attention_kernel(
    const _Float16* __restrict__ q16, const _Float16* __restrict__ k_plane,
    const _Float16* __restrict__ v_plane, const int32_t* __restrict__ chunk_idx,
    _Float16* __restrict__ out, AttnGeom g, float* __restrict__ part_o, float* __restrict__ part_ml,
    int tiles_per_split) {
    constexpr int KS = D / 16;
    constexpr int DB = D / 32;                      // 32-wide blocks of the head dimension
    constexpr int kRowPieces = D / 8;
    constexpr int kThreads = 64 * kAttnWaves;
    constexpr int kTilePieces = 32 * kRowPieces;    // 16-byte pieces of a K (or V) tile
    constexpr int kPer = (kTilePieces + kThreads - 1) / kThreads;
    __shared__ ru4_t ktile[2][32 * kRowPieces];
    // V stays in cache order, [token][channel] with 32 bytes of padding per token row; the
    // operand of O^T += V^T P^T (a channel per lane, tokens along the contraction) is taken with
    // the LDS transpose read (ds_read_b64_tr_b16): the 16 lanes of a group hand in the sixteen
    // 8-byte pieces of a 4-token x 16-channel block, row by row, and lane i receives the four
    // tokens of channel i.  The padding puts the four token rows of a block on different banks.
    constexpr int kVPitch = D + 16;
    __shared__ __align__(16) _Float16 vt[2][32 * kVPitch];
    auto swz = [](int r) __attribute__((always_inline)) { return D == 64 ? (r >> 1) & 7 : r & 15; };

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int lrow = lane & 31, half = lane >> 5;
    // Workgroups are handed to the 8 XCDs in turn (linear id modulo 8), each with an L2 of its
    // own: the workgroups of one kv head are placed on one XCD, so that its K/V planes are
    // fetched into one L2 only.  Needs n_kv_heads % 8 == 0, otherwise the plain order is kept.
    int kvh = blockIdx.y, bxi = blockIdx.x;
    if (!SPLIT && g.Hkv % 8 == 0) {
        const int lin = blockIdx.y * gridDim.x + blockIdx.x;
        const int per_xcd = lin >> 3;                       // position among this XCD's workgroups
        kvh = (lin & 7) + 8 * (per_xcd / static_cast<int>(gridDim.x));
        bxi = per_xcd % static_cast<int>(gridDim.x);
    }
    const int per = g.Hq / g.Hkv;
    // workgroups with the longest key ranges are dispatched first
    const int bx = static_cast<int>(gridDim.x) - 1 - bxi;
    const int pair = bx * kAttnWaves + wave;
    const bool valid = pair < g.pairs;
    const int head = kvh * per + (valid ? pair % per : 0);
    const int rb = valid ? pair / per : 0;
    const int m = rb * 32 + lrow;
    const bool ok = valid && m < g.M;
    const int pos = ok ? global_position(chunk_idx, g.T, m) : -1;
    // rows ascend in position: first and last row of this wavefront, last row of the workgroup
    const int min_pos = valid ? global_position(chunk_idx, g.T, rb * 32) : -1;
    const int max_pos = valid ? global_position(chunk_idx, g.T, min(rb * 32 + 31, g.M - 1)) : -1;
    const int rb_hi = min(bx * kAttnWaves + kAttnWaves - 1, g.pairs - 1) / per;
    const int wg_max_pos = global_position(chunk_idx, g.T, min(rb_hi * 32 + 31, g.M - 1));
    // key tiles [t_first, n_tiles) of this workgroup
    const int t_first = SPLIT ? static_cast<int>(blockIdx.z) * tiles_per_split : 0;
    const int n_tiles = SPLIT ? min(wg_max_pos / 32 + 1, t_first + tiles_per_split) : wg_max_pos / 32 + 1;

    rv8h_t qreg[KS];
    {
        const _Float16* qp = q16 + (static_cast<int64_t>(ok ? m : 0) * g.Hq + head) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            rv8h_t v = {0, 0, 0, 0, 0, 0, 0, 0};
            if (ok) v = *reinterpret_cast<const rv8h_t*>(qp + ks * 16);
            qreg[ks] = v;
        }
    }
    const ru4_t* kbase = reinterpret_cast<const ru4_t*>(k_plane + static_cast<int64_t>(kvh) * g.N * D);
    const ru4_t* vbase = reinterpret_cast<const ru4_t*>(v_plane + static_cast<int64_t>(kvh) * g.N * D);
    // tiles in flight: set 0 holds even tiles, set 1 odd ones (loads are issued two tiles ahead)
    ru4_t kst[2][kPer], vst[2][kPer];
    auto fetch = [&](int set, int t) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const int p = min(i * kThreads + tid, kTilePieces - 1);       // surplus threads repeat the last piece
            const int token = min(t * 32 + p / kRowPieces, g.N - 1);      // rows past the cache are masked anyway
            const int64_t src = static_cast<int64_t>(token) * kRowPieces + p % kRowPieces;
            kst[set][i] = kbase[src];
            vst[set][i] = vbase[src];
        }
    };
    auto park = [&](int set, int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const int p = min(i * kThreads + tid, kTilePieces - 1);
            const int r = p / kRowPieces, c = p % kRowPieces;
            ktile[buf][r * kRowPieces + (c ^ swz(r))] = kst[set][i];
            *reinterpret_cast<ru4_t*>(&vt[buf][r * kVPitch + c * 8]) = vst[set][i];
        }
    };

    rv16f_t o_acc[DB];
#pragma unroll
    for (int b = 0; b < DB; ++b) o_acc[b] = rv16f_t{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    float m_run = -INFINITY, l_run = 0.0f;

    // one tile: the arithmetic on LDS buffer `buf` (tile t), then tile t + 1 (fetched two steps ago
    // into the other register set) goes to the other buffer and its set fetches tile t + 3
    auto step = [&](int t, int buf) __attribute__((always_inline)) {
        if (t * 32 <= max_pos) {            // wave-uniform
            rv8h_t kreg[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                kreg[ks] = __builtin_bit_cast(rv8h_t, ktile[buf][lrow * kRowPieces + ((2 * ks + half) ^ swz(lrow))]);
            rv16f_t acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(kreg[ks], qreg[ks], acc, 0, 0, 0);
            // acc[v]: token t*32 + 8*(v/4) + 4*half + v%4 against this lane's query row
            // maxima on the raw logits (the scale is positive), the scale folded into the exponent
            const bool masked = t * 32 + 31 > min_pos;     // wave-uniform
            float mloc = -INFINITY;
            if (masked) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int tk = t * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                    if (tk > pos) acc[v] = -INFINITY;
                }
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) mloc = fmaxf(mloc, acc[v]);
            const float m_new = fmaxf(m_run, xhalf_max(mloc) * g.scale_log2e);
            const float m_safe = (m_new == -INFINITY) ? 0.0f : m_new;
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);
            float psum = 0.0f;
            rv8h_t pb[2];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(acc[v], g.scale_log2e, -m_safe));
                psum += pv;
                pb[v / 8][v % 8] = static_cast<_Float16>(pv);
            }
            l_run = l_run * alpha + xhalf_sum(psum);
            const bool moved = m_new != m_run;
            m_run = m_new;
            if (__any(moved)) {             // wave-uniform: some row's maximum moved
#pragma unroll
                for (int b = 0; b < DB; ++b)
#pragma unroll
                    for (int v = 0; v < 16; ++v) o_acc[b][v] *= alpha;
            }
            // contraction slot (half, e) of step st holds token 16*st + 4*half + e (e < 4) or
            // 16*st + 8 + 4*half + e - 4: the order of acc[8*st .. 8*st+7] on the P side
#pragma unroll
            for (int b = 0; b < DB; ++b) {
                // this lane's piece of the block of its 16-lane group: token row (lane % 16) / 4, channels
                // 32 b + 16 (group % 2) + 4 (lane % 4) ..; the read returns channel 32 b + lane % 32
                const _Float16* vblk = &vt[buf][((lane & 15) >> 2) * kVPitch + 32 * b + 16 * ((lane >> 4) & 1) + 4 * (lane & 3)];
#pragma unroll
                for (int st = 0; st < 2; ++st) {
                    const rv4s_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (__attribute__((address_space(3))) rv4s_t*)(vblk + (16 * st + 4 * half) * kVPitch));
                    const rv4s_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (__attribute__((address_space(3))) rv4s_t*)(vblk + (16 * st + 8 + 4 * half) * kVPitch));
                    const rv4h_t lo_h = __builtin_bit_cast(rv4h_t, lo), hi_h = __builtin_bit_cast(rv4h_t, hi);
                    const rv8h_t a = {lo_h[0], lo_h[1], lo_h[2], lo_h[3], hi_h[0], hi_h[1], hi_h[2], hi_h[3]};
                    o_acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, pb[st], o_acc[b], 0, 0, 0);
                }
            }
        }
        if (t + 1 < n_tiles) park(buf ^ 1, buf ^ 1);
        if (t + 3 < n_tiles) fetch(buf ^ 1, t + 3);
        __syncthreads();
    };
    if (t_first < n_tiles) {            // uniform per workgroup
        fetch(0, t_first);
        park(0, 0);
        fetch(1, min(t_first + 1, n_tiles - 1));
        fetch(0, min(t_first + 2, n_tiles - 1));
        __syncthreads();
        for (int t = t_first; t < n_tiles; t += 2) {
            step(t, 0);
            if (t + 1 < n_tiles) step(t + 1, 1);
        }
    }
    if constexpr (SPLIT) {
        if (ok) {
            // the share of this workgroup: an empty one has m = -inf, l = 0 and zeros
            const int64_t row = (static_cast<int64_t>(blockIdx.z) * g.M + m) * g.Hq + head;
            if (half == 0) {
                part_ml[row * 2] = m_run;
                part_ml[row * 2 + 1] = l_run;
            }
            float* dst = part_o + row * D;
#pragma unroll
            for (int b = 0; b < DB; ++b)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const rv4f_t o4 = {o_acc[b][4 * j], o_acc[b][4 * j + 1], o_acc[b][4 * j + 2], o_acc[b][4 * j + 3]};
                    *reinterpret_cast<rv4f_t*>(dst + 32 * b + 8 * j + 4 * half) = o4;
                }
        }
        return;
    }
    if (ok) {
        // o_acc[b][v]: head dimension 32*b + 8*(v/4) + 4*half + v%4 of this lane's query row
        const float inv = 1.0f / l_run;         // a row sees at least its own token
        _Float16* dst = out + (static_cast<int64_t>(m) * g.Hq + head) * D;
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                rv4h_t o4;
#pragma unroll
                for (int k = 0; k < 4; ++k) o4[k] = static_cast<_Float16>(o_acc[b][4 * j + k] * inv);
                *reinterpret_cast<rv4h_t*>(dst + 32 * b + 8 * j + 4 * half) = o4;
            }
    }
}

// Merges the shares of a split attention: out[row][head][:] = sum_s w_s o_s / sum_s w_s l_s with
// w_s = 2^(m_s - max_s m_s), shares taken in ascending order.  One thread per 4 channels.
template <int D>
__global__ __launch_bounds__(256) void attention_combine_kernel(const float* __restrict__ part_o,
                                                                const float* __restrict__ part_ml,
                                                                _Float16* __restrict__ out, int64_t rows,
                                                                int n_splits) {
    constexpr int kQuads = D / 4;
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i >= rows * kQuads) return;
    const int64_t row = i / kQuads;
    const int quad = static_cast<int>(i % kQuads);
    // all loads of a pass are issued before its arithmetic: up to kMaxSplits shares, a clamped
    // index for the surplus slots (their weight is forced to zero)
    float m_s[kMaxSplits], l_s[kMaxSplits];
#pragma unroll
    for (int s = 0; s < kMaxSplits; ++s) {
        const int sc = s < n_splits ? s : n_splits - 1;
        const float2 ml = *reinterpret_cast<const float2*>(part_ml + (sc * rows + row) * 2);
        m_s[s] = s < n_splits ? ml.x : -INFINITY;
        l_s[s] = ml.y;
    }
    float m_all = -INFINITY;
#pragma unroll
    for (int s = 0; s < kMaxSplits; ++s) m_all = fmaxf(m_all, m_s[s]);
    float l_all = 0.0f;
    rv4f_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int s0 = 0; s0 < kMaxSplits; s0 += 4) {
        if (s0 >= n_splits) break;
        rv4f_t o[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int sc = s0 + k < n_splits ? s0 + k : n_splits - 1;
            o[k] = *reinterpret_cast<const rv4f_t*>(part_o + (sc * rows + row) * D + quad * 4);
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            // an empty share (m = -inf) and a surplus slot weigh nothing
            const float w = m_s[s0 + k] == -INFINITY ? 0.0f : __builtin_amdgcn_exp2f(m_s[s0 + k] - m_all);
            l_all += w * l_s[s0 + k];
            acc += o[k] * w;
        }
    }
    const float inv = 1.0f / l_all;                     // a row sees at least its own token
    rv4h_t o4;
#pragma unroll
    for (int k = 0; k < 4; ++k) o4[k] = static_cast<_Float16>(acc[k] * inv);
    *reinterpret_cast<rv4h_t*>(out + row * D + quad * 4) = o4;
}

}  // namespace kvs
