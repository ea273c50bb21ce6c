// gfx950 kernels for the information density of chunks (Sec. 3.2, Eq. 1):
// A = softmax(mask(Q K^T / sqrt(D))) per (layer, head), column mass per chunk,
// mean over layers and heads.
//
// K is read once.  Kernel 1 sweeps K in tiles of 32 tokens; one wavefront holds
// one or two blocks of 32 query rows in registers and produces, per tile, the
// 32x32 logit block with MFMA (K tile as the A operand, so a lane owns one query
// row and 16 of the tile's tokens, which makes the row reductions mostly
// in-lane).  Because the softmax denominator of a row is only known after the
// whole sweep, each tile is exponentiated against its own row maximum and the
// partial results are written out: per (row, tile) the local maximum and sum,
// per (row, sub-block of min(T,32) tokens) the weighted sum.  Kernel 2 combines
// them per (layer, head) into chunk masses; kernel 3 averages over layers and
// heads.  All reductions run in a fixed order: results are deterministic.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kvs {

typedef _Float16 v8h_t __attribute__((ext_vector_type(8)));
typedef float v16f_t __attribute__((ext_vector_type(16)));

struct ScoreGeom {
    int32_t L, Hkv, Hq, N, R;
    int32_t T;            // chunk tokens (power of two >= 8)
    int32_t sb_tokens;    // min(T, 32): tokens per stored sub-block
    int32_t n_tiles;      // N / 32
    int32_t RB;           // ceil(R / 32): row blocks per head
    int32_t rows_p;       // RB * 32
    int32_t n_rb;         // (Hq / Hkv) * RB: row blocks per kv head
    int32_t n_rg;         // row groups (each NRBW row blocks) per kv head
    int32_t rg_per_wg;    // row groups handled by one workgroup (1..4)
    int32_t tile_par;     // tiles processed in parallel by one workgroup (4 / rg_per_wg)
    int32_t tiles_per_wg; // consecutive tiles per workgroup
    int32_t norm_mode;    // 0: divide each column by its number of visible rows; 1: plain sums
    float   scale_log2e;  // log2(e) / sqrt(D)
};

// Workspace planes (floats): m_tile [L*Hq][n_tiles][rows_p], l_tile same, e_sub [L*Hq][n_sb][rows_p].
struct ScoreWs {
    float* m_tile;
    float* l_tile;
    float* e_sub;
};

__device__ __forceinline__ float xhalf_f(float v) { return __shfl_xor(v, 32); }

template <int D, int NRBW>
__global__ __launch_bounds__(256) void score_tiles_kernel(const _Float16* __restrict__ q,
                                                          const _Float16* __restrict__ kv,
                                                          ScoreGeom g, ScoreWs ws) {
    constexpr int KS = D / 16;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int lrow = lane & 31, half = lane >> 5;
    const int rg_local = wave % g.rg_per_wg, tpar = wave / g.rg_per_wg;
    if (tpar >= g.tile_par) return;
    const int rg = blockIdx.y * g.rg_per_wg + rg_local;
    if (rg >= g.n_rg) return;
    const int l = blockIdx.z / g.Hkv, kvh = blockIdx.z % g.Hkv;
    const int qh_per_kv = g.Hq / g.Hkv;
    const int n_sb = g.N / g.sb_tokens;
    const int sb_per_tile = 32 / g.sb_tokens;

    // query rows of this wave, resident for the whole sweep
    v8h_t qreg[NRBW][KS];
    int row[NRBW];       // row inside its head, or -1 if padding
    int lh[NRBW];        // layer * Hq + head
#pragma unroll
    for (int u = 0; u < NRBW; ++u) {
        const int rb = rg * NRBW + u;
        const int head = kvh * qh_per_kv + rb / g.RB;
        const int r = (rb % g.RB) * 32 + lrow;
        const bool ok = rb < g.n_rb && r < g.R;
        row[u] = ok ? r : -1;
        lh[u] = l * g.Hq + (rb < g.n_rb ? head : 0);
        const _Float16* qp = q + (static_cast<int64_t>(lh[u]) * g.R + (ok ? r : 0)) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            v8h_t v = {0, 0, 0, 0, 0, 0, 0, 0};
            if (ok) v = *reinterpret_cast<const v8h_t*>(qp + ks * 16);
            qreg[u][ks] = v;
        }
    }

    const _Float16* kbase = kv + (static_cast<int64_t>(l) * 2 * g.Hkv + kvh) * g.N * D;
    const int first_q_pos = g.N - g.R;
    const int tile_end = min((blockIdx.x + 1) * g.tiles_per_wg, g.n_tiles);
    for (int tile = blockIdx.x * g.tiles_per_wg + tpar; tile < tile_end; tile += g.tile_par) {
        const int t0 = tile * 32;
        v8h_t kreg[KS];
        const _Float16* kp = kbase + static_cast<int64_t>(t0 + lrow) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) kreg[ks] = *reinterpret_cast<const v8h_t*>(kp + ks * 16);
        const bool tail = (t0 + 31 > first_q_pos);   // wave-uniform: some entry may be masked
#pragma unroll
        for (int u = 0; u < NRBW; ++u) {
            if (rg * NRBW + u >= g.n_rb) break;
            v16f_t acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(kreg[ks], qreg[u][ks], acc, 0, 0, 0);
            // acc[v] = logit of (token t0 + 8*(v/4) + 4*half + v%4, query row lrow)
            float s[16];
            float mloc = -INFINITY;
            const int last_visible = (row[u] >= 0) ? first_q_pos + row[u] : -1;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int tk = t0 + 8 * (v / 4) + 4 * half + (v % 4);
                float x = acc[v] * g.scale_log2e;
                if (tail || row[u] < 0) x = (tk <= last_visible) ? x : -INFINITY;
                s[v] = x;
                mloc = fmaxf(mloc, x);
            }
            const float m_t = fmaxf(mloc, xhalf_f(mloc));
            const float m_use = (m_t == -INFINITY) ? 0.0f : m_t;
            float lsum = 0.0f;
            float esub[4] = {0.0f, 0.0f, 0.0f, 0.0f};   // up to 4 sub-blocks of 8 tokens
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int tk = t0 + 8 * (v / 4) + 4 * half + (v % 4);
                const float e = __builtin_amdgcn_exp2f(s[v] - m_use);
                lsum += e;
                float w = 1.0f;
                if (g.norm_mode == 0) {
                    const int vis = g.N - max(tk, first_q_pos);
                    w = tail ? 1.0f / static_cast<float>(vis) : 1.0f;   // constant 1/R applied below
                }
                const float ew = e * w;
                // sub-block index inside the tile: token offset / sb_tokens
                if (g.sb_tokens == 8) esub[v / 4] += ew;
                else if (g.sb_tokens == 16) esub[v / 8] += ew;
                else esub[0] += ew;
            }
            if (g.norm_mode == 0 && !tail) {
                const float w = 1.0f / static_cast<float>(g.R);
#pragma unroll
                for (int k = 0; k < 4; ++k) esub[k] *= w;
            }
            lsum += xhalf_f(lsum);
#pragma unroll
            for (int k = 0; k < 4; ++k) esub[k] += xhalf_f(esub[k]);
            if (half == 0 && row[u] >= 0) {
                const int64_t ti = (static_cast<int64_t>(lh[u]) * g.n_tiles + tile) * g.rows_p + row[u];
                ws.m_tile[ti] = m_t;
                ws.l_tile[ti] = lsum;
                for (int k = 0; k < sb_per_tile; ++k) {
                    const int64_t ei = (static_cast<int64_t>(lh[u]) * n_sb + tile * sb_per_tile + k) *
                                       g.rows_p + row[u];
                    ws.e_sub[ei] = esub[k];
                }
            }
        }
    }
}

// One workgroup per (layer, head): global row maximum and denominator from
// the per-tile partials, then the chunk masses.
__global__ __launch_bounds__(256) void score_combine_kernel(ScoreGeom g, ScoreWs ws,
                                                            float* __restrict__ chunk_mass) {
    __shared__ float sh_m[256];
    __shared__ float sh_l[256];
    __shared__ float row_m[256];
    __shared__ float row_f[256];
    const int lh = blockIdx.x;
    const int tid = threadIdx.x;
    const int parts = 256 / g.rows_p;            // rows_p in {32,...,256}
    const int r = tid % g.rows_p, part = tid / g.rows_p;
    const float* mt = ws.m_tile + static_cast<int64_t>(lh) * g.n_tiles * g.rows_p;
    const float* lt = ws.l_tile + static_cast<int64_t>(lh) * g.n_tiles * g.rows_p;
    float m = -INFINITY, lsum = 0.0f;
    if (part < parts && r < g.R) {
        for (int t = part; t < g.n_tiles; t += parts) {
            const float mi = mt[static_cast<int64_t>(t) * g.rows_p + r];
            const float li = lt[static_cast<int64_t>(t) * g.rows_p + r];
            if (mi > m) {
                lsum = lsum * __builtin_amdgcn_exp2f(m - mi) + li;   // m == -inf: lsum is 0
                m = mi;
            } else if (mi != -INFINITY) {
                lsum += li * __builtin_amdgcn_exp2f(mi - m);
            }
        }
    }
    sh_m[tid] = m;
    sh_l[tid] = lsum;
    __syncthreads();
    if (tid < g.rows_p && tid < g.R) {
        float M = -INFINITY;
        for (int p = 0; p < parts; ++p) M = fmaxf(M, sh_m[p * g.rows_p + tid]);
        float Lr = 0.0f;
        for (int p = 0; p < parts; ++p) {
            const float mi = sh_m[p * g.rows_p + tid];
            if (mi != -INFINITY) Lr += sh_l[p * g.rows_p + tid] * __builtin_amdgcn_exp2f(mi - M);
        }
        row_m[tid] = M;
        row_f[tid] = 1.0f / Lr;      // every row sees at least its own token: Lr >= 1
    }
    __syncthreads();

    // chunk masses: 32 lanes per chunk, lane <-> row (coalesced), fixed-order sums
    const int n_chunks = g.N / g.T;
    const int sb_per_chunk = g.T / g.sb_tokens;
    const int sb_per_tile = 32 / g.sb_tokens;
    const int n_sb = g.N / g.sb_tokens;
    const float* es = ws.e_sub + static_cast<int64_t>(lh) * n_sb * g.rows_p;
    const int grp = tid >> 5, gl = tid & 31;
    for (int c = grp; c < n_chunks; c += 8) {
        float acc = 0.0f;
        for (int k = 0; k < sb_per_chunk; ++k) {
            const int sb = c * sb_per_chunk + k;
            const int tile = sb / sb_per_tile;
            for (int rr = gl; rr < g.R; rr += 32) {
                const float mi = mt[static_cast<int64_t>(tile) * g.rows_p + rr];
                const float e = es[static_cast<int64_t>(sb) * g.rows_p + rr];
                if (mi != -INFINITY) acc += e * __builtin_amdgcn_exp2f(mi - row_m[rr]) * row_f[rr];
            }
        }
#pragma unroll
        for (int o = 16; o >= 1; o >>= 1) acc += __shfl_xor(acc, o);
        if (gl == 0) chunk_mass[static_cast<int64_t>(lh) * n_chunks + c] = acc;
    }
}

// density[i] = mean over (layer, head) of chunk_mass[.][i], per token of the chunk.
// Block = 64 chunks x 16 partial sums over the (layer, head) axis; the 16
// partials are added in a fixed order.
__global__ __launch_bounds__(1024) void score_density_kernel(const float* __restrict__ chunk_mass,
                                                             float* __restrict__ density,
                                                             int32_t n_lh, int32_t n_chunks,
                                                             float inv_norm) {
    __shared__ float part[16][64];
    const int ci = threadIdx.x & 63, p = threadIdx.x >> 6;
    const int i = blockIdx.x * 64 + ci;
    float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (i < n_chunks) {
        int k = p;
        for (; k + 48 < n_lh; k += 64) {
#pragma unroll
            for (int u = 0; u < 4; ++u)
                acc[u] += chunk_mass[static_cast<int64_t>(k + 16 * u) * n_chunks + i];
        }
        for (; k < n_lh; k += 16) acc[0] += chunk_mass[static_cast<int64_t>(k) * n_chunks + i];
    }
    part[p][ci] = (acc[0] + acc[1]) + (acc[2] + acc[3]);
    __syncthreads();
    if (p == 0 && i < n_chunks) {
        float t = 0.0f;
#pragma unroll
        for (int k = 0; k < 16; ++k) t += part[k][ci];
        density[i] = t * inv_norm;
    }
}

}  // namespace kvs
