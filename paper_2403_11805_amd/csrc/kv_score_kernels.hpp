// gfx950 kernels for the information density of chunks (Sec. 3.2, Eq. 1):
// A = softmax(mask(Q K^T / sqrt(D))) per (layer, head), column mass per chunk,
// mean over layers and heads.
//
// K is read once.  Kernel 1 sweeps K in tiles of 32 tokens; one wavefront holds
// one or two blocks of 32 query rows in registers, walks a contiguous run of
// tiles and produces, per tile, the 32x32 logit block with MFMA (K tile as the A
// operand, so a lane owns one query row and 16 of the tile's tokens, which makes
// the row reductions mostly in-lane).  Because the softmax denominator of a row
// is only known after the whole sweep, each tile is exponentiated against its
// own row maximum and partial results are written out: per (row, tile) the
// local maximum, per (row, sub-block of min(T,32) tokens) the weighted sum, and
// per (row, run) the running maximum and denominator of the run (kept in
// registers, flash-attention style).  Kernel 2 combines them per (layer, head)
// into chunk masses; kernel 3 averages over layers and heads.  Where a head has
// one block of query rows and there are many heads, score_head_kernel does the
// work of kernels 1 and 2 in one workgroup per head, with the partials in LDS.
// All reductions run in a fixed order: results are deterministic.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kv_lane_ops.hpp"

namespace kvs {

typedef _Float16 v8h_t __attribute__((ext_vector_type(8)));
typedef float v16f_t __attribute__((ext_vector_type(16)));

struct ScoreGeom {
    int32_t L, Hkv, Hq, N, R;
    int32_t Nv;           // valid tokens (<= N): the query rows are the last R of them, the rest is padding
    int32_t T;            // chunk tokens (power of two >= 8)
    int32_t sb_tokens;    // min(T, 32): tokens per stored sub-block
    int32_t n_tiles;      // N / 32
    int32_t RB;           // ceil(R / 32): row blocks per head
    int32_t rows_p;       // RB * 32
    int32_t n_rb;         // (Hq / Hkv) * RB: row blocks per kv head
    int32_t n_rg;         // row groups (each NRBW row blocks) per kv head
    int32_t rg_per_wg;    // row groups handled by one workgroup (1..4)
    int32_t tile_par;     // runs of tiles processed side by side by one workgroup (4 / rg_per_wg)
    int32_t run_len;      // consecutive tiles per wavefront run
    int32_t n_runs;       // ceil(n_tiles / run_len): runs per (layer, head)
    int32_t norm_mode;    // 0: divide each column by its number of visible rows; 1: plain sums
    float   scale_log2e;  // log2(e) / sqrt(D)
    float   inv_R;        // 1 / R
};

// Workspace planes (floats), row index fastest:
//   m_tile [L*Hq][n_tiles][rows_p]   tile-local row maximum (log2 units)
//   e_sub  [L*Hq][n_sb][rows_p]      weighted sum of 2^(s - m_tile) over the sub-block
//   m_run, l_run [L*Hq][n_runs][rows_p]  maximum and denominator of a run of tiles
//   m_fast [L*Hq][n_runs][rows_p]        the ONE reference of the tiles of the run that lie below the
//                                        causal diagonal, if they were all exponentiated against it (their
//                                        m_tile slots are then not written); NaN if every tile has its own
struct ScoreWs {
    float* m_tile;
    float* e_sub;
    float* m_run;
    float* l_run;
    float* m_fast;
};

// Softmax partials of one 32-token tile for one block of 32 query rows.
// acc[v] = raw logit of (token tile*32 + 8*(v/4) + 4*half + v%4, query row of this lane);
// row < 0 marks a padding row.  Writes the tile's reference exponent and the
// weighted sub-block sums, and folds the tile into the run's reference / denominator.
//
// Every row keeps ONE reference exponent m_ref for a whole run of tiles: the
// maximum of the run's first tile.  Later tiles are exponentiated against it
// without a maximum pass of their own; should a tile's sum leave the safe range
// (a logit more than 60 binary orders above the reference) the tile is redone
// against its own maximum, which becomes the new reference.  The partials only
// promise "sum of w * 2^(s - m_tile)" for the m_tile stored beside them.
constexpr float kRefOverflow = 1.152921504606846976e18f;   // 2^60

// stage_m / stage_e (both or neither): LDS slots of this tile, [32] and [n_sub][32] floats indexed by
// the row inside its block; the caller copies them to the workspace later.  NULL: store directly.
__device__ __forceinline__ void tile_epilogue(const v16f_t& acc, const ScoreGeom& g, const ScoreWs& ws,
                                              int tile, int row, int lh, int half, bool first,
                                              float& m_ref, float& l_run, float* stage_m = nullptr,
                                              float* stage_e = nullptr) {
    const int t0 = tile * 32;
    const int first_q_pos = g.Nv - g.R;
    const bool tail = (t0 + 31 > first_q_pos);   // wave-uniform: some entry may be masked
    float m_t;
    // q4[k]: (weighted) sum over the lane's tokens 8k..8k+7 of the tile; l4[k]: unweighted
    float q4[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    float l4[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    float lsum;
    if (!tail) {
        // every entry is visible and every column has the same weight
        bool own_max = first;
        for (;;) {
            if (own_max) {
                float mloc = acc[0];
#pragma unroll
                for (int v = 1; v < 16; ++v) mloc = fmaxf(mloc, acc[v]);
                // the reference never decreases, so the rescaling factor is at most 1
                // (a padding row has logits 0: its reference is 0, its sums are never stored)
                const float m_new = fmaxf(m_ref, xhalf_max(mloc) * g.scale_log2e);
                l_run = (m_ref == -INFINITY) ? 0.0f : l_run * __builtin_amdgcn_exp2f(m_ref - m_new);
                m_ref = m_new;
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) l4[k] = 0.0f;
#pragma unroll
            for (int v = 0; v < 16; ++v)
                l4[v / 4] += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[v], g.scale_log2e, -m_ref));
            lsum = xhalf_sum((l4[0] + l4[1]) + (l4[2] + l4[3]));
            // wave-uniform: redo the tile against its own maximum if any row left the safe range
            if (own_max || !__any(!(lsum < kRefOverflow))) break;
            own_max = true;
        }
        m_t = m_ref;
        l_run += lsum;
        const float w_const = (g.norm_mode == 0) ? g.inv_R : 1.0f;
#pragma unroll
        for (int k = 0; k < 4; ++k) q4[k] = l4[k] * w_const;
    } else {
        float s[16];
        float mloc = -INFINITY;
        const int last_visible = (row >= 0) ? first_q_pos + row : -1;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int tk = t0 + 8 * (v / 4) + 4 * half + (v % 4);
            const float x = (tk <= last_visible) ? acc[v] * g.scale_log2e : -INFINITY;
            s[v] = x;
            mloc = fmaxf(mloc, x);
        }
        m_t = xhalf_max(mloc);
        const float m_use = (m_t == -INFINITY) ? 0.0f : m_t;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int tk = t0 + 8 * (v / 4) + 4 * half + (v % 4);
            const float e = __builtin_amdgcn_exp2f(s[v] - m_use);
            l4[v / 4] += e;
            float w = 1.0f;
            // rows that see token tk; a padding token is seen by none and its e is 0: no 0 * inf
            const int seen = g.Nv - max(tk, first_q_pos);
            if (g.norm_mode == 0) w = seen > 0 ? 1.0f / static_cast<float>(seen) : 0.0f;
            q4[v / 4] += e * w;
        }
        lsum = xhalf_sum((l4[0] + l4[1]) + (l4[2] + l4[3]));
        // this tile keeps its own maximum; the run's reference moves to the larger of the two
        const float m_new = fmaxf(m_ref, m_t);
        const float m_safe = (m_new == -INFINITY) ? 0.0f : m_new;
        l_run = l_run * __builtin_amdgcn_exp2f(m_ref - m_safe) + lsum * __builtin_amdgcn_exp2f(m_t - m_safe);
        m_ref = m_new;
    }
    // sub-block sums: 8, 16 or 32 tokens each (uniform branch), both halves together
    float esub[4];
    int n_sub;
    if (g.sb_tokens == 8) {
        n_sub = 4;
#pragma unroll
        for (int k = 0; k < 4; ++k) esub[k] = xhalf_sum(q4[k]);
    } else if (g.sb_tokens == 16) {
        n_sub = 2;
        const float a = q4[0] + q4[1], b2 = q4[2] + q4[3];
        esub[0] = xhalf_sum(a);
        esub[1] = xhalf_sum(b2);
        esub[2] = esub[3] = 0.0f;
    } else {
        n_sub = 1;
        const float a = (q4[0] + q4[1]) + (q4[2] + q4[3]);
        esub[0] = xhalf_sum(a);
        esub[1] = esub[2] = esub[3] = 0.0f;
    }
    if (half == 0 && row >= 0) {
        if (stage_m) {
            stage_m[row & 31] = m_t;
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (k < n_sub) stage_e[k * 32 + (row & 31)] = esub[k];
        } else {
            const int n_sb = g.N / g.sb_tokens;
            ws.m_tile[(static_cast<int64_t>(lh) * g.n_tiles + tile) * g.rows_p + row] = m_t;
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (k < n_sub)
                    ws.e_sub[(static_cast<int64_t>(lh) * n_sb + tile * n_sub + k) * g.rows_p + row] = esub[k];
        }
    }
}

template <int D, int NRBW>
__global__ __launch_bounds__(256) void score_tiles_kernel(const _Float16* __restrict__ q,
                                                          const _Float16* __restrict__ kv,
                                                          ScoreGeom g, ScoreWs ws) {
    constexpr int KS = D / 16;
    constexpr int kMaxRun = 8;       // tiles per run at most (host: run_len <= 8 for this kernel)
    // Partials of a run are collected in LDS and written out after the run: stores issued between
    // the K loads would hold back every wait for the next tile (one counter tracks both).
    __shared__ float stage_m[4][NRBW][kMaxRun][32];
    __shared__ float stage_e[4][NRBW][kMaxRun * 4][32];
    const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6)), lane = threadIdx.x & 63;
    const int lrow = lane & 31, half = lane >> 5;
    const int rg_local = wave % g.rg_per_wg, tpar = wave / g.rg_per_wg;
    if (tpar >= g.tile_par) return;
    const int rg = blockIdx.y * g.rg_per_wg + rg_local;
    if (rg >= g.n_rg) return;
    const int run = blockIdx.x * g.tile_par + tpar;
    const int tile_begin = run * g.run_len;
    if (tile_begin >= g.n_tiles) return;
    const int tile_end = min(tile_begin + g.run_len, g.n_tiles);
    const int l = blockIdx.z / g.Hkv, kvh = blockIdx.z % g.Hkv;
    const int qh_per_kv = g.Hq / g.Hkv;
    const int n_sub_tile = 32 / g.sb_tokens;         // sub-blocks per tile: 1, 2 or 4

    // query rows of this wave, resident for the whole run
    v8h_t qreg[NRBW][KS];
    int row[NRBW];       // row inside its head, or -1 if padding
    int lh[NRBW];        // layer * Hq + head
    float m_run[NRBW], l_run[NRBW];
#pragma unroll
    for (int u = 0; u < NRBW; ++u) {
        const int rb = rg * NRBW + u;
        const int head = kvh * qh_per_kv + rb / g.RB;
        const int r = (rb % g.RB) * 32 + lrow;
        const bool ok = rb < g.n_rb && r < g.R;
        row[u] = ok ? r : -1;
        lh[u] = l * g.Hq + (rb < g.n_rb ? head : 0);
        m_run[u] = -INFINITY;
        l_run[u] = 0.0f;
        const _Float16* qp = q + (static_cast<int64_t>(lh[u]) * g.R + (ok ? r : 0)) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            v8h_t v = {0, 0, 0, 0, 0, 0, 0, 0};
            if (ok) v = *reinterpret_cast<const v8h_t*>(qp + ks * 16);
            qreg[u][ks] = v;
        }
    }

    const _Float16* kbase = kv + (static_cast<int64_t>(l) * 2 * g.Hkv + kvh) * g.N * D;
    // K tiles are double-buffered in registers: the loads of the next tile are
    // in flight while the current one goes through MFMA and the softmax.
    v8h_t knext[KS];
    {
        const _Float16* kp = kbase + static_cast<int64_t>(tile_begin * 32 + lrow) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) knext[ks] = *reinterpret_cast<const v8h_t*>(kp + ks * 16);
    }
    for (int tile = tile_begin; tile < tile_end; ++tile) {
        const int t0 = tile * 32;
        v8h_t kreg[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) kreg[ks] = knext[ks];
        if (tile + 1 < tile_end) {
            const _Float16* kp = kbase + static_cast<int64_t>(t0 + 32 + lrow) * D + half * 8;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) knext[ks] = *reinterpret_cast<const v8h_t*>(kp + ks * 16);
        }
        // independent accumulators of the row blocks are interleaved so that
        // consecutive MFMAs do not depend on each other
        v16f_t acc[NRBW];
#pragma unroll
        for (int u = 0; u < NRBW; ++u) acc[u] = v16f_t{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int u = 0; u < NRBW; ++u)
                acc[u] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kreg[ks], qreg[u][ks], acc[u], 0, 0, 0);
#pragma unroll
        for (int u = 0; u < NRBW; ++u) {
            if (rg * NRBW + u >= g.n_rb) break;
            const int tl = tile - tile_begin;
            tile_epilogue(acc[u], g, ws, tile, row[u], lh[u], half, tile == tile_begin, m_run[u], l_run[u],
                          stage_m[wave][u][tl], stage_e[wave][u][tl * n_sub_tile]);
        }
    }
    // the wavefront's own LDS writes are ordered before its reads below
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int ntl = tile_end - tile_begin;
    const int n_sb = g.N / g.sb_tokens;
#pragma unroll
    for (int u = 0; u < NRBW; ++u) {
        const int rb = rg * NRBW + u;
        if (rb >= g.n_rb) break;
        const int row_base = (rb % g.RB) * 32;          // first row of this block inside its head
        for (int i = lane; i < ntl * 32; i += 64) {
            const int r = row_base + (i & 31);
            if (r < g.R)
                ws.m_tile[(static_cast<int64_t>(lh[u]) * g.n_tiles + tile_begin + (i >> 5)) * g.rows_p + r] =
                    stage_m[wave][u][i >> 5][i & 31];
        }
        for (int i = lane; i < ntl * n_sub_tile * 32; i += 64) {
            const int r = row_base + (i & 31);
            if (r < g.R)
                ws.e_sub[(static_cast<int64_t>(lh[u]) * n_sb + tile_begin * n_sub_tile + (i >> 5)) * g.rows_p + r] =
                    stage_e[wave][u][i >> 5][i & 31];
        }
        if (half == 0 && row[u] >= 0) {
            const int64_t ri = (static_cast<int64_t>(lh[u]) * g.n_runs + run) * g.rows_p + row[u];
            ws.m_run[ri] = m_run[u];
            ws.l_run[ri] = l_run[u];
            ws.m_fast[ri] = __builtin_nanf("");      // every tile of this kernel has a reference of its own
        }
    }
}

// Partials of a tile whose entries are all visible, against the row's current
// reference, with no branch and no maximum pass: straight-line code that can be
// interleaved with the MFMAs of the next tile.  Both halves of the wavefront
// store the same values to the same slots; padding rows have slots of their own
// (rows_p per tile).  `bad` collects rows whose sum left the safe range: the
// caller then redoes the tile through tile_epilogue.
//   SBT = sub-blocks per tile (32 / sb_tokens); es = this lane's slots of the tile.  The reference is
//   the same for every tile of the pass and is stored once per run by the caller (ScoreWs::m_fast).
template <int SBT>
__device__ __forceinline__ void fast_epilogue(const v16f_t& acc, float scale_log2e, float w,
                                              float m_ref, float& l_run, uint32_t& bad,
                                              float* __restrict__ es, int rows_p) {
    float l4[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        float a = __builtin_amdgcn_exp2f(__builtin_fmaf(acc[4 * k], scale_log2e, -m_ref));
#pragma unroll
        for (int i = 1; i < 4; ++i)
            a += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[4 * k + i], scale_log2e, -m_ref));
        l4[k] = a;
    }
    float sub[SBT];
    float lsum;
    if constexpr (SBT == 1) {
        sub[0] = xhalf_sum((l4[0] + l4[1]) + (l4[2] + l4[3]));
        lsum = sub[0];
    } else if constexpr (SBT == 2) {
        sub[0] = xhalf_sum(l4[0] + l4[1]);
        sub[1] = xhalf_sum(l4[2] + l4[3]);
        lsum = sub[0] + sub[1];
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) sub[k] = xhalf_sum(l4[k]);
        lsum = (sub[0] + sub[1]) + (sub[2] + sub[3]);
    }
    l_run += lsum;
    bad |= (lsum < kRefOverflow) ? 0u : 1u;
#pragma unroll
    for (int k = 0; k < SBT; ++k) es[k * rows_p] = sub[k] * w;
}

// Variant for grouped-query attention: the 2-4 wavefronts of a workgroup hold
// the row blocks (two each) of different query heads that read the SAME kv head,
// so K is fetched once per workgroup (fully coalesced, 16 bytes per thread and
// access), staged in LDS (two buffers of two tiles; the 16-byte pieces of a row
// are permuted by its row number so that the operand reads are bank-conflict
// free) and read from there by every wavefront: one barrier per 64 tokens.
//
// A run is processed in up to three passes over its tiles:
//  - the fast pass over the tiles below the causal diagonal.  The row references
//    come from the run's first tile; the loads of a stage are issued two stages
//    ahead (two register sets used in turn), and inside a wavefront the MFMAs of
//    a tile are interleaved, instruction by instruction, with the softmax
//    partials (fast_epilogue) of the tile before it (two accumulator sets used in
//    turn), so that the matrix pipe and the VALU work overlap;
//  - the general pass (tile_epilogue) over the tiles that reach the diagonal;
//  - the general pass over the whole fast range again if some sum left the safe
//    range there (workgroup-wide decision), or instead of the fast pass if a
//    wavefront holds only one row block.
template <int D, int SBT>
__global__ __launch_bounds__(256, 2) void score_tiles_shared_kernel(const _Float16* __restrict__ q,
                                                                    const _Float16* __restrict__ kv,
                                                                    ScoreGeom g, ScoreWs ws) {
    constexpr int NRBW = 2;
    constexpr int KS = D / 16;
    constexpr int kRowPieces = D / 8;               // 16-byte pieces per token row
    constexpr int kTilePieces = 32 * kRowPieces;
    constexpr int TS = D <= 128 ? 2 : 1;                 // tiles per LDS stage (two 32 KiB buffers at most)
    constexpr int kPerThread = TS * kTilePieces / 256;   // 16-byte loads per thread and stage
    typedef unsigned int su4_t __attribute__((ext_vector_type(4)));
    __shared__ su4_t kstage[2][TS * 32 * kRowPieces];
    // piece c of stage row r sits at r * kRowPieces + (c ^ swz(r)): 16 consecutive rows of one
    // piece column fall into 16 different 16-byte bank groups
    auto swz = [](int r) __attribute__((always_inline)) { return D == 64 ? (r >> 1) & 7 : r & 15; };

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int lrow = lane & 31, half = lane >> 5;
    const int run = blockIdx.x;
    const int tile_begin = run * g.run_len;
    if (tile_begin >= g.n_tiles) return;             // whole workgroup
    const int tile_end = min(tile_begin + g.run_len, g.n_tiles);
    const int rg = blockIdx.y * g.rg_per_wg + wave;
    const bool active = wave < g.rg_per_wg && rg < g.n_rg;
    const int l = blockIdx.z / g.Hkv, kvh = blockIdx.z % g.Hkv;
    const int qh_per_kv = g.Hq / g.Hkv;
    // tiles from here on touch the causal diagonal
    const int first_tail_tile = (g.Nv - g.R + 1) / 32;
    const bool two_blocks = rg * NRBW + 1 < g.n_rb;
    // the fast pass needs both row blocks in every wavefront (workgroup-uniform)
    const int fast_end = (g.n_rb % NRBW == 0) ? min(tile_end, max(first_tail_tile, tile_begin)) : tile_begin;

    v8h_t qreg[NRBW][KS];
    int row[NRBW], lh[NRBW];
    float m_run[NRBW], l_run[NRBW];
    float* es_base[NRBW];     // this lane's slot of tile 0 in e_sub
#pragma unroll
    for (int u = 0; u < NRBW; ++u) {
        const int rb = rg * NRBW + u;
        const bool exists = active && rb < g.n_rb;
        const int head = kvh * qh_per_kv + (exists ? rb / g.RB : 0);
        const int r = (rb % g.RB) * 32 + lrow;          // slot inside the head: < rows_p
        const bool ok = exists && r < g.R;
        row[u] = ok ? r : -1;
        lh[u] = l * g.Hq + head;
        m_run[u] = -INFINITY;
        l_run[u] = 0.0f;
        es_base[u] = ws.e_sub + static_cast<int64_t>(lh[u]) * g.n_tiles * SBT * g.rows_p + r;
        const _Float16* qp = q + (static_cast<int64_t>(lh[u]) * g.R + (ok ? r : 0)) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            v8h_t v = {0, 0, 0, 0, 0, 0, 0, 0};
            if (ok) v = *reinterpret_cast<const v8h_t*>(qp + ks * 16);
            qreg[u][ks] = v;
        }
    }

    const su4_t* kbase = reinterpret_cast<const su4_t*>(
        kv + (static_cast<int64_t>(l) * 2 * g.Hkv + kvh) * g.N * D);
    // pieces of the stage that starts at tile t (< stop).  Loads are unconditional so that they
    // stay in flight: a tile at or beyond `stop` is replaced by tile stop - 1 and never used.
    auto fetch = [&](su4_t (&st)[kPerThread], int t, int stop) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) {
            const int p = i * 256 + tid;
            const int tile = min(t + p / kTilePieces, stop - 1);
            st[i] = kbase[static_cast<int64_t>(tile) * kTilePieces + p % kTilePieces];
        }
    };
    auto park = [&](const su4_t (&st)[kPerThread], int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) {
            const int p = i * 256 + tid;
            const int r = p / kRowPieces, c = p % kRowPieces;
            kstage[buf][r * kRowPieces + (c ^ swz(r))] = st[i];
        }
    };
    // K operand of tile j (0 or 1) of a stage, then the logits of both row blocks
    auto logits = [&](v16f_t (&a)[NRBW], int buf, int j) __attribute__((always_inline)) {
        v8h_t kreg[KS];
        const int r = j * 32 + lrow;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            kreg[ks] = __builtin_bit_cast(v8h_t, kstage[buf][r * kRowPieces + ((2 * ks + half) ^ swz(r))]);
#pragma unroll
        for (int u = 0; u < NRBW; ++u) a[u] = v16f_t{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        // independent accumulators interleaved: consecutive MFMAs do not depend on each other
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int u = 0; u < NRBW; ++u)
                a[u] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kreg[ks], qreg[u][ks], a[u], 0, 0, 0);
    };

    // General pass over tiles [from, to): plain double buffering, partials right behind the MFMAs.
    auto general_pass = [&](int from, int to) __attribute__((always_inline)) {
        su4_t st[kPerThread];
        fetch(st, from, to);
        park(st, 0);
        __syncthreads();
        for (int t = from; t < to; t += TS) {
            const int buf = ((t - from) / TS) & 1;
            const bool more = t + TS < to;
            if (more) fetch(st, t + TS, to);
            if (active) {
                for (int j = 0; j < TS && t + j < to; ++j) {
                    v16f_t a[NRBW];
                    logits(a, buf, j);
#pragma unroll
                    for (int u = 0; u < NRBW; ++u) {
                        if (u == 1 && !two_blocks) break;
                        tile_epilogue(a[u], g, ws, t + j, row[u], lh[u], half, t + j == tile_begin,
                                      m_run[u], l_run[u]);
                    }
                }
            }
            if (more) park(st, buf ^ 1);
            __syncthreads();
        }
    };

    int dirty = 0;
    if (fast_end > tile_begin) {
        const float w_const = (g.norm_mode == 0) ? g.inv_R : 1.0f;
        su4_t sa[kPerThread], sb[kPerThread];   // stages in flight: sa holds odd stages, sb even ones
        fetch(sb, tile_begin, fast_end);
        park(sb, 0);
        fetch(sa, tile_begin + TS, fast_end);
        __syncthreads();
        v16f_t acc[2][NRBW];
        uint32_t bad = 0;
        if (active) {
            // row references: the maxima of the first tile
            logits(acc[0], 0, 0);
#pragma unroll
            for (int u = 0; u < NRBW; ++u) {
                float mloc = acc[0][u][0];
#pragma unroll
                for (int v = 1; v < 16; ++v) mloc = fmaxf(mloc, acc[0][u][v]);
                m_run[u] = xhalf_max(mloc) * g.scale_log2e;
            }
        }
        // the MFMAs of tile `tile` (set cur) interleaved with the partials of tile - 1 (set cur ^ 1)
        auto fast_tile = [&](int cur, int buf, int j, int tile) __attribute__((always_inline)) {
            if (tile == tile_begin) {
                logits(acc[cur], buf, j);
                return;
            }
            logits(acc[cur], buf, j);
#pragma unroll
            for (int u = 0; u < NRBW; ++u)
                fast_epilogue<SBT>(acc[cur ^ 1][u], g.scale_log2e, w_const, m_run[u], l_run[u], bad,
                                   es_base[u] + static_cast<int64_t>(tile - 1) * SBT * g.rows_p, g.rows_p);
            // one MFMA, then a share of the VALU work, and so on
#pragma unroll
            for (int i = 0; i < KS * NRBW; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x402, (2 * (66 + 2 * SBT)) / (KS * NRBW) + 1, 0);
            }
        };
        // stage s (TS tiles from t) is in kstage[s & 1]; `next` holds stage s + 1, `far` receives
        // stage s + 2.  Tiles use the accumulator sets in turn: set = (tile - tile_begin) & 1.
        auto fast_stage = [&](int t, int buf, su4_t (&next)[kPerThread], su4_t (&far)[kPerThread])
                              __attribute__((always_inline)) {
            if (t + 2 * TS < fast_end) fetch(far, t + 2 * TS, fast_end);
            if (active) {
                if constexpr (TS == 2) {
                    fast_tile(0, buf, 0, t);
                    if (t + 1 < fast_end) fast_tile(1, buf, 1, t + 1);
                } else {
                    fast_tile(buf, buf, 0, t);
                }
            }
            if (t + TS < fast_end) park(next, buf ^ 1);
            __syncthreads();
        };
        for (int t = tile_begin; t < fast_end; t += 2 * TS) {
            fast_stage(t, 0, sa, sb);
            if (t + TS < fast_end) fast_stage(t + TS, 1, sb, sa);
        }
        if (active) {
            // partials of the last tile of the pass
            const int last = fast_end - 1;
            const int set = (last - tile_begin) & 1;
#pragma unroll
            for (int u = 0; u < NRBW; ++u) {
                float* es = es_base[u] + static_cast<int64_t>(last) * SBT * g.rows_p;
                if (set == 0) fast_epilogue<SBT>(acc[0][u], g.scale_log2e, w_const, m_run[u], l_run[u], bad, es, g.rows_p);
                else fast_epilogue<SBT>(acc[1][u], g.scale_log2e, w_const, m_run[u], l_run[u], bad, es, g.rows_p);
            }
        }
        dirty = __syncthreads_or(static_cast<int>(bad));
    }
    // the reference of the fast pass, for the combine kernel (NaN: no fast pass, or it is redone below)
    if (active) {
        const bool fast_ok = fast_end > tile_begin && !dirty;
#pragma unroll
        for (int u = 0; u < NRBW; ++u)
            if (half == 0 && row[u] >= 0)
                ws.m_fast[(static_cast<int64_t>(lh[u]) * g.n_runs + run) * g.rows_p + row[u]] =
                    fast_ok ? m_run[u] : __builtin_nanf("");
    }
    if (dirty) {
        // start over through the general path (which writes every slot of these tiles again)
#pragma unroll
        for (int u = 0; u < NRBW; ++u) {
            m_run[u] = -INFINITY;
            l_run[u] = 0.0f;
        }
    }
    for (int pass = dirty ? 0 : 1; pass < 2; ++pass) {
        const int from = pass == 0 ? tile_begin : fast_end;
        const int to = pass == 0 ? fast_end : tile_end;
        if (from < to) general_pass(from, to);
    }
    if (active) {
#pragma unroll
        for (int u = 0; u < NRBW; ++u) {
            if (half == 0 && row[u] >= 0) {
                const int64_t ri = (static_cast<int64_t>(lh[u]) * g.n_runs + run) * g.rows_p + row[u];
                ws.m_run[ri] = m_run[u];
                ws.l_run[ri] = l_run[u];
            }
        }
    }
}

// One workgroup per (layer, head) when a head has a single block of query rows and many heads
// are scored (multi-head attention, R <= 32): the four wavefronts take the runs of tiles in
// turn, the partial results stay in LDS, relative to ONE reference per (row, run), and the
// workgroup itself turns them into the chunk masses.  No partials travel through HBM and no
// combine launch is needed.  Dynamic LDS (floats), rows fastest:
//   e_all [n_sb][32]   weighted sub-block sums relative to the run's final reference
//   m_run, l_run [n_runs][32]
//   tmp [4 wavefronts][5][32]   the slots tile_epilogue fills for one tile
//   row_m, row_f [32]
template <int D>
__global__ __launch_bounds__(256, 4) void score_head_kernel(const _Float16* __restrict__ q,
                                                         const _Float16* __restrict__ kv, ScoreGeom g,
                                                         float* __restrict__ chunk_mass) {
    constexpr int KS = D / 16;
    extern __shared__ float score_head_lds[];
    const int n_sub_tile = 32 / g.sb_tokens;
    const int n_sb = g.n_tiles * n_sub_tile;
    float* e_all = score_head_lds;
    float* m_run_l = e_all + n_sb * 32;
    float* l_run_l = m_run_l + g.n_runs * 32;
    float* tmp = l_run_l + g.n_runs * 32;
    float* row_m = tmp + 4 * 5 * 32;
    float* row_f = row_m + 32;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;   // uniform: run and tile bookkeeping in scalar registers
    const int lrow = lane & 31, half = lane >> 5;
    const int l = blockIdx.x / g.Hkv, kvh = blockIdx.x % g.Hkv;
    const int lh = l * g.Hq + kvh;                    // one query head per kv head
    const int row = lrow < g.R ? lrow : -1;
    float* tmp_m = tmp + wave * 5 * 32;
    float* tmp_e = tmp_m + 32;
    const ScoreWs no_ws = {nullptr, nullptr, nullptr, nullptr, nullptr};

    v8h_t qreg[KS];
    {
        const _Float16* qp = q + (static_cast<int64_t>(lh) * g.R + (row >= 0 ? row : 0)) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            v8h_t v = {0, 0, 0, 0, 0, 0, 0, 0};
            if (row >= 0) v = *reinterpret_cast<const v8h_t*>(qp + ks * 16);
            qreg[ks] = v;
        }
    }
    const _Float16* kbase = kv + (static_cast<int64_t>(l) * 2 * g.Hkv + kvh) * g.N * D;
    // K tiles are double-buffered in registers across the tiles and runs of this wavefront.  A wavefront
    // walks a contiguous quarter of the plane: four streams a quarter plane apart
    const int runs_per_wave = (g.n_runs + 3) / 4;
    const int run_first = wave * runs_per_wave, run_last = min(run_first + runs_per_wave, g.n_runs);
    // ... each plane starting at another of its runs, so that the streams of different planes are not all at
    // the same offset of their planes at the same time
    const int n_mine = run_last - run_first;
    const int rot = n_mine > 0 ? static_cast<int>(blockIdx.x % static_cast<uint32_t>(n_mine)) : 0;
    auto nth_run = [&](int i) __attribute__((always_inline)) {
        const int k = i + rot;
        return run_first + (k >= n_mine ? k - n_mine : k);
    };
    v8h_t knext[KS];
    {
        const int t_first = min(nth_run(0) * g.run_len, g.n_tiles - 1);
        const _Float16* kp = kbase + static_cast<int64_t>(t_first * 32 + lrow) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) knext[ks] = *reinterpret_cast<const v8h_t*>(kp + ks * 16);
    }
    for (int ri = 0; ri < n_mine; ++ri) {
        const int run = nth_run(ri);
        const int tile_begin = run * g.run_len;
        const int tile_end = min(tile_begin + g.run_len, g.n_tiles);
        float m_ref = -INFINITY, l_run = 0.0f;
        for (int tile = tile_begin; tile < tile_end; ++tile) {
            v8h_t kreg[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) kreg[ks] = knext[ks];
            {   // the next tile of the run, or the first tile of this wavefront's next run
                int nt = tile + 1;
                if (nt >= tile_end) nt = min(nth_run(ri + 1 < n_mine ? ri + 1 : ri) * g.run_len, g.n_tiles - 1);
                const _Float16* kp = kbase + static_cast<int64_t>(nt * 32 + lrow) * D + half * 8;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) knext[ks] = *reinterpret_cast<const v8h_t*>(kp + ks * 16);
            }
            v16f_t acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(kreg[ks], qreg[ks], acc, 0, 0, 0);
            const float m_before = m_ref;
            tile_epilogue(acc, g, no_ws, tile, row, lh, half, tile == tile_begin, m_ref, l_run, tmp_m, tmp_e);
            // the lane that owns a row wrote its slots and reads them back: same lane, in order
            if (half == 0 && row >= 0) {
                const float m_t = tmp_m[lrow];
                const float f = (m_t == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(m_t - m_ref);
                for (int k = 0; k < n_sub_tile; ++k)
                    e_all[(tile * n_sub_tile + k) * 32 + lrow] = tmp_e[k * 32 + lrow] * f;
                if (tile != tile_begin && m_ref != m_before) {
                    // the reference of this row moved: earlier sums of the run follow it
                    const float r = (m_before == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(m_before - m_ref);
                    for (int i = tile_begin * n_sub_tile; i < tile * n_sub_tile; ++i) e_all[i * 32 + lrow] *= r;
                }
            }
        }
        if (half == 0 && row >= 0) {
            m_run_l[run * 32 + lrow] = m_ref;
            l_run_l[run * 32 + lrow] = l_run;
        }
    }
    __syncthreads();
    // row reference and denominator over the runs, in ascending order
    if (tid < 32 && tid < g.R) {
        float M = -INFINITY;
        for (int r = 0; r < g.n_runs; ++r) M = fmaxf(M, m_run_l[r * 32 + tid]);
        float Lr = 0.0f;
        for (int r = 0; r < g.n_runs; ++r) {
            const float mi = m_run_l[r * 32 + tid];
            if (mi != -INFINITY) Lr += l_run_l[r * 32 + tid] * __builtin_amdgcn_exp2f(mi - M);
        }
        row_m[tid] = M;
        row_f[tid] = 1.0f / Lr;          // every row sees at least its own token
    }
    __syncthreads();
    // one factor per (run, row) takes a sum from its run's reference to the normalised row
    // (kept where the run's denominator was); rows beyond R get 0
    for (int i = tid; i < g.n_runs * 32; i += 256) {
        const int r = i & 31;
        const float mi = m_run_l[i];
        l_run_l[i] = (r < g.R && mi != -INFINITY) ? __builtin_amdgcn_exp2f(mi - row_m[r]) * row_f[r] : 0.0f;
    }
    __syncthreads();
    // chunk masses: 32 lanes per chunk, lane <-> row, fixed-order sums, two chunks in flight
    const int n_chunks = g.N / g.T;
    const int sb_per_chunk = g.T / g.sb_tokens;
    const int sb_per_run = g.run_len * n_sub_tile;
    const int grp = tid >> 5, gl = tid & 31;
    const bool live = gl < g.R;
    for (int c = grp; c < n_chunks; c += 16) {
        const int c2 = min(c + 8, n_chunks - 1);
        float a = 0.0f, b = 0.0f;
        for (int k = 0; k < sb_per_chunk; ++k) {
            const int sa = c * sb_per_chunk + k, sb2 = c2 * sb_per_chunk + k;
            // padding rows hold no sums: their factor is 0, the product must not be NaN
            const float ea = live ? e_all[sa * 32 + gl] : 0.0f, eb = live ? e_all[sb2 * 32 + gl] : 0.0f;
            a += ea * l_run_l[(sa / sb_per_run) * 32 + gl];
            b += eb * l_run_l[(sb2 / sb_per_run) * 32 + gl];
        }
#pragma unroll
        for (int o = 16; o >= 1; o >>= 1) {
            a += __shfl_xor(a, o);
            b += __shfl_xor(b, o);
        }
        if (gl == 0) {
            chunk_mass[static_cast<int64_t>(lh) * n_chunks + c] = a;
            if (c + 8 < n_chunks) chunk_mass[static_cast<int64_t>(lh) * n_chunks + c + 8] = b;
        }
    }
}

// Grid (layer * head, parts): global row maximum and denominator from the per-run
// partials, then the chunk masses from the per-tile partials.  `parts` workgroups
// divide the chunks of a head among themselves so that long contexts keep enough
// wavefronts in flight.
constexpr int kCombineMaxRuns = 8192;       // runs per head the combine kernel keeps a bit for (host-checked)

__global__ __launch_bounds__(256, 8) void score_combine_kernel(ScoreGeom g, ScoreWs ws,
                                                            float* __restrict__ chunk_mass) {
    __shared__ float sh_m[256];
    __shared__ float sh_l[256];
    __shared__ __align__(16) float row_m[256];
    __shared__ __align__(16) float row_f[256];
    const int lh = blockIdx.x;
    const int tid = threadIdx.x;
    const int parts = 256 / g.rows_p;            // rows_p in {32,...,256}
    const int r = tid % g.rows_p, part = tid / g.rows_p;
    const float* mr = ws.m_run + static_cast<int64_t>(lh) * g.n_runs * g.rows_p;
    const float* lr = ws.l_run + static_cast<int64_t>(lh) * g.n_runs * g.rows_p;
    float m = -INFINITY, lsum = 0.0f;
    if (part < parts && r < g.R) {
        // four runs per pass, their loads issued together; a slot beyond the last run repeats it as an empty one
        for (int t = part; t < g.n_runs; t += 4 * parts) {
            float mi4[4], li4[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int tu = min(t + u * parts, g.n_runs - 1);
                mi4[u] = mr[static_cast<int64_t>(tu) * g.rows_p + r];
                li4[u] = lr[static_cast<int64_t>(tu) * g.rows_p + r];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float mi = t + u * parts < g.n_runs ? mi4[u] : -INFINITY;
                const float li = li4[u];
                if (mi > m) {
                    lsum = lsum * __builtin_amdgcn_exp2f(m - mi) + li;   // m == -inf: lsum is 0
                    m = mi;
                } else if (mi != -INFINITY) {
                    lsum += li * __builtin_amdgcn_exp2f(mi - m);
                }
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

    // chunk masses: 16 lanes per chunk, a lane holds four adjacent rows (16-byte loads), fixed-order sums
    const float* mt = ws.m_tile + static_cast<int64_t>(lh) * g.n_tiles * g.rows_p;
    const int n_chunks = g.N / g.T;
    const int sb_per_chunk = g.T / g.sb_tokens;
    const int sb_per_tile = 32 / g.sb_tokens;
    const int n_sb = g.N / g.sb_tokens;
    const float* es = ws.e_sub + static_cast<int64_t>(lh) * n_sb * g.rows_p;
    const int grp = tid >> 4, gl = tid & 15;
    // tiles of a run below the causal diagonal share the run's fast reference where there is one:
    // one bit per run (the decision is the same for every row of a head), so that the choice
    // between the two planes is known before either is loaded
    const float* mf = ws.m_fast + static_cast<int64_t>(lh) * g.n_runs * g.rows_p;
    const int first_tail_tile = (g.Nv - g.R + 1) / 32;
    // run_len is a power of two whenever a head has more than one run; sb_per_tile is 1, 2 or 4
    const int run_shift = g.n_runs > 1 ? __builtin_ctz(static_cast<unsigned>(g.run_len)) : 31;
    const int sbt_shift = __builtin_ctz(static_cast<unsigned>(sb_per_tile));
    __shared__ uint32_t fast_bits[kCombineMaxRuns / 32];
    // one run per lane, the wavefront's 64 answers collected by a ballot (loads side by side, not in turn)
    for (int t0 = tid & ~63; t0 < g.n_runs; t0 += 256) {
        const int t = t0 + (tid & 63);
        const float v = mf[static_cast<int64_t>(min(t, g.n_runs - 1)) * g.rows_p];   // row 0 exists in every head
        const uint64_t ok = __ballot(t < g.n_runs && v == v);
        if ((tid & 63) == 0) {
            fast_bits[t0 >> 5] = static_cast<uint32_t>(ok);
            fast_bits[(t0 >> 5) + 1] = static_cast<uint32_t>(ok >> 32);
        }
    }
    __syncthreads();
    // two chunks per group and pass, all their loads issued before the arithmetic: 62 registers, eight
    // wavefronts per SIMD (four chunks at four wavefronts per SIMD measured 10 % slower)
    constexpr int kUnroll = 2;
    // gridDim.y workgroups share a head's chunks (each derives the row statistics above for itself:
    // they are a few KB); a chunk belongs to exactly one group of one workgroup
    const int groups_all = 16 * static_cast<int>(gridDim.y);
    for (int c0 = (static_cast<int>(blockIdx.y) * 16 + grp) * kUnroll; c0 < n_chunks; c0 += groups_all * kUnroll) {
        float acc[kUnroll] = {};
        for (int k = 0; k < sb_per_chunk; ++k) {
            // rows_p is a multiple of 32 and the planes start 16-byte aligned: rr..rr+3 lie in one
            // aligned piece, rows at or beyond R (padding) are loaded and dropped
            for (int rr = 4 * gl; rr < g.R; rr += 64) {
                float4 mi[kUnroll], e[kUnroll];
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    const int c = min(c0 + u, n_chunks - 1);
                    const int sb = c * sb_per_chunk + k;
                    const int tile = sb >> sbt_shift;
                    const int rn = tile >> run_shift;
                    // (uniform per group: a chunk's sub-block lies in one tile)
                    const bool fast = tile < first_tail_tile && ((fast_bits[rn >> 5] >> (rn & 31)) & 1u);
                    mi[u] = *reinterpret_cast<const float4*>(fast ? mf + static_cast<int64_t>(rn) * g.rows_p + rr
                                                                  : mt + static_cast<int64_t>(tile) * g.rows_p + rr);
                    e[u] = *reinterpret_cast<const float4*>(es + static_cast<int64_t>(sb) * g.rows_p + rr);
                }
                const float4 rm = *reinterpret_cast<const float4*>(row_m + rr);
                const float4 rf = *reinterpret_cast<const float4*>(row_f + rr);
                const bool l1 = rr + 1 < g.R, l2 = rr + 2 < g.R, l3 = rr + 3 < g.R;
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    // a select, not a product with 0: what padding rows hold need not be a number
                    const float t0 = mi[u].x != -INFINITY ? e[u].x * __builtin_amdgcn_exp2f(mi[u].x - rm.x) * rf.x : 0.0f;
                    const float t1 = (l1 && mi[u].y != -INFINITY) ? e[u].y * __builtin_amdgcn_exp2f(mi[u].y - rm.y) * rf.y : 0.0f;
                    const float t2 = (l2 && mi[u].z != -INFINITY) ? e[u].z * __builtin_amdgcn_exp2f(mi[u].z - rm.z) * rf.z : 0.0f;
                    const float t3 = (l3 && mi[u].w != -INFINITY) ? e[u].w * __builtin_amdgcn_exp2f(mi[u].w - rm.w) * rf.w : 0.0f;
                    acc[u] += (t0 + t1) + (t2 + t3);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            float a = acc[u];
#pragma unroll
            for (int o = 8; o >= 1; o >>= 1) a += __shfl_xor(a, o);
            if (gl == 0 && c0 + u < n_chunks) chunk_mass[static_cast<int64_t>(lh) * n_chunks + c0 + u] = a;
        }
    }
}

// density[i] = mean over (layer, head) of chunk_mass[.][i], per token of the chunk.
// Block = 16 chunks x 64 partial sums over the (layer, head) axis (a few blocks of long
// dependent load chains would be all latency); the 64 partials are added in a fixed order,
// eight at a time.
constexpr int kDensityChunks = 16;
__global__ __launch_bounds__(1024) void score_density_kernel(const float* __restrict__ chunk_mass,
                                                             float* __restrict__ density,
                                                             int32_t n_lh, int32_t n_chunks,
                                                             float inv_norm, int32_t chunk_tokens,
                                                             int32_t n_valid) {
    constexpr int kParts = 1024 / kDensityChunks;
    __shared__ float part[kParts][kDensityChunks];
    __shared__ float part8[8][kDensityChunks];
    const int ci = threadIdx.x % kDensityChunks, p = threadIdx.x / kDensityChunks;
    const int i = blockIdx.x * kDensityChunks + ci;
    float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (i < n_chunks) {
        int k = p;
        for (; k + 3 * kParts < n_lh; k += 4 * kParts) {
#pragma unroll
            for (int u = 0; u < 4; ++u)
                acc[u] += chunk_mass[static_cast<int64_t>(k + kParts * u) * n_chunks + i];
        }
        for (; k < n_lh; k += kParts) acc[0] += chunk_mass[static_cast<int64_t>(k) * n_chunks + i];
    }
    part[p][ci] = (acc[0] + acc[1]) + (acc[2] + acc[3]);
    __syncthreads();
    if (p < 8) {
        float t = 0.0f;
#pragma unroll
        for (int k = 0; k < kParts / 8; ++k) t += part[p * (kParts / 8) + k][ci];
        part8[p][ci] = t;
    }
    __syncthreads();
    if (p == 0 && i < n_chunks) {
        float t = 0.0f;
#pragma unroll
        for (int k = 0; k < 8; ++k) t += part8[k][ci];
        // inv_norm = 1 / (chunk_tokens * n_lh); a chunk at the end of the valid tokens has fewer
        const int have = min(chunk_tokens, n_valid - i * chunk_tokens);
        density[i] = have == chunk_tokens ? t * inv_norm
                                          : (have > 0 ? t / (static_cast<float>(have) * static_cast<float>(n_lh)) : 0.0f);
    }
}

}  // namespace kvs
