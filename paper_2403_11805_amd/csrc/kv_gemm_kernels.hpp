// gfx950 GEMM for the dense projections of the recompute path (Sec. 3.3): row-major
// C[M][N] = A[M][K] * B[K][N] (+ Cin), fp16 operands, binary32 accumulation on MFMA, result in
// binary32 or rounded once to fp16.  The weights B keep their [in][out] layout and are streamed
// through LDS as they lie in memory; the MFMA operand with an output column per lane and the
// contraction index along the register comes out of the LDS transpose read (ds_read_b64_tr_b16).
//
// A workgroup of four wavefronts owns a tile of MB*32 rows x 128 columns (a wavefront: 32
// columns, MB accumulator blocks of 32x32) and walks a slice of K in steps of 32: global loads run
// three steps ahead in registers, LDS holds two steps.  With few rows (the usual case: some tens of
// chunks are recomputed beside a Load) the tiles alone do not fill 256 CUs: K is then divided among
// up to 16 workgroups per tile, each of which writes a binary32 partial tile.  The kernel that reads
// the product next adds the partial tiles in split order as it loads them (rotary encoding, the
// second norm, the gate activation: kv_recompute_kernels.hpp); gemm_reduce_kernel does it where no
// such kernel follows.  (Measured: a workgroup that counts itself in on a tile counter and, as the
// last to arrive, adds the tiles itself needs device-scope fences around the counter; with some 500
// workgroups per launch these more than double the time of a layer.)  Up to three weight matrices
// that share A (q | k | v, gate | up) go through one launch, which needs fewer splits and fewer
// launches.  All extents are guarded: M any, N and K multiples of 8.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kvs {

typedef _Float16 gv8h_t __attribute__((ext_vector_type(8)));
typedef _Float16 gv4h_t __attribute__((ext_vector_type(4)));
typedef short gv4s_t __attribute__((ext_vector_type(4)));
typedef float gv16f_t __attribute__((ext_vector_type(16)));
typedef unsigned int gu4_t __attribute__((ext_vector_type(4)));

constexpr int kGemmKStep = 32;
constexpr int kGemmXPitch = kGemmKStep + 8;  // halves per LDS row of the activation tile
constexpr int kGemmXRow = kGemmKStep / 8;    // 16-byte pieces per row of the activation tile
constexpr int kGemmMaxSplits = 16;
constexpr int kGemmMaxMats = 3;

struct GemmArgs {
    const _Float16* A;                  // [M][K]
    const _Float16* B[kGemmMaxMats];    // [K][N[j]]
    void* C[kGemmMaxMats];              // [M][N[j]] fp16 or binary32
    const _Float16* Cin;                // [M][N[0]] fp16 or NULL (added before the result is rounded; one matrix only)
    float* part;                        // matrix j: part + part_at[j], [splits][M][N[j]] binary32 (splits > 1)
    uint64_t part_at[kGemmMaxMats];
    int32_t N[kGemmMaxMats];
    int32_t tile_end[kGemmMaxMats];     // column tiles of matrices 0..j together; unused entries: the total
    int32_t M, K;
    int32_t k_slice;                    // K range of one split: a multiple of kGemmKStep
    int32_t splits;
    int32_t out_f32;
};

// Grid (column tiles of all matrices, splits, ceil(M / (MB * 32))), 256 threads; MB in {1, 2, 4}.  (Measured on MI355X: taller
// tiles - eight row blocks per wavefront, or 256 x 128 tiles with the wavefronts two by two - are slower at
// every size, 600 against 720-760 TFLOP/s at 4096 rows; the GEMM library reaches 1.2-1.4 PFLOP/s there, which
// is why the host side hands problems of more than 256 rows to it.)
template <int MB>
__global__ __launch_bounds__(256) void gemm_f16_kernel(GemmArgs g) {
    constexpr int NB = 1, WM = 1;                    // one column block per wavefront, four wavefronts side by side
    constexpr int WN = 4 / WM;
    constexpr int kCols = 32 * WN * NB;
    constexpr int kRows = 32 * WM * MB;
    constexpr int kGemmWPitch = kCols + 16;          // halves per LDS row of the weight tile
    constexpr int WPER = kGemmKStep * kCols / 8 / 256;     // 16-byte weight pieces per thread and step
    constexpr int WROW = kCols / 8;                  // pieces per weight row
    __shared__ __attribute__((aligned(16))) _Float16 wt[2][kGemmKStep * kGemmWPitch];
    __shared__ __attribute__((aligned(16))) _Float16 xt[2][kRows * kGemmXPitch];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tile = blockIdx.x;
    const int mat = (tile >= g.tile_end[0]) + (tile >= g.tile_end[1]);
    const int n0 = (tile - (mat ? g.tile_end[mat - 1] : 0)) * kCols;
    const int m0 = blockIdx.z * kRows;
    const int N = g.N[mat];
    const _Float16* __restrict__ Bm = g.B[mat];
    const int wm = wave / WN, wn = wave % WN;
    const int kb = blockIdx.y * g.k_slice;
    const int ke = min(g.K, kb + g.k_slice);
    const int n_steps = (ke - kb + kGemmKStep - 1) / kGemmKStep;
    constexpr int XPIECES = kRows * kGemmXRow;       // 16-byte pieces of an activation tile
    constexpr int XPER = (XPIECES + 255) / 256;
    constexpr int PF = 3;                            // global loads in flight: this many k-steps ahead
    gu4_t wreg[PF][WPER], xreg[PF][XPER];
    const gu4_t zero = {0u, 0u, 0u, 0u};
    // Loads are unconditional in their address (clamped into the matrices) so that they stay in flight;
    // what lies outside the tile's extents is replaced by zeros when it is parked.
    auto fetch = [&](int set, int step) __attribute__((always_inline)) {
        const int kk = kb + min(step, n_steps - 1) * kGemmKStep;
#pragma unroll
        for (int p = 0; p < WPER; ++p) {
            const int id = tid + 256 * p;            // k row id / WROW, 8 columns at (id % WROW) * 8
            const int kr = min(kk + id / WROW, g.K - 1);
            const int nc = min(n0 + (id % WROW) * 8, N - 8);
            wreg[set][p] = *reinterpret_cast<const gu4_t*>(Bm + static_cast<size_t>(kr) * N + nc);
        }
#pragma unroll
        for (int p = 0; p < XPER; ++p) {
            const int id = tid + 256 * p;
            const int row = min(m0 + min(id / kGemmXRow, kRows - 1), g.M - 1);
            const int kc = min(kk + (id % kGemmXRow) * 8, g.K - 8);
            xreg[set][p] = *reinterpret_cast<const gu4_t*>(g.A + static_cast<size_t>(row) * g.K + kc);
        }
    };
    auto park = [&](int set, int buf, int step) __attribute__((always_inline)) {
        const int kk = kb + step * kGemmKStep;
#pragma unroll
        for (int p = 0; p < WPER; ++p) {
            const int id = tid + 256 * p;
            const bool in = kk + id / WROW < ke && n0 + (id % WROW) * 8 < N;
            *reinterpret_cast<gu4_t*>(&wt[buf][(id / WROW) * kGemmWPitch + (id % WROW) * 8]) = in ? wreg[set][p] : zero;
        }
#pragma unroll
        for (int p = 0; p < XPER; ++p) {
            const int id = tid + 256 * p;
            if (id < XPIECES) {
                const bool in = kk + (id % kGemmXRow) * 8 < ke;      // rows beyond M repeat row M - 1 and are never stored
                *reinterpret_cast<gu4_t*>(&xt[buf][(id / kGemmXRow) * kGemmXPitch + (id % kGemmXRow) * 8]) =
                    in ? xreg[set][p] : zero;
            }
        }
    };
    gv16f_t acc[NB][MB];
#pragma unroll
    for (int c = 0; c < NB; ++c)
#pragma unroll
        for (int b = 0; b < MB; ++b) acc[c][b] = gv16f_t{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    const int grp = lane >> 4, i16 = lane & 15;
    auto compute = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int ks = 0; ks < kGemmKStep / 16; ++ks) {
            // B operand: column wave*32 + lane%32, rows ks*16 + 8*(lane/32) + 0..7, through two transpose reads:
            // the 16 lanes of a group hand in sixteen 8-byte pieces of a 4-row x 16-column block and lane i
            // receives the four rows of column i
            const int krow = ks * 16 + 8 * (grp >> 1);
            gv8h_t b[NB];
#pragma unroll
            for (int c = 0; c < NB; ++c) {
                const int ncol = c * (32 * WN) + wn * 32 + 16 * (grp & 1);
                const _Float16* wa = &wt[buf][(krow + (i16 >> 2)) * kGemmWPitch + ncol + 4 * (i16 & 3)];
                const gv4s_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) gv4s_t*)wa);
                const gv4s_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) gv4s_t*)(wa + 4 * kGemmWPitch));
                const gv4h_t lo_h = __builtin_bit_cast(gv4h_t, lo), hi_h = __builtin_bit_cast(gv4h_t, hi);
                b[c] = gv8h_t{lo_h[0], lo_h[1], lo_h[2], lo_h[3], hi_h[0], hi_h[1], hi_h[2], hi_h[3]};
            }
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                const gv8h_t a = *reinterpret_cast<const gv8h_t*>(
                    &xt[buf][((wm * MB + mb) * 32 + (lane & 31)) * kGemmXPitch + ks * 16 + 8 * (lane >> 5)]);
#pragma unroll
                for (int c = 0; c < NB; ++c) acc[c][mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b[c], acc[c][mb], 0, 0, 0);
            }
        }
    };
    // step s lives in register set s % 3 and LDS buffer s % 2; six steps per trip keep both indices static
    fetch(0, 0);
    fetch(1, 1);
    fetch(2, 2);
    park(0, 0, 0);
    __syncthreads();
    auto one = [&](int step, int set, int buf) __attribute__((always_inline)) {
        if (step < n_steps) {                        // uniform
            fetch(set, step + 3);                    // this step's set is free: it was parked before the last barrier
            compute(buf);
            if (step + 1 < n_steps) park((set + 1) % 3, buf ^ 1, step + 1);
            __syncthreads();
        }
    };
    for (int step = 0; step < n_steps; step += 6) {
        one(step + 0, 0, 0);
        one(step + 1, 1, 1);
        one(step + 2, 2, 0);
        one(step + 3, 0, 1);
        one(step + 4, 1, 0);
        one(step + 5, 2, 1);
    }
    // acc[c][mb][v]: row m0 + (wm*MB + mb)*32 + 8*(v/4) + 4*(lane/32) + v%4, column n0 + c*WN*32 + wn*32 + lane%32
    if (g.splits == 1) {
#pragma unroll
        for (int c = 0; c < NB; ++c) {
            const int n = n0 + c * (32 * WN) + wn * 32 + (lane & 31);
            if (n >= N) continue;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = m0 + (wm * MB + mb) * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v % 4);
                    if (m < g.M) {
                        const size_t at = static_cast<size_t>(m) * N + n;
                        float r = acc[c][mb][v];
                        if (g.Cin) r += static_cast<float>(g.Cin[at]);
                        if (g.out_f32) static_cast<float*>(g.C[mat])[at] = r;
                        else static_cast<_Float16*>(g.C[mat])[at] = static_cast<_Float16>(r);
                    }
                }
        }
        return;
    }
    float* dst = g.part + g.part_at[mat] + blockIdx.y * (static_cast<size_t>(g.M) * N);
#pragma unroll
    for (int c = 0; c < NB; ++c) {
        const int n = n0 + c * (32 * WN) + wn * 32 + (lane & 31);
        if (n >= N) continue;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + (wm * MB + mb) * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v % 4);
                if (m < g.M) dst[static_cast<size_t>(m) * N + n] = acc[c][mb][v];
            }
    }
}

// C[0] = sum of matrix 0's partial tiles in split order + Cin, rounded once; four adjacent columns per thread.
__global__ __launch_bounds__(256) void gemm_reduce_kernel(GemmArgs g) {
    typedef float f4_t __attribute__((ext_vector_type(4)));
    const size_t n4 = static_cast<size_t>(g.M) * g.N[0] / 4;
    const size_t i = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i >= n4) return;
    const f4_t* part = reinterpret_cast<const f4_t*>(g.part);
    f4_t a = part[i];
    for (int s = 1; s < g.splits; ++s) a += part[static_cast<size_t>(s) * n4 + i];
    if (g.Cin) {
        const gv4h_t c = reinterpret_cast<const gv4h_t*>(g.Cin)[i];
        a += f4_t{static_cast<float>(c[0]), static_cast<float>(c[1]), static_cast<float>(c[2]), static_cast<float>(c[3])};
    }
    if (g.out_f32) {
        reinterpret_cast<f4_t*>(g.C[0])[i] = a;
    } else {
        const gv4h_t h = {static_cast<_Float16>(a[0]), static_cast<_Float16>(a[1]), static_cast<_Float16>(a[2]),
                          static_cast<_Float16>(a[3])};
        reinterpret_cast<gv4h_t*>(g.C[0])[i] = h;
    }
}

}  // namespace kvs
