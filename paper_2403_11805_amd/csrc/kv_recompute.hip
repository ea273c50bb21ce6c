// libkvswitch: recompute of interleaved chunks through one Llama-style block
// (Sec. 3.3, "Making interleaved chunks recomputable").  Host side: argument
// checks, the workspace plan, the dense projections and the launches of the
// kernels in kv_recompute_kernels.hpp.  The projections of up to kHandGemmRows
// recomputed tokens - what a plan of Eq. 4 recomputes beside a Load - run on the
// library's own MFMA GEMM (kv_gemm_kernels.hpp); larger ones go to rocBLAS, which
// is loaded at run time if it is there (the rest of the library does not depend
// on it, and without it every size runs on the library's own kernel).

#include <dlfcn.h>
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <new>
#include <vector>

#include "kv_gemm_kernels.hpp"
#include "kv_internal.h"
#include "kv_recompute_kernels.hpp"

using namespace kvs;

namespace {

// The few rocBLAS entry points used, with the library's published C signatures and enum values.
typedef void* rb_handle;
typedef int (*rb_create_fn)(rb_handle*);
typedef int (*rb_destroy_fn)(rb_handle);
typedef int (*rb_set_stream_fn)(rb_handle, hipStream_t);
typedef int (*rb_gemm_ex_fn)(rb_handle, int, int, int, int, int, const void*, const void*, int, int,
                             const void*, int, int, const void*, const void*, int, int, void*, int, int,
                             int, int, int32_t, uint32_t);
constexpr int kRbOpNone = 111;        // rocblas_operation_none
constexpr int kRbF16 = 150;           // rocblas_datatype_f16_r
constexpr int kRbF32 = 151;           // rocblas_datatype_f32_r
constexpr int kRbAlgoStandard = 0;    // rocblas_gemm_algo_standard
constexpr int kRbAlgoSolution = 1;    // rocblas_gemm_algo_solution_index
// Lists the library's kernels ("solutions") that can run a given gemm_ex call (same arguments,
// then flags, list, list size; a NULL list returns the count).
typedef int (*rb_get_solutions_fn)(rb_handle, int, int, int, int, int, const void*, const void*, int, int,
                                   const void*, int, int, const void*, const void*, int, int, void*, int, int,
                                   int, int, uint32_t, int*, int*);

uint64_t align256(uint64_t v) { return (v + 255) & ~static_cast<uint64_t>(255); }

struct Plan {
    uint64_t xn, q32, k32, v32, q16, attn, x1, gate, up, part_o, part_ml, gemm_part, total;
    int splits;          // workgroups that share the key range of one attention row block (1: no split)
};

// Measured on MI355X (Llama-2-7B layer; the seven projections in us, the library's after kv_recompute_tune,
// and the whole layer in ms):
//   128 rows   own 164   library 266   layer 0.27 against 0.34
//   256 rows   own 211   library 253   layer 0.32 against 0.35
//   512 rows   own 349   library 363   layer 0.47 against 0.49
//   1024 rows  own 640   library 474   layer 0.79 against 0.67
//   4096 rows  own 2200 (750 TFLOP/s)   library 1420 (1.2-1.4 PFLOP/s)
constexpr int64_t kHandGemmRows = KV_RECOMPUTE_OWN_GEMM_ROWS;

// Up to three weight matrices [K][N[j]] applied to the same activations in one launch.
struct GemmGroup {
    int n;
    int64_t N[kGemmMaxMats];
    const void* B[kGemmMaxMats];
    void* C[kGemmMaxMats];
};

// Launch shape of the library's own GEMM: row blocks per tile, K range per split, number of splits.
struct HandGemm {
    int mb, k_slice, splits;
    uint32_t tiles_n, tiles_m;
    uint64_t part_bytes;
};

HandGemm hand_gemm_plan(int64_t M, const int64_t* N, int n_mats, int64_t K) {
    HandGemm h;
    h.mb = M <= 32 ? 1 : (M <= 64 ? 2 : 4);
    h.tiles_n = 0;
    int64_t n_sum = 0;
    for (int j = 0; j < n_mats; ++j) {
        h.tiles_n += static_cast<uint32_t>((N[j] + 127) / 128);
        n_sum += N[j];
    }
    h.tiles_m = static_cast<uint32_t>((M + h.mb * 32 - 1) / (h.mb * 32));
    // K is divided until some 512 workgroups exist (two per CU), at least 256 of K per split.  Up to 128
    // rows 256 workgroups are as fast (measured: the four launches of a layer take 164-168 us with 256,
    // 384, 512 and 768 workgroups) and leave half the partial products for the next kernel to add.
    const int64_t tiles = static_cast<int64_t>(h.tiles_n) * h.tiles_m;
    const int64_t groups = M <= 128 ? 256 : 512;
    int64_t want = (groups + tiles - 1) / tiles;
    want = std::min<int64_t>(want, std::min<int64_t>(kGemmMaxSplits, std::max<int64_t>(1, K / 256)));
    h.k_slice = static_cast<int>(((K + want - 1) / want + kGemmKStep - 1) / kGemmKStep * kGemmKStep);
    h.splits = static_cast<int>((K + h.k_slice - 1) / h.k_slice);
    h.part_bytes = h.splits > 1 ? static_cast<uint64_t>(h.splits) * M * n_sum * 4u : 0u;
    return h;
}

// With few recomputed rows the attention kernel has too few workgroups to fill 256 CUs: the key
// range is then divided among up to 16 workgroups (one workgroup per CU in total: measured, more
// shares cost more in partial results than they gain; at least four key tiles per share, at most
// 64 MiB of partial results).
int attention_splits(const kv_shape_t& s, int64_t M) {
    const int64_t pairs = static_cast<int64_t>(s.n_q_heads / s.n_kv_heads) * ((M + 31) / 32);
    const int64_t base = (pairs + kAttnWaves - 1) / kAttnWaves * s.n_kv_heads;
    int64_t splits = 256 / base;
    splits = std::min<int64_t>(splits, (s.n_tokens + 31) / 32 / 4);
    splits = std::min<int64_t>(splits, kMaxSplits);
    const int64_t per_split = M * s.n_q_heads * (s.head_dim + 2) * 4;
    splits = std::min<int64_t>(splits, (64ll << 20) / per_split);
    return static_cast<int>(std::max<int64_t>(splits, 1));
}

Plan plan_workspace(const kv_shape_t& s, const kv_layer_dims_t& d, int64_t M) {
    const uint64_t dq = static_cast<uint64_t>(s.n_q_heads) * s.head_dim;
    const uint64_t dkv = static_cast<uint64_t>(s.n_kv_heads) * s.head_dim;
    Plan p;
    uint64_t o = 0;
    p.xn = o;   o += align256(M * d.d_model * 2u);
    p.q32 = o;  o += align256(M * dq * 4u);
    p.k32 = o;  o += align256(M * dkv * 4u);
    p.v32 = o;  o += align256(M * dkv * 4u);
    p.q16 = o;  o += align256(M * dq * 2u);
    p.attn = o; o += align256(M * dq * 2u);
    p.x1 = o;   o += align256(M * d.d_model * 2u);
    p.gate = o; o += align256(M * static_cast<uint64_t>(d.d_ff) * 2u);
    p.up = o;   o += align256(M * static_cast<uint64_t>(d.d_ff) * 2u);
    p.splits = attention_splits(s, M);
    p.part_o = o;
    if (p.splits > 1) o += align256(static_cast<uint64_t>(p.splits) * M * dq * 4u);
    p.part_ml = o;
    if (p.splits > 1) o += align256(static_cast<uint64_t>(p.splits) * M * s.n_q_heads * 8u);
    // the library's own GEMM: partial tiles of the largest of its four launches
    const int64_t n_qkv[3] = {static_cast<int64_t>(dq), static_cast<int64_t>(dkv), static_cast<int64_t>(dkv)};
    const int64_t n_o[1] = {d.d_model}, n_ff[2] = {d.d_ff, d.d_ff};
    const HandGemm hg[4] = {hand_gemm_plan(M, n_qkv, 3, d.d_model), hand_gemm_plan(M, n_o, 1, static_cast<int64_t>(dq)),
                            hand_gemm_plan(M, n_ff, 2, d.d_model), hand_gemm_plan(M, n_o, 1, d.d_ff)};
    uint64_t part = 0;
    for (const HandGemm& h : hg) part = std::max(part, h.part_bytes);
    p.gemm_part = o;
    o += align256(part);
    p.total = o;
    return p;
}

int check_layer(const kv_shape_t* shape, const kv_layer_dims_t* dims, int32_t n_missing) {
    if (int rc = check_shape(shape)) return rc;
    if (!dims) return fail(KV_EINVAL, "dims is NULL");
    if (!is_f16(*shape)) return fail(KV_ESHAPE, "recompute needs an fp16 cache format");
    if (shape->head_dim != 64 && shape->head_dim != 128)
        return fail(KV_ESHAPE, "recompute needs head_dim 64 or 128, got %d", shape->head_dim);
    if (dims->d_model <= 0 || dims->d_model % 8 || dims->d_ff <= 0 || dims->d_ff % 8)
        return fail(KV_ESHAPE, "d_model %d and d_ff %d must be positive multiples of 8", dims->d_model, dims->d_ff);
    if (!(dims->rope_base > 1.0f) || !(dims->rms_eps >= 0.0f))
        return fail(KV_EINVAL, "rope_base must exceed 1 and rms_eps must not be negative");
    const int32_t n_chunks = shape->n_tokens / shape->chunk_tokens;
    if (n_missing < 1 || n_missing > n_chunks)
        return fail(KV_EINVAL, "n_missing %d outside [1,%d]", n_missing, n_chunks);
    return KV_OK;
}

}  // namespace

// One projection of the block: row-major C[M][N] = A[M][K] * B[K][N] (+ Cin), fp16 operands.
struct GemmShape {
    int64_t M, N, K;
    bool out_f32, add;
    bool operator==(const GemmShape& o) const {
        return M == o.M && N == o.N && K == o.K && out_f32 == o.out_f32 && add == o.add;
    }
};

struct kv_recompute {
    void* lib = nullptr;
    rb_handle handle = nullptr;
    rb_destroy_fn destroy = nullptr;
    rb_set_stream_fn set_stream = nullptr;
    rb_gemm_ex_fn gemm_ex = nullptr;
    rb_get_solutions_fn get_solutions = nullptr;     // optional
    std::vector<std::pair<GemmShape, int>> tuned;    // shapes kv_recompute_tune examined: kernel, or -1 = standard
};

namespace {

// The GEMM library's status for C[M][N] = A * B (+ Cin) with the standard choice of kernel
// (solution < 0) or a given one.  Column-major view: Cout^T [N][M] = B^T [N][K] * A^T [K][M].
int gemm_status(kv_recompute* rc, const GemmShape& g, const void* A, const void* B, const void* Cin, void* Cout,
                int solution) {
    const float alpha = 1.0f, beta = g.add ? 1.0f : 0.0f;
    const int ct = g.out_f32 ? kRbF32 : kRbF16;
    return rc->gemm_ex(rc->handle, kRbOpNone, kRbOpNone, static_cast<int>(g.N), static_cast<int>(g.M),
                       static_cast<int>(g.K), &alpha, B, kRbF16, static_cast<int>(g.N), A, kRbF16,
                       static_cast<int>(g.K), &beta, g.add ? Cin : Cout, ct, static_cast<int>(g.N), Cout, ct,
                       static_cast<int>(g.N), kRbF32, solution < 0 ? kRbAlgoStandard : kRbAlgoSolution,
                       solution < 0 ? 0 : solution, 0);
}

// The library's own GEMM (kv_gemm_kernels.hpp) over a group of weight matrices; `part` holds what hand_gemm_plan
// asks for.  With `splits_left` a product that was divided along K stays in `part` as *splits_left > 1 partial
// products per matrix ([splits][M][N[j]], matrix after matrix) for the caller's next kernel to add; otherwise
// (one matrix only) it is added here.
int hand_gemm(hipStream_t st, int64_t M, int64_t K, const void* A, const GemmGroup& grp, const void* Cin,
              bool out_f32, float* part, int* splits_left, const char* what) {
    if (splits_left) *splits_left = 1;
    if (!splits_left && grp.n != 1) return fail(KV_EINVAL, "GEMM (%s): a group is added by its reader", what);
    if (K % 8 || K < 8 || M < 1 || grp.n < 1 || grp.n > kGemmMaxMats || (Cin && grp.n != 1))
        return fail(KV_ESHAPE, "GEMM (%s): unsupported shape", what);
    for (int j = 0; j < grp.n; ++j)
        if (grp.N[j] % 8 || grp.N[j] < 8) return fail(KV_ESHAPE, "GEMM (%s) needs N a multiple of 8", what);
    const HandGemm h = hand_gemm_plan(M, grp.N, grp.n, K);
    GemmArgs g;
    g.A = static_cast<const _Float16*>(A);
    g.Cin = static_cast<const _Float16*>(Cin);
    g.part = part;
    int32_t tiles = 0;
    uint64_t at = 0;
    for (int j = 0; j < kGemmMaxMats; ++j) {
        const int k = std::min(j, grp.n - 1);                 // unused entries repeat the last matrix and get no tile
        g.B[j] = static_cast<const _Float16*>(grp.B[k]);
        g.C[j] = grp.C[k];
        g.N[j] = static_cast<int32_t>(grp.N[k]);
        g.part_at[j] = at;
        if (j < grp.n) {
            tiles += static_cast<int32_t>((grp.N[j] + 127) / 128);
            at += static_cast<uint64_t>(h.splits) * M * grp.N[j];
        }
        g.tile_end[j] = tiles;
    }
    g.M = static_cast<int32_t>(M);
    g.K = static_cast<int32_t>(K);
    g.k_slice = h.k_slice;
    g.splits = h.splits;
    g.out_f32 = out_f32 ? 1 : 0;
    const dim3 grid(h.tiles_n, static_cast<uint32_t>(h.splits), h.tiles_m);
    if (h.mb == 1) hipLaunchKernelGGL(gemm_f16_kernel<1>, grid, dim3(256), 0, st, g);
    else if (h.mb == 2) hipLaunchKernelGGL(gemm_f16_kernel<2>, grid, dim3(256), 0, st, g);
    else hipLaunchKernelGGL(gemm_f16_kernel<4>, grid, dim3(256), 0, st, g);
    if (h.splits > 1) {
        if (splits_left) *splits_left = h.splits;
        else hipLaunchKernelGGL(gemm_reduce_kernel, dim3(static_cast<uint32_t>((M * grp.N[0] / 4 + 255) / 256)),
                                dim3(256), 0, st, g);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(KV_EHIP, "gemm_f16_kernel launch (%s): %s", what, hipGetErrorString(e));
    return KV_OK;
}

// The projections of a group: one launch of the library's own kernel, or one GEMM of the library per matrix.
int gemm(kv_recompute* rc, hipStream_t stream, float* part, int* splits_left, int64_t M, int64_t K, const void* A,
         const GemmGroup& grp, const void* Cin, bool out_f32, const char* what) {
    if (M <= kHandGemmRows || !rc->gemm_ex)
        return hand_gemm(stream, M, K, A, grp, Cin, out_f32, part, splits_left, what);
    if (splits_left) *splits_left = 1;
    for (int j = 0; j < grp.n; ++j) {
        const GemmShape g = {M, grp.N[j], K, out_f32, Cin != nullptr};
        int solution = -1;
        for (const auto& t : rc->tuned)
            if (t.first == g) solution = t.second;
        const int st = gemm_status(rc, g, A, grp.B[j], Cin, grp.C[j], solution);
        if (st != 0) return fail(KV_EHIP, "rocblas_gemm_ex (%s, matrix %d) failed with status %d", what, j, st);
    }
    return KV_OK;
}

// One projection of a block with its operands.
struct GemmJob {
    GemmShape g;
    const void* A;
    const void* B;
    const void* Cin;
    void* Cout;
};

// Picks the kernel of jobs[which] in two passes.  Pass 1 times every kernel the library lists
// back to back, which ranks them with the weights sitting in the last-level cache; pass 2 times
// the standard choice and the best few of pass 1 with cold weights, as a layer meets them: the
// other projections of the block (several hundred MB of weights) run in between.  The fastest of
// pass 2 is remembered if it beats the standard choice by more than 5 %.  Synchronises `st`.
int tune_gemm(kv_recompute* rc, const GemmJob* jobs, int n_jobs, int which, hipStream_t st, hipEvent_t e0,
              hipEvent_t e1, int* improved) {
    const GemmJob& job = jobs[which];
    const GemmShape& g = job.g;
    for (const auto& t : rc->tuned)
        if (t.first == g) return KV_OK;                       // already tuned
    const float alpha = 1.0f, beta = g.add ? 1.0f : 0.0f;
    const int ct = g.out_f32 ? kRbF32 : kRbF16;
    int n = 0;
    auto list = [&](int* out, int* count) {
        return rc->get_solutions(rc->handle, kRbOpNone, kRbOpNone, static_cast<int>(g.N), static_cast<int>(g.M),
                                 static_cast<int>(g.K), &alpha, job.B, kRbF16, static_cast<int>(g.N), job.A, kRbF16,
                                 static_cast<int>(g.K), &beta, g.add ? job.Cin : job.Cout, ct, static_cast<int>(g.N),
                                 job.Cout, ct, static_cast<int>(g.N), kRbF32, kRbAlgoSolution, 0, out, count);
    };
    if (list(nullptr, &n) != 0 || n <= 0) return KV_OK;      // nothing to choose from
    std::vector<int> sols(static_cast<size_t>(n));
    if (list(sols.data(), &n) != 0) return KV_OK;
    auto run = [&](int solution) { return gemm_status(rc, g, job.A, job.B, job.Cin, job.Cout, solution); };
    // elapsed time of `reps` runs; 1: this kernel cannot run the problem; -1: the runtime failed
    auto time_ms = [&](int solution, int reps, float* ms) -> int {
        hipError_t e = hipEventRecord(e0, st);
        for (int r = 0; r < reps && e == hipSuccess; ++r)
            if (run(solution) != 0) return 1;
        if (e == hipSuccess) e = hipEventRecord(e1, st);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        if (e == hipSuccess) e = hipEventElapsedTime(ms, e0, e1);
        return e == hipSuccess ? 0 : -1;
    };
    constexpr int kKeep = 6;
    int keep[kKeep];
    float keep_ms[kKeep];
    int n_keep = 0;
    for (int i = 0; i < n; ++i) {
        const int sol = sols[static_cast<size_t>(i)];
        float t = 0.0f;
        if (run(sol) != 0) continue;                          // warm-up, and "can it run"
        const int rc_t = time_ms(sol, 3, &t);
        if (rc_t < 0) return fail(KV_EHIP, "timing a GEMM kernel failed");
        if (rc_t != 0) continue;
        int at;                                               // insertion into the sorted short list
        if (n_keep < kKeep) at = n_keep++;
        else if (t < keep_ms[kKeep - 1]) at = kKeep - 1;
        else continue;
        while (at > 0 && keep_ms[at - 1] > t) {
            keep[at] = keep[at - 1];
            keep_ms[at] = keep_ms[at - 1];
            --at;
        }
        keep[at] = sol;
        keep_ms[at] = t;
    }
    auto cold_ms = [&](int solution, float* ms) -> int {
        *ms = 1e30f;
        for (int rep = 0; rep < 3; ++rep) {
            for (int k = 0; k < n_jobs; ++k)                  // push this job's weights out of the cache
                if (jobs[k].B != job.B) {
                    const GemmJob& o = jobs[k];
                    if (gemm_status(rc, o.g, o.A, o.B, o.Cin, o.Cout, -1) != 0) return -1;
                }
            float t = 0.0f;
            const int rc_t = time_ms(solution, 1, &t);
            if (rc_t != 0) return rc_t;
            if (t < *ms) *ms = t;
        }
        return 0;
    };
    float t_std = 0.0f;
    if (cold_ms(-1, &t_std) != 0) return fail(KV_EHIP, "timing the standard GEMM kernel failed");
    float t_best = t_std;
    int best = -1;
    for (int i = 0; i < n_keep; ++i) {
        float t = 0.0f;
        const int rc_t = cold_ms(keep[i], &t);
        if (rc_t < 0) return fail(KV_EHIP, "timing a GEMM kernel failed");
        if (rc_t == 0 && t < t_best) {
            t_best = t;
            best = keep[i];
        }
    }
    const bool better = best >= 0 && t_best < 0.95f * t_std;
    rc->tuned.emplace_back(g, better ? best : -1);            // examined: not timed again
    if (better) ++*improved;
    return KV_OK;
}

}  // namespace

extern "C" {

kv_recompute_t* kv_recompute_create(void) {
    clear_error();
    kv_recompute* rc = new (std::nothrow) kv_recompute();
    if (!rc) {
        fail(KV_ENOMEM, "out of host memory");
        return nullptr;
    }
    // KVSWITCH_OWN_GEMM=1 in the environment keeps the GEMM library out: every projection then runs
    // on the library's own kernel, as it does where rocBLAS is not installed
    const char* own = getenv("KVSWITCH_OWN_GEMM");
    if (own && own[0] == '1') return rc;
    rc->lib = dlopen("librocblas.so.5", RTLD_NOW | RTLD_LOCAL);
    if (!rc->lib) rc->lib = dlopen("librocblas.so", RTLD_NOW | RTLD_LOCAL);
    if (!rc->lib) return rc;
    rb_create_fn create = reinterpret_cast<rb_create_fn>(dlsym(rc->lib, "rocblas_create_handle"));
    rc->destroy = reinterpret_cast<rb_destroy_fn>(dlsym(rc->lib, "rocblas_destroy_handle"));
    rc->set_stream = reinterpret_cast<rb_set_stream_fn>(dlsym(rc->lib, "rocblas_set_stream"));
    rc->gemm_ex = reinterpret_cast<rb_gemm_ex_fn>(dlsym(rc->lib, "rocblas_gemm_ex"));
    rc->get_solutions = reinterpret_cast<rb_get_solutions_fn>(dlsym(rc->lib, "rocblas_gemm_ex_get_solutions"));
    if (!create || !rc->destroy || !rc->set_stream || !rc->gemm_ex) {
        fail(KV_EHIP, "rocBLAS lacks a required entry point");
        dlclose(rc->lib);
        delete rc;
        return nullptr;
    }
    const int st = create(&rc->handle);
    if (st != 0 || !rc->handle) {
        fail(KV_EHIP, "rocblas_create_handle failed with status %d", st);
        dlclose(rc->lib);
        delete rc;
        return nullptr;
    }
    return rc;
}

void kv_recompute_destroy(kv_recompute_t* rc) {
    if (!rc) return;
    if (rc->handle && rc->destroy) rc->destroy(rc->handle);
    // the library stays loaded: other users in the process may share it
    delete rc;
}

uint64_t kv_recompute_workspace_bytes(const kv_shape_t* shape, const kv_layer_dims_t* dims, int32_t n_missing) {
    if (check_layer(shape, dims, n_missing) != KV_OK) return 0;
    return plan_workspace(*shape, *dims, static_cast<int64_t>(n_missing) * shape->chunk_tokens).total;
}

int32_t kv_recompute_tune(kv_recompute_t* rc, const kv_shape_t* shape, const kv_layer_dims_t* dims,
                          const kv_layer_weights_t* w, int32_t n_missing, void* workspace,
                          uint64_t workspace_bytes, void* stream, int32_t* n_improved) {
    if (n_improved) *n_improved = 0;
    if (!rc) return fail(KV_EINVAL, "handle is NULL");
    if (int st = check_layer(shape, dims, n_missing)) return st;
    if (!w || !w->wq || !w->wk || !w->wv || !w->wo || !w->w_gate || !w->w_up || !w->w_down)
        return fail(KV_EINVAL, "a weight pointer is NULL");
    if (!workspace || !aligned(workspace, 256)) return fail(KV_EINVAL, "workspace must be a 256-byte aligned device pointer");
    const kv_shape_t& s = *shape;
    const int64_t M = static_cast<int64_t>(n_missing) * s.chunk_tokens;
    const Plan p = plan_workspace(s, *dims, M);
    if (workspace_bytes < p.total)
        return fail(KV_ENOMEM, "workspace %llu bytes, %llu needed", static_cast<unsigned long long>(workspace_bytes),
                    static_cast<unsigned long long>(p.total));
    // projections of few rows run on the library's own kernel; nothing to choose there, nor without a GEMM library
    if (M <= kHandGemmRows || !rc->gemm_ex || !rc->get_solutions) return KV_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (rc->set_stream(rc->handle, st) != 0) return fail(KV_EHIP, "rocblas_set_stream failed");
    // operands of ordinary magnitude and varied bits in every buffer a GEMM reads
    const int64_t n_words = static_cast<int64_t>(p.total / 4);
    hipLaunchKernelGGL(fill_noise_kernel, dim3(static_cast<uint32_t>((n_words + 255) / 256)), dim3(256), 0, st,
                       static_cast<uint32_t*>(workspace), n_words);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(KV_EHIP, "fill_noise_kernel launch: %s", hipGetErrorString(e));
    hipEvent_t e0 = nullptr, e1 = nullptr;
    e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    if (e != hipSuccess) {
        if (e0) (void)hipEventDestroy(e0);
        return fail(KV_EHIP, "hipEventCreate: %s", hipGetErrorString(e));
    }
    uint8_t* base = static_cast<uint8_t*>(workspace);
    void *xn = base + p.xn, *q32 = base + p.q32, *k32 = base + p.k32, *attn = base + p.attn, *x1 = base + p.x1,
         *gate = base + p.gate;
    const int64_t dq = static_cast<int64_t>(s.n_q_heads) * s.head_dim;
    const int64_t dkv = static_cast<int64_t>(s.n_kv_heads) * s.head_dim;
    void* up = base + p.up;
    void* v32 = base + p.v32;
    const GemmShape gq = {M, dq, dims->d_model, true, false}, gk = {M, dkv, dims->d_model, true, false};
    const GemmShape go = {M, dims->d_model, dq, false, true}, gg = {M, dims->d_ff, dims->d_model, false, false};
    const GemmShape gd = {M, dims->d_model, dims->d_ff, false, true};
    const GemmJob jobs[7] = {{gq, xn, w->wq, nullptr, q32}, {gk, xn, w->wk, nullptr, k32}, {gk, xn, w->wv, nullptr, v32},
                             {go, attn, w->wo, xn, x1},     {gg, xn, w->w_gate, nullptr, gate},
                             {gg, xn, w->w_up, nullptr, up}, {gd, gate, w->w_down, x1, xn}};
    int improved = 0;
    int rcode = KV_OK;
    for (int which : {0, 1, 3, 4, 6})
        if (!rcode) rcode = tune_gemm(rc, jobs, 7, which, st, e0, e1, &improved);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (n_improved) *n_improved = improved;
    return rcode;
}

int32_t kv_recompute_layer(kv_recompute_t* rc, const kv_shape_t* shape, const kv_layer_dims_t* dims,
                           const kv_layer_weights_t* w, int32_t layer, const int32_t* chunk_idx_dev,
                           int32_t n_missing, const void* x_in, void* kv, void* x_out, void* workspace,
                           uint64_t workspace_bytes, void* stream) {
    if (!rc) return fail(KV_EINVAL, "handle is NULL");
    if (int st = check_layer(shape, dims, n_missing)) return st;
    if (layer < 0 || layer >= shape->n_layers) return fail(KV_EINVAL, "layer %d outside [0,%d)", layer, shape->n_layers);
    if (!w || !w->w_norm1 || !w->wq || !w->wk || !w->wv || !w->wo || !w->w_norm2 || !w->w_gate || !w->w_up ||
        !w->w_down)
        return fail(KV_EINVAL, "a weight pointer is NULL");
    if (!chunk_idx_dev || !x_in || !kv || !x_out || !workspace) return fail(KV_EINVAL, "NULL device pointer");
    if (!aligned(x_in, 16) || !aligned(x_out, 16) || !aligned(kv, 16) || !aligned(workspace, 256) ||
        !aligned(chunk_idx_dev, 4))
        return fail(KV_EINVAL, "x_in/x_out/kv must be 16-byte aligned, workspace 256-byte aligned");
    const void* ws_ptrs[] = {w->w_norm1, w->wq, w->wk, w->wv, w->wo, w->w_norm2, w->w_gate, w->w_up, w->w_down};
    for (const void* p : ws_ptrs)
        if (!aligned(p, 16)) return fail(KV_EINVAL, "weights must be 16-byte aligned");
    const kv_shape_t& s = *shape;
    const int64_t M = static_cast<int64_t>(n_missing) * s.chunk_tokens;
    const Plan p = plan_workspace(s, *dims, M);
    if (workspace_bytes < p.total)
        return fail(KV_ENOMEM, "workspace %llu bytes, %llu needed", static_cast<unsigned long long>(workspace_bytes),
                    static_cast<unsigned long long>(p.total));
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (rc->gemm_ex && M > kHandGemmRows && rc->set_stream(rc->handle, st) != 0)
        return fail(KV_EHIP, "rocblas_set_stream failed");

    uint8_t* base = static_cast<uint8_t*>(workspace);
    float* gpart = reinterpret_cast<float*>(base + p.gemm_part);
    _Float16* xn = reinterpret_cast<_Float16*>(base + p.xn);
    float* q32 = reinterpret_cast<float*>(base + p.q32);
    float* k32 = reinterpret_cast<float*>(base + p.k32);
    float* v32 = reinterpret_cast<float*>(base + p.v32);
    _Float16* q16 = reinterpret_cast<_Float16*>(base + p.q16);
    _Float16* attn = reinterpret_cast<_Float16*>(base + p.attn);
    _Float16* x1 = reinterpret_cast<_Float16*>(base + p.x1);
    _Float16* gate = reinterpret_cast<_Float16*>(base + p.gate);
    _Float16* up = reinterpret_cast<_Float16*>(base + p.up);
    const _Float16* xin = static_cast<const _Float16*>(x_in);
    const int D = s.head_dim, Hq = s.n_q_heads, Hkv = s.n_kv_heads;
    const int64_t dq = static_cast<int64_t>(Hq) * D, dkv = static_cast<int64_t>(Hkv) * D;
    _Float16* k_plane = static_cast<_Float16*>(kv) + (static_cast<int64_t>(layer) * 2 + 0) * Hkv * s.n_tokens * D;
    _Float16* v_plane = k_plane + static_cast<int64_t>(Hkv) * s.n_tokens * D;
    const dim3 rows(static_cast<uint32_t>((M + 3) / 4));

    // 1. norm, q/k/v projections (binary32 results, rounded once after the rotation)
    // (a product whose K range was divided stays in `gpart` as partial products, which the next kernel adds)
    const float* no_part = nullptr;
    hipLaunchKernelGGL(rmsnorm_kernel, rows, dim3(256), 0, st, xin, static_cast<const _Float16*>(w->w_norm1), xn,
                       static_cast<int32_t>(M), dims->d_model, dims->rms_eps);
    int sp = 1;
    const GemmGroup qkv = {3, {dq, dkv, dkv}, {w->wq, w->wk, w->wv}, {q32, k32, v32}};
    if (int e = gemm(rc, st, gpart, &sp, M, dims->d_model, xn, qkv, nullptr, true, "q | k | v")) return e;
    const float* q_src = sp > 1 ? gpart : q32;
    const float* k_src = sp > 1 ? gpart + sp * M * dq : k32;
    const float* v_src = sp > 1 ? gpart + sp * M * (dq + dkv) : v32;
    // 2. global position encoding; the recomputed K/V go to their places in the cache
    RopeTable tab;
    for (int i = 0; i < D / 2; ++i) tab.theta[i] = std::pow(static_cast<double>(dims->rope_base), -2.0 * i / D);
    hipLaunchKernelGGL(rope_scatter_kernel, dim3(static_cast<uint32_t>(M), 4), dim3(256), 0, st, q_src, k_src, v_src,
                       chunk_idx_dev, q16, k_plane, v_plane, tab, s.chunk_tokens, s.n_tokens, Hq, Hkv, D, sp);
    // 3. causal attention over the recovered K/V
    AttnGeom g;
    g.M = static_cast<int32_t>(M);
    g.T = s.chunk_tokens;
    g.N = s.n_tokens;
    g.Hq = Hq;
    g.Hkv = Hkv;
    g.n_rb = static_cast<int32_t>((M + 31) / 32);
    g.pairs = (Hq / Hkv) * g.n_rb;
    g.scale_log2e = static_cast<float>(1.4426950408889634 / std::sqrt(static_cast<double>(D)));
    const uint32_t pair_blocks = static_cast<uint32_t>((g.pairs + kAttnWaves - 1) / kAttnWaves);
    if (p.splits > 1) {
        float* part_o = reinterpret_cast<float*>(base + p.part_o);
        float* part_ml = reinterpret_cast<float*>(base + p.part_ml);
        const int n_tiles = (s.n_tokens + 31) / 32;
        const int per_split = (n_tiles + p.splits - 1) / p.splits;
        const dim3 agrid(pair_blocks, static_cast<uint32_t>(Hkv), static_cast<uint32_t>(p.splits));
        const int64_t rows = M * Hq;
        if (D == 64) {
            hipLaunchKernelGGL((recompute_attention_kernel<64, true>), agrid, dim3(64 * kAttnWaves), 0, st, q16,
                               k_plane, v_plane, chunk_idx_dev, attn, g, part_o, part_ml, per_split);
            hipLaunchKernelGGL(attention_combine_kernel<64>, dim3(static_cast<uint32_t>((rows * 16 + 255) / 256)),
                               dim3(256), 0, st, part_o, part_ml, attn, rows, p.splits);
        } else {
            hipLaunchKernelGGL((recompute_attention_kernel<128, true>), agrid, dim3(64 * kAttnWaves), 0, st, q16,
                               k_plane, v_plane, chunk_idx_dev, attn, g, part_o, part_ml, per_split);
            hipLaunchKernelGGL(attention_combine_kernel<128>, dim3(static_cast<uint32_t>((rows * 32 + 255) / 256)),
                               dim3(256), 0, st, part_o, part_ml, attn, rows, p.splits);
        }
    } else {
        const dim3 agrid(pair_blocks, static_cast<uint32_t>(Hkv));
        if (D == 64)
            hipLaunchKernelGGL((recompute_attention_kernel<64, false>), agrid, dim3(64 * kAttnWaves), 0, st, q16,
                               k_plane, v_plane, chunk_idx_dev, attn, g, nullptr, nullptr, 0);
        else
            hipLaunchKernelGGL((recompute_attention_kernel<128, false>), agrid, dim3(64 * kAttnWaves), 0, st, q16,
                               k_plane, v_plane, chunk_idx_dev, attn, g, nullptr, nullptr, 0);
    }
    // 4. output projection + residual, feed-forward + residual
    const GemmGroup og = {1, {dims->d_model}, {w->wo}, {x1}};
    if (int e = gemm(rc, st, gpart, &sp, M, dq, attn, og, xin, false, "o")) return e;
    if (sp > 1)
        hipLaunchKernelGGL(rmsnorm_sum_kernel, dim3(static_cast<uint32_t>(M)), dim3(256), 0, st, gpart, sp, xin, x1,
                           static_cast<const _Float16*>(w->w_norm2), xn, static_cast<int32_t>(M), dims->d_model,
                           dims->rms_eps);
    else
        hipLaunchKernelGGL(rmsnorm_kernel, rows, dim3(256), 0, st, x1, static_cast<const _Float16*>(w->w_norm2), xn,
                           static_cast<int32_t>(M), dims->d_model, dims->rms_eps);
    const GemmGroup ff = {2, {dims->d_ff, dims->d_ff}, {w->w_gate, w->w_up}, {gate, up}};
    if (int e = gemm(rc, st, gpart, &sp, M, dims->d_model, xn, ff, nullptr, false, "gate | up")) return e;
    const int64_t n8 = M * dims->d_ff / 8;
    hipLaunchKernelGGL(silu_mul_kernel, dim3(static_cast<uint32_t>((n8 + 255) / 256)), dim3(256), 0, st, gate, up,
                       gate, n8, sp > 1 ? gpart : no_part, sp > 1 ? gpart + sp * M * dims->d_ff : no_part, sp);
    const GemmGroup down = {1, {dims->d_model}, {w->w_down}, {x_out}};
    if (int e = gemm(rc, st, gpart, nullptr, M, dims->d_ff, gate, down, x1, false, "down")) return e;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(KV_EHIP, "recompute launch: %s", hipGetErrorString(e));
    return KV_OK;
}

}  // extern "C"
