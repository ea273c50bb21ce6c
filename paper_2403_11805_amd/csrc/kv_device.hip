// Device entry points of libkvswitch: argument checks on the host, then kernel
// launches on the caller's stream.  Nothing here synchronises or allocates
// device memory.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <mutex>
#include <new>
#include <vector>

#include "kv_internal.h"
#include "kv_quant_kernels.hpp"
#include "kv_quant_i8_kernels.hpp"
#include "kv_plan_kernels.hpp"
#include "kv_score_kernels.hpp"

using namespace kvs;

namespace {

int hip_fail(hipError_t e, const char* what) {
    return fail(KV_EHIP, "%s: %s", what, hipGetErrorString(e));
}

#define KV_HIP(call)                                         \
    do {                                                     \
        hipError_t e_ = (call);                              \
        if (e_ != hipSuccess) return hip_fail(e_, #call);    \
    } while (0)

int ilog2(int v) {
    int l = 0;
    while ((1 << l) < v) ++l;
    return l;
}

// Measured on MI355X (llama2-7b-4k, widths by score terciles): compress streams best with 4 pieces
// per lane walking the slabs of one chunk (record-major: its write side is one forward stream);
// swap-in with 4 pieces per lane and up to 16 wavefronts per workgroup in strip order
// (strip_task_at: every XCD writes one plane of the cache as a forward stream).
constexpr int kCompressPiecesPerLane = 4;
constexpr int kSwapinPiecesPerLane = 4;
constexpr int kLinkWaves = 4;          // wavefronts per workgroup where the records come over the host link

QuantGeom quant_geom(const kv_shape_t& s) {
    QuantGeom g;
    g.n_tokens = s.n_tokens;
    g.chunk_tokens = s.chunk_tokens;
    g.slabs = static_cast<int32_t>(slabs_of(s));
    g.slab0 = 0;
    g.slab_count = g.slabs;
    g.pieces = s.chunk_tokens * s.head_dim / 8;
    g.row_pieces = s.head_dim / 8;
    g.lpg_log2 = ilog2(s.group / 8);
    g.tpu = 0;
    g.tpu_shift = -1;
    g.record_major = 0;
    g.strip = kStripSlabs;
    g.groups = 0;
    return g;
}

// int8 channel-wise format: one wavefront task per (chunk, slab) unit of 16-byte pieces.
QuantGeom quant_geom_i8(const kv_shape_t& s, int* ppl) {
    QuantGeom g;
    g.n_tokens = s.n_tokens;
    g.chunk_tokens = s.chunk_tokens;
    g.slabs = static_cast<int32_t>(slabs_of(s));
    g.slab0 = 0;
    g.slab_count = g.slabs;
    g.pieces = s.chunk_tokens * s.head_dim / 16;
    g.row_pieces = s.head_dim / 16;
    g.lpg_log2 = ilog2(g.row_pieces);
    g.tpu = 1;
    g.tpu_shift = 0;
    g.record_major = 0;
    g.strip = kStripSlabs;
    g.groups = 0;
    *ppl = g.pieces / 64;      // 1, 2 or 4 (shape check)
    return g;
}

I8View i8_view(const kv_shape_t& s) {
    I8View v;
    v.head_dim = s.head_dim;
    v.group_lanes = s.head_dim / 4 < 64 ? s.head_dim / 4 : 64;
    v.share_log2 = 6 - ilog2(v.group_lanes);
    v.half_meta = s.format == KV_FMT_I8_CHANNELS_H ? 1 : 0;
    return v;
}

// Calls LAUNCH(NDW, GPL) for the int8 format's (dwords per lane, channel groups per lane).
#define KV_I8_DISPATCH(ppl, head_dim, LAUNCH)                                   \
    do {                                                                        \
        const int gpl_ = (head_dim) > 256 ? (head_dim) / 256 : 1;               \
        switch ((ppl) * 4 * 8 + gpl_) {                                         \
            case 4 * 8 + 1: LAUNCH(4, 1); break;                                \
            case 4 * 8 + 2: LAUNCH(4, 2); break;                                \
            case 4 * 8 + 4: LAUNCH(4, 4); break;                                \
            case 8 * 8 + 1: LAUNCH(8, 1); break;                                \
            case 8 * 8 + 2: LAUNCH(8, 2); break;                                \
            case 8 * 8 + 4: LAUNCH(8, 4); break;                                \
            case 16 * 8 + 1: LAUNCH(16, 1); break;                              \
            case 16 * 8 + 2: LAUNCH(16, 2); break;                              \
            case 16 * 8 + 4: LAUNCH(16, 4); break;                              \
            default: return fail(KV_ESHAPE, "int8 format: unsupported unit");   \
        }                                                                       \
    } while (0)

// Pieces per lane of a wavefront task (the largest of 4, 2, 1 that is at most
// max_ppl and divides the unit) and the resulting tasks per unit.
int plan_tasks(QuantGeom* g, int max_ppl) {
    const int wpu = g->pieces / 64;
    const int ppl = (wpu % 4 == 0 && max_ppl >= 4) ? 4 : ((wpu % 2 == 0 && max_ppl >= 2) ? 2 : 1);
    g->tpu = wpu / ppl;
    g->tpu_shift = ((g->tpu & (g->tpu - 1)) == 0) ? ilog2(g->tpu) : -1;
    return ppl;
}

dim3 task_grid(const QuantGeom& g, int n_units) {
    const int along_x = g.record_major ? g.slab_count : n_units;
    const int along_y = g.record_major ? n_units : g.slab_count;
    const int64_t tasks = static_cast<int64_t>(along_x) * g.tpu;
    return dim3(static_cast<uint32_t>((tasks + kWavesPerBlock - 1) / kWavesPerBlock),
                static_cast<uint32_t>(along_y));
}

// Launch shape of a Load kernel of the fp16 formats over n_units listed records (g.tpu and g.slab_count
// set): wavefronts per workgroup (at most wpb_max, no more than a slab has tasks), workgroups per slab
// into g.groups, and the one-dimensional grid.  0 if the grid does not fit.
// A Load runs fastest with 24 wavefronts on a CU, not the 32 that fit: its stores are 2.7 times its reads,
// and a store stream is served best with few bytes in flight per CU (stores alone: 7.5 TB/s with 32 KB in
// flight per CU, 5.9 TB/s with 128 KB), while the record reads want many.  Measured over the 2 GiB cache:
// 20 wavefronts per CU 0.521 ms, 24: 0.473, 28: 0.482, 32: 0.487-0.494 (workgroups of 16, 8 or 4 wavefronts
// alike); the pool's switch (0.58 GB) 0.1069 against 0.1091 ms, gemma2b-4k (0.1 GB) 0.0210 against 0.0212.
// The cap is set by asking for LDS that the kernel does not use (*idle_lds bytes per workgroup of 4
// wavefronts: six such workgroups fit the 160 KB of a CU).  Launches under 32 MiB (a Fault) keep
// workgroups of up to 8 wavefronts and no cap; where a unit has fewer than 256 pieces, so that a wavefront
// moves 1 or 2 KiB instead of 4, workgroups of 4 without a cap do best (chunks of 4 and 8 tokens at
// head_dim 128: 0.69 and 0.51 ms against 0.80 and 0.55 ms with 16).
constexpr uint32_t kIdleLdsBytes = 26 * 1024;
uint32_t load_grid(QuantGeom* g, int n_units, int wpb_max, int* wpb, uint32_t* idle_lds) {
    const int64_t tasks = static_cast<int64_t>(n_units) * g->tpu;          // per slab
    const int64_t out_bytes = static_cast<int64_t>(n_units) * g->pieces * 16 * g->slab_count;
    *idle_lds = 0;
    if (out_bytes < (32LL << 20)) wpb_max = std::min(wpb_max, 8);
    else if (wpb_max == kLoadWavesMax && g->pieces >= 256) {
        wpb_max = 4;
        *idle_lds = kIdleLdsBytes;
    }
    if (g->pieces < 256) wpb_max = std::min(wpb_max, 4);
    *wpb = static_cast<int>(std::min<int64_t>(wpb_max, tasks));
    g->groups = static_cast<int32_t>((tasks + *wpb - 1) / *wpb);
    const int64_t total = static_cast<int64_t>(g->groups) * g->slab_count;
    return total > 0x7fffffffLL ? 0u : static_cast<uint32_t>(total);
}

int launch_status(const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, what);
    return KV_OK;
}

// One launch of the Load kernel whose (short) gather list travels in the kernel
// arguments; offsets in the list are relative to `base`.
int launch_swapin_batch(const kv_shape_t& shape, const QuantGeom& g_in, int ppl, const uint8_t* base,
                        const SwapinBatch& list, u4_t* dst, hipStream_t st) {
    QuantGeom g = g_in;
    if (is_i8(shape)) {
        int wpb = 0;
        uint32_t idle_lds = 0;
        const uint32_t wgs = load_grid(&g, list.n, kWavesPerBlock, &wpb, &idle_lds);
        if (!wgs) return fail(KV_ESHAPE, "Load grid exceeds 2^31 workgroups");
        const dim3 grid(wgs), block(static_cast<uint32_t>(wpb) * 64);
        const I8View v = i8_view(shape);
#define KV_LAUNCH_I8(NDW, GPL) \
        do {                                                                                                    \
            if (v.half_meta) hipLaunchKernelGGL((swapin_i8_batch_kernel<NDW, GPL, true>), grid, block, 0, st, base, list, dst, g, v); \
            else hipLaunchKernelGGL((swapin_i8_batch_kernel<NDW, GPL, false>), grid, block, 0, st, base, list, dst, g, v);            \
        } while (0)
        KV_I8_DISPATCH(ppl, shape.head_dim, KV_LAUNCH_I8);
#undef KV_LAUNCH_I8
    } else {
        const bool hp = shape.format == KV_FMT_F16_GROUPS_H;
        int wpb = 0;
        uint32_t idle_lds = 0;
        const uint32_t wgs = load_grid(&g, list.n, kLoadWavesMax, &wpb, &idle_lds);
        if (!wgs) return fail(KV_ESHAPE, "Load grid exceeds 2^31 workgroups");
        const dim3 grid(wgs), block(static_cast<uint32_t>(wpb) * 64);
#define KV_LAUNCH_F16(PPL)                                                                                        \
        do {                                                                                                      \
            if (hp) hipLaunchKernelGGL((swapin_batch_kernel<PPL, true>), grid, block, idle_lds, st, base, list, dst, g); \
            else hipLaunchKernelGGL((swapin_batch_kernel<PPL, false>), grid, block, idle_lds, st, base, list, dst, g);   \
        } while (0)
        if (ppl == 4) KV_LAUNCH_F16(4);
        else if (ppl == 2) KV_LAUNCH_F16(2);
        else KV_LAUNCH_F16(1);
#undef KV_LAUNCH_F16
    }
    return launch_status("swapin_batch_kernel launch");
}

}  // namespace

extern "C" {

// Compression of all chunks (chunk_list NULL, n_units = n_chunks) or of the listed ones.
static int32_t compress_launch(const kv_shape_t* shape, const void* kv, const uint8_t* bits_dev,
                               const uint64_t* off_dev, const int32_t* chunk_list, int32_t n_units,
                               void* packed_out, void* stream) {
    const bool i8 = is_i8(*shape);
    int ppl = 0;
    QuantGeom g = i8 ? quant_geom_i8(*shape, &ppl) : quant_geom(*shape);
    if (!i8) ppl = plan_tasks(&g, kCompressPiecesPerLane);
    g.record_major = n_units <= 65535 ? 1 : 0;
    if (!g.record_major && g.slabs > 65535)
        return fail(KV_ESHAPE, "more than 65535 chunks and slabs exceed the launch grid");
    const dim3 grid = task_grid(g, n_units);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const u4_t* src = static_cast<const u4_t*>(kv);
    uint8_t* dst = static_cast<uint8_t*>(packed_out);
    if (i8) {
        const I8View v = i8_view(*shape);
#define KV_LAUNCH_I8(NDW, GPL)                                                                               \
        do {                                                                                                 \
            if (v.half_meta)                                                                                 \
                hipLaunchKernelGGL((compress_i8_kernel<NDW, GPL, true>), grid, dim3(256), 0, st, src, bits_dev, \
                                   off_dev, dst, g, v, n_units, chunk_list);                                 \
            else                                                                                             \
                hipLaunchKernelGGL((compress_i8_kernel<NDW, GPL, false>), grid, dim3(256), 0, st, src, bits_dev, \
                                   off_dev, dst, g, v, n_units, chunk_list);                                 \
        } while (0)
        KV_I8_DISPATCH(ppl, shape->head_dim, KV_LAUNCH_I8);
#undef KV_LAUNCH_I8
        return launch_status("compress_i8_kernel launch");
    }
    const bool hp = shape->format == KV_FMT_F16_GROUPS_H;
#define KV_LAUNCH_F16(PPL)                                                                                     \
    do {                                                                                                       \
        if (hp) hipLaunchKernelGGL((compress_kernel<PPL, true>), grid, dim3(256), 0, st, src, bits_dev, off_dev, dst, g, n_units, chunk_list); \
        else hipLaunchKernelGGL((compress_kernel<PPL, false>), grid, dim3(256), 0, st, src, bits_dev, off_dev, dst, g, n_units, chunk_list);   \
    } while (0)
    if (ppl == 4) KV_LAUNCH_F16(4);
    else if (ppl == 2) KV_LAUNCH_F16(2);
    else KV_LAUNCH_F16(1);
#undef KV_LAUNCH_F16
    return launch_status("compress_kernel launch");
}

int32_t kv_compress_chunks(const kv_shape_t* shape, const void* kv, const uint8_t* bits_dev,
                           const uint64_t* off_dev, void* packed_out, void* stream) {
    if (int rc = check_shape(shape)) return rc;
    if (!kv || !bits_dev || !off_dev || !packed_out) return fail(KV_EINVAL, "NULL device pointer");
    if (!aligned(kv, 16) || !aligned(packed_out, 16) || !aligned(off_dev, 8))
        return fail(KV_EINVAL, "kv/packed_out must be 16-byte aligned, off_dev 8-byte aligned");
    return compress_launch(shape, kv, bits_dev, off_dev, nullptr, shape->n_tokens / shape->chunk_tokens,
                           packed_out, stream);
}

int32_t kv_compress_selected(const kv_shape_t* shape, const void* kv, const uint8_t* bits_dev,
                             const uint64_t* off_dev, const int32_t* chunk_idx_dev, int32_t n_sel,
                             void* packed_out, void* stream) {
    if (int rc = check_shape(shape)) return rc;
    const int32_t n_chunks = shape->n_tokens / shape->chunk_tokens;
    if (n_sel < 0 || n_sel > n_chunks) return fail(KV_EINVAL, "n_sel %d outside [0,%d]", n_sel, n_chunks);
    if (n_sel == 0) return KV_OK;
    if (!kv || !bits_dev || !off_dev || !chunk_idx_dev || !packed_out) return fail(KV_EINVAL, "NULL device pointer");
    if (!aligned(kv, 16) || !aligned(packed_out, 16) || !aligned(off_dev, 8) || !aligned(chunk_idx_dev, 4))
        return fail(KV_EINVAL, "kv/packed_out must be 16-byte aligned, off_dev 8-byte, chunk_idx_dev 4-byte aligned");
    return compress_launch(shape, kv, bits_dev, off_dev, chunk_idx_dev, n_sel, packed_out, stream);
}

// Where a record pool lives: device memory (1), pinned host memory that the device addresses (2:
// the Load kernels then read the records over the host link and are launched as a small strided
// grid), or memory the runtime does not know, e.g. pageable host memory (0: a kernel must not
// touch it).
static int pool_kind(const void* p) {
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, p) != hipSuccess) {
        (void)hipGetLastError();
        return 0;
    }
    if (attr.type == hipMemoryTypeHost) return 2;
    if (attr.type == hipMemoryTypeUnregistered) return 0;
    return 1;
}

// Load of the listed chunks into the cache, all layers or the layers [layer_begin, layer_end).
static int32_t swapin_launch(const kv_shape_t* shape, const void* packed, const uint64_t* src_off_dev,
                             const int32_t* dst_tok_dev, const uint8_t* sel_bits_dev, int32_t n_sel,
                             int32_t layer_begin, int32_t layer_end, void* kv_out, void* stream) {
    const int32_t n_chunks = shape->n_tokens / shape->chunk_tokens;
    if (n_sel < 0 || n_sel > n_chunks) return fail(KV_EINVAL, "n_sel %d outside [0,%d]", n_sel, n_chunks);
    if (n_sel == 0 || layer_begin == layer_end) return KV_OK;
    if (!packed || !src_off_dev || !dst_tok_dev || !sel_bits_dev || !kv_out)
        return fail(KV_EINVAL, "NULL device pointer");
    if (!aligned(kv_out, 16) || !aligned(packed, 16) || !aligned(src_off_dev, 8) ||
        !aligned(dst_tok_dev, 4))
        return fail(KV_EINVAL, "kv_out/packed must be 16-byte aligned, lists naturally aligned");
    const bool i8 = is_i8(*shape);
    int ppl = 0;
    QuantGeom g = i8 ? quant_geom_i8(*shape, &ppl) : quant_geom(*shape);
    if (!i8) ppl = plan_tasks(&g, kSwapinPiecesPerLane);
    g.slab0 = layer_begin * 2 * shape->n_kv_heads;
    g.slab_count = (layer_end - layer_begin) * 2 * shape->n_kv_heads;
    const int kind = pool_kind(packed);
    if (kind == 0) return fail(KV_EINVAL, "packed is neither device memory nor pinned host memory");
    // strip order; the int8 kernels keep a slab in LDS per wavefront and stay at four wavefronts per workgroup
    int wpb = 0;
    uint32_t idle_lds = 0;
    const dim3 grid(load_grid(&g, n_sel, i8 ? kWavesPerBlock : (kind == 2 ? kLinkWaves : kLoadWavesMax), &wpb, &idle_lds));
    if (!grid.x) return fail(KV_ESHAPE, "Load grid exceeds 2^31 workgroups");
    const dim3 block(static_cast<uint32_t>(wpb) * 64);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint8_t* src = static_cast<const uint8_t*>(packed);
    u4_t* dst = static_cast<u4_t*>(kv_out);
    if (kind == 2) {
        const dim3 lgrid(std::min<uint32_t>(grid.x, kLinkBlocks));
        if (i8) {
            const I8View v = i8_view(*shape);
#define KV_LAUNCH_I8(NDW, GPL)                                                                            \
            do {                                                                                          \
                if (v.half_meta)                                                                          \
                    hipLaunchKernelGGL((swapin_i8_link_kernel<NDW, GPL, true>), lgrid, block, 0, st, src,        \
                                       src_off_dev, dst_tok_dev, sel_bits_dev, dst, g, v, n_sel, grid.x);         \
                else                                                                                      \
                    hipLaunchKernelGGL((swapin_i8_link_kernel<NDW, GPL, false>), lgrid, block, 0, st, src,       \
                                       src_off_dev, dst_tok_dev, sel_bits_dev, dst, g, v, n_sel, grid.x);         \
            } while (0)
            KV_I8_DISPATCH(ppl, shape->head_dim, KV_LAUNCH_I8);
#undef KV_LAUNCH_I8
            return launch_status("swapin_i8_link_kernel launch");
        }
        const bool hp = shape->format == KV_FMT_F16_GROUPS_H;
#define KV_LAUNCH_F16(PPL)                                                                                     \
        do {                                                                                                   \
            if (hp) hipLaunchKernelGGL((swapin_link_kernel<PPL, true>), lgrid, block, 0, st, src, src_off_dev, dst_tok_dev, sel_bits_dev, dst, g, n_sel, grid.x); \
            else hipLaunchKernelGGL((swapin_link_kernel<PPL, false>), lgrid, block, 0, st, src, src_off_dev, dst_tok_dev, sel_bits_dev, dst, g, n_sel, grid.x);   \
        } while (0)
        if (ppl == 4) KV_LAUNCH_F16(4);
        else if (ppl == 2) KV_LAUNCH_F16(2);
        else KV_LAUNCH_F16(1);
#undef KV_LAUNCH_F16
        return launch_status("swapin_link_kernel launch");
    }
    if (i8) {
        const I8View v = i8_view(*shape);
#define KV_LAUNCH_I8(NDW, GPL)                                                                            \
        do {                                                                                              \
            if (v.half_meta)                                                                              \
                hipLaunchKernelGGL((swapin_i8_kernel<NDW, GPL, true>), grid, block, 0, st, src, src_off_dev,     \
                                   dst_tok_dev, sel_bits_dev, dst, g, v, n_sel);                          \
            else                                                                                          \
                hipLaunchKernelGGL((swapin_i8_kernel<NDW, GPL, false>), grid, block, 0, st, src, src_off_dev,    \
                                   dst_tok_dev, sel_bits_dev, dst, g, v, n_sel);                          \
        } while (0)
        KV_I8_DISPATCH(ppl, shape->head_dim, KV_LAUNCH_I8);
#undef KV_LAUNCH_I8
        return launch_status("swapin_i8_kernel launch");
    }
    const bool hp = shape->format == KV_FMT_F16_GROUPS_H;
#define KV_LAUNCH_F16(PPL)                                                                                     \
    do {                                                                                                       \
        if (hp) hipLaunchKernelGGL((swapin_kernel<PPL, true>), grid, block, idle_lds, st, src, src_off_dev, dst_tok_dev, sel_bits_dev, dst, g, n_sel); \
        else hipLaunchKernelGGL((swapin_kernel<PPL, false>), grid, block, idle_lds, st, src, src_off_dev, dst_tok_dev, sel_bits_dev, dst, g, n_sel);   \
    } while (0)
    if (ppl == 4) KV_LAUNCH_F16(4);
    else if (ppl == 2) KV_LAUNCH_F16(2);
    else KV_LAUNCH_F16(1);
#undef KV_LAUNCH_F16
    return launch_status("swapin_kernel launch");
}

int32_t kv_swapin_chunks(const kv_shape_t* shape, const void* packed, const uint64_t* src_off_dev,
                         const int32_t* dst_tok_dev, const uint8_t* sel_bits_dev, int32_t n_sel,
                         void* kv_out, void* stream) {
    if (int rc = check_shape(shape)) return rc;
    return swapin_launch(shape, packed, src_off_dev, dst_tok_dev, sel_bits_dev, n_sel, 0, shape->n_layers, kv_out,
                         stream);
}

int32_t kv_swapin_layers(const kv_shape_t* shape, const void* packed, const uint64_t* src_off_dev,
                         const int32_t* dst_tok_dev, const uint8_t* sel_bits_dev, int32_t n_sel,
                         int32_t layer_begin, int32_t layer_end, void* kv_out, void* stream) {
    if (int rc = check_shape(shape)) return rc;
    if (layer_begin < 0 || layer_end < layer_begin || layer_end > shape->n_layers)
        return fail(KV_EINVAL, "layers [%d,%d) outside [0,%d]", layer_begin, layer_end, shape->n_layers);
    return swapin_launch(shape, packed, src_off_dev, dst_tok_dev, sel_bits_dev, n_sel, layer_begin, layer_end, kv_out,
                         stream);
}

// --------------------------------------------------------------------- scoring

static int score_geom(const kv_shape_t* shape, int32_t n_queries, int32_t n_valid, int32_t norm_mode,
                      ScoreGeom* out, int* nrbw) {
    if (int rc = check_shape(shape)) return rc;
    const kv_shape_t& s = *shape;
    if (!is_f16(s)) return fail(KV_ESHAPE, "scoring needs an fp16 cache format");
    if (n_queries < 1 || n_queries > s.n_tokens || n_queries > 256)
        return fail(KV_EINVAL, "n_queries %d outside [1, min(n_tokens, 256)]", n_queries);
    if (n_valid < n_queries || n_valid > s.n_tokens)
        return fail(KV_EINVAL, "n_valid %d outside [n_queries, n_tokens]", n_valid);
    if (norm_mode != KV_NORM_VISIBLE && norm_mode != KV_NORM_NONE)
        return fail(KV_EINVAL, "norm_mode %d unknown", norm_mode);
    if (s.head_dim != 64 && s.head_dim != 128 && s.head_dim != 256)
        return fail(KV_ESHAPE, "scoring needs head_dim in {64,128,256}, got %d", s.head_dim);
    if (s.chunk_tokens < 8 || (s.chunk_tokens & (s.chunk_tokens - 1)))
        return fail(KV_ESHAPE, "scoring needs chunk_tokens a power of two >= 8, got %d", s.chunk_tokens);
    if (s.n_tokens % 32) return fail(KV_ESHAPE, "scoring needs n_tokens %% 32 == 0, got %d", s.n_tokens);
    ScoreGeom g;
    g.L = s.n_layers; g.Hkv = s.n_kv_heads; g.Hq = s.n_q_heads; g.N = s.n_tokens; g.R = n_queries;
    g.Nv = n_valid;
    g.T = s.chunk_tokens;
    g.sb_tokens = std::min(s.chunk_tokens, 32);
    g.n_tiles = s.n_tokens / 32;
    g.RB = (n_queries + 31) / 32;
    g.rows_p = g.RB * 32;
    g.n_rb = (s.n_q_heads / s.n_kv_heads) * g.RB;
    *nrbw = g.n_rb == 1 ? 1 : 2;
    g.n_rg = (g.n_rb + *nrbw - 1) / *nrbw;
    g.rg_per_wg = std::min(g.n_rg, 4);
    // several row groups per kv head: the workgroup shares each K tile through LDS and all
    // its wavefronts walk the same run; a single row group: four independent runs per workgroup
    g.tile_par = g.rg_per_wg > 1 ? 1 : 4;
    g.run_len = std::min(g.n_tiles, g.tile_par == 1 ? 64 : 8);
    g.n_runs = (g.n_tiles + g.run_len - 1) / g.run_len;
    if (g.n_runs > kCombineMaxRuns)        // 2M tokens with one block of query rows per kv head, 16M otherwise
        return fail(KV_ESHAPE, "scoring handles at most %d runs of tiles per head, this shape has %d", kCombineMaxRuns,
                    g.n_runs);
    g.norm_mode = norm_mode;
    g.scale_log2e = static_cast<float>(1.4426950408889634 / std::sqrt(static_cast<double>(s.head_dim)));
    g.inv_R = 1.0f / static_cast<float>(n_queries);
    *out = g;
    return KV_OK;
}

static uint64_t ws_floats_tile(const ScoreGeom& g) {
    return static_cast<uint64_t>(g.L) * g.Hq * g.n_tiles * g.rows_p;
}
static uint64_t ws_floats_sub(const ScoreGeom& g) {
    return static_cast<uint64_t>(g.L) * g.Hq * (g.N / g.sb_tokens) * g.rows_p;
}
static uint64_t ws_floats_run(const ScoreGeom& g) {
    return static_cast<uint64_t>(g.L) * g.Hq * g.n_runs * g.rows_p;
}

uint64_t kv_score_workspace_bytes(const kv_shape_t* shape, int32_t n_queries) {
    ScoreGeom g;
    int nrbw;
    if (!shape || score_geom(shape, n_queries, shape->n_tokens, KV_NORM_VISIBLE, &g, &nrbw) != KV_OK) return 0;
    const uint64_t bytes = (ws_floats_tile(g) + ws_floats_sub(g) + 3 * ws_floats_run(g)) * sizeof(float);
    return (bytes + 255) & ~static_cast<uint64_t>(255);
}

int32_t kv_score_chunks(const kv_shape_t* shape, const void* q, int32_t n_queries, const void* kv,
                        int32_t norm_mode, void* workspace, uint64_t workspace_bytes,
                        float* chunk_mass, float* density, void* stream) {
    if (!shape) return fail(KV_EINVAL, "NULL shape");
    return kv_score_chunks_valid(shape, q, n_queries, kv, shape->n_tokens, norm_mode, workspace, workspace_bytes,
                                 chunk_mass, density, stream);
}

// LDS of score_head_kernel for this geometry (one workgroup scores a whole head and keeps the
// partials there), or 0 where that kernel does not apply: it needs one block of query rows per
// head, at least one (layer, head) per CU and at most 40 KiB, so that four workgroups share a CU.
static uint64_t score_head_lds_bytes(const ScoreGeom& g, int head_dim) {
    const uint64_t head_lds = (static_cast<uint64_t>(g.N / g.sb_tokens) * 32 + 2ull * g.n_runs * 32 + 4 * 5 * 32 + 64) *
                              sizeof(float);
    return (g.n_rb == 1 && g.L * g.Hkv >= 256 && head_lds <= 40960 && head_dim <= 128) ? head_lds : 0;
}

static int32_t score_launch(const kv_shape_t* shape, const ScoreGeom& g, int nrbw, const void* q, const void* kv,
                            void* workspace, float* chunk_mass, float* density, void* stream);

int32_t kv_score_chunks_valid(const kv_shape_t* shape, const void* q, int32_t n_queries, const void* kv,
                              int32_t n_valid, int32_t norm_mode, void* workspace, uint64_t workspace_bytes,
                              float* chunk_mass, float* density, void* stream) {
    ScoreGeom g;
    int nrbw;
    if (!shape) return fail(KV_EINVAL, "NULL shape");
    if (int rc = score_geom(shape, n_queries, n_valid, norm_mode, &g, &nrbw)) return rc;
    if (!q || !kv || !workspace || !chunk_mass || !density) return fail(KV_EINVAL, "NULL device pointer");
    if (!aligned(q, 16) || !aligned(kv, 16) || !aligned(workspace, 256))
        return fail(KV_EINVAL, "q/kv must be 16-byte aligned, workspace 256-byte aligned");
    const uint64_t need = kv_score_workspace_bytes(shape, n_queries);
    if (workspace_bytes < need)
        return fail(KV_ENOMEM, "workspace %llu bytes, %llu needed",
                    static_cast<unsigned long long>(workspace_bytes), static_cast<unsigned long long>(need));
    return score_launch(shape, g, nrbw, q, kv, workspace, chunk_mass, density, stream);
}

// ---- scoring for callers that cannot allocate: the partials live in a static device array ----

// Scratch of kv_score_chunks_static: one copy per GPU the library runs on, held until the process
// ends.  In host code the name is only a handle; the device address comes from
// hipGetSymbolAddress, once per device.
constexpr uint64_t kStaticScratchBytes = KV_SCORE_STATIC_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex scratch_mutex;
static void* scratch_ptr[kMaxDevices];       // device address of `scratch` on each device, once known

static int static_scratch(void** out) {
    int dev = -1;
    KV_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(KV_EINVAL, "device %d outside [0,%d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> hold(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void* p = nullptr;
        KV_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(KV_EHIP, "hipGetSymbolAddress returned a NULL address");
        scratch_ptr[dev] = p;
    }
    *out = scratch_ptr[dev];
    return KV_OK;
}

int32_t kv_score_chunks_static(const kv_shape_t* shape, const void* q, int32_t n_queries, const void* kv,
                               int32_t norm_mode, float* chunk_mass, float* density, void* stream) {
    ScoreGeom g;
    int nrbw;
    if (!shape) return fail(KV_EINVAL, "NULL shape");
    if (int rc = score_geom(shape, n_queries, shape->n_tokens, norm_mode, &g, &nrbw)) return rc;
    if (!q || !kv || !chunk_mass || !density) return fail(KV_EINVAL, "NULL device pointer");
    if (!aligned(q, 16) || !aligned(kv, 16)) return fail(KV_EINVAL, "q/kv must be 16-byte aligned");
    // a head scored by one workgroup keeps its partials in LDS and needs no scratch at all
    const uint64_t need = score_head_lds_bytes(g, shape->head_dim) ? 0 : kv_score_workspace_bytes(shape, n_queries);
    if (need > kStaticScratchBytes)
        return fail(KV_ENOMEM, "scoring this shape needs %llu bytes of scratch, the static buffer holds %llu: "
                    "use kv_score_chunks with a workspace",
                    static_cast<unsigned long long>(need), static_cast<unsigned long long>(kStaticScratchBytes));
    void* ws = nullptr;
    if (int rc = static_scratch(&ws)) return rc;
    // every slot of the partial planes is written before it is read: nothing has to start at zero
    return score_launch(shape, g, nrbw, q, kv, ws, chunk_mass, density, stream);
}

static int32_t score_launch(const kv_shape_t* shape, const ScoreGeom& g, int nrbw, const void* q, const void* kv,
                            void* workspace, float* chunk_mass, float* density, void* stream) {
    ScoreWs ws;
    ws.m_tile = static_cast<float*>(workspace);
    ws.e_sub = ws.m_tile + ws_floats_tile(g);
    ws.m_run = ws.e_sub + ws_floats_sub(g);
    ws.l_run = ws.m_run + ws_floats_run(g);
    ws.m_fast = ws.l_run + ws_floats_run(g);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid((g.n_runs + g.tile_par - 1) / g.tile_par,
                    (g.n_rg + g.rg_per_wg - 1) / g.rg_per_wg, g.L * g.Hkv);
    const _Float16* qp = static_cast<const _Float16*>(q);
    const _Float16* kp = static_cast<const _Float16*>(kv);
#define KV_SCORE_SHARED(DD)                                                                           \
    do {                                                                                             \
        if (g.sb_tokens == 32)                                                                       \
            hipLaunchKernelGGL((score_tiles_shared_kernel<DD, 1>), grid, dim3(256), 0, st, qp, kp, g, ws); \
        else if (g.sb_tokens == 16)                                                                  \
            hipLaunchKernelGGL((score_tiles_shared_kernel<DD, 2>), grid, dim3(256), 0, st, qp, kp, g, ws); \
        else                                                                                         \
            hipLaunchKernelGGL((score_tiles_shared_kernel<DD, 4>), grid, dim3(256), 0, st, qp, kp, g, ws); \
    } while (0)
#define KV_SCORE_DIRECT(DD, NR) \
    hipLaunchKernelGGL((score_tiles_kernel<DD, NR>), grid, dim3(256), 0, st, qp, kp, g, ws)
    const int D = shape->head_dim;
    // One block of query rows per head and at least one (layer, head) per CU: a workgroup scores a
    // whole head, keeps the partials in LDS and writes the chunk masses itself (at most 40 KiB of
    // LDS, so that four workgroups share a CU).
    const uint64_t head_lds = score_head_lds_bytes(g, D);
    if (head_lds) {
        const dim3 hgrid(static_cast<uint32_t>(g.L * g.Hkv));
        if (D == 64)
            hipLaunchKernelGGL(score_head_kernel<64>, hgrid, dim3(256), head_lds, st, qp, kp, g, chunk_mass);
        else
            hipLaunchKernelGGL(score_head_kernel<128>, hgrid, dim3(256), head_lds, st, qp, kp, g, chunk_mass);
        if (int rc = launch_status("score_head_kernel launch")) return rc;
        const int n_chunks_h = g.N / g.T;
        const float inv_norm_h = static_cast<float>(1.0 / (static_cast<double>(g.T) * g.L * g.Hq));
        hipLaunchKernelGGL(score_density_kernel, dim3((n_chunks_h + kDensityChunks - 1) / kDensityChunks), dim3(1024), 0, st, chunk_mass, density,
                           g.L * g.Hq, n_chunks_h, inv_norm_h, g.T, g.Nv);
        return launch_status("score_density_kernel launch");
    }
    if (g.rg_per_wg > 1) {          // several row groups per kv head: two row blocks per wavefront
        if (D == 64) KV_SCORE_SHARED(64);
        else if (D == 128) KV_SCORE_SHARED(128);
        else KV_SCORE_SHARED(256);
    } else if (D == 64 && nrbw == 1) KV_SCORE_DIRECT(64, 1);
    else if (D == 64) KV_SCORE_DIRECT(64, 2);
    else if (D == 128 && nrbw == 1) KV_SCORE_DIRECT(128, 1);
    else if (D == 128) KV_SCORE_DIRECT(128, 2);
    else if (nrbw == 1) KV_SCORE_DIRECT(256, 1);
    else KV_SCORE_DIRECT(256, 2);
#undef KV_SCORE_SHARED
#undef KV_SCORE_DIRECT
    if (int rc = launch_status("score_tiles_kernel launch")) return rc;
    // 32 chunks per pass of a workgroup; a head's chunks are divided among several workgroups where the
    // heads alone would leave the chip short of eight workgroups per CU (each then still has two passes)
    const int n_chunks_c = g.N / g.T;
    const int n_heads_c = g.L * g.Hq;
    const uint32_t combine_parts = static_cast<uint32_t>(
        std::max(1, std::min((2048 + n_heads_c - 1) / n_heads_c, n_chunks_c / 64)));
    hipLaunchKernelGGL(score_combine_kernel, dim3(g.L * g.Hq, combine_parts), dim3(256), 0, st, g, ws, chunk_mass);
    if (int rc = launch_status("score_combine_kernel launch")) return rc;
    const int n_chunks = g.N / g.T;
    const float inv_norm = static_cast<float>(1.0 / (static_cast<double>(g.T) * g.L * g.Hq));
    hipLaunchKernelGGL(score_density_kernel, dim3((n_chunks + kDensityChunks - 1) / kDensityChunks), dim3(1024), 0, st,
                       chunk_mass, density, g.L * g.Hq, n_chunks, inv_norm, g.T, g.Nv);
    return launch_status("score_density_kernel launch");
}

int32_t kv_load_chunks(const kv_shape_t* shape, const void* packed, const uint64_t* off,
                       const uint8_t* bits, const int32_t* chunk_idx, int32_t n_sel, void* kv_out,
                       void* stream) {
    if (int rc = check_shape(shape)) return rc;
    const int32_t n_chunks = shape->n_tokens / shape->chunk_tokens;
    if (n_sel < 0 || n_sel > n_chunks) return fail(KV_EINVAL, "n_sel %d outside [0,%d]", n_sel, n_chunks);
    if (n_sel == 0) return KV_OK;
    if (!packed || !off || !bits || !chunk_idx || !kv_out) return fail(KV_EINVAL, "NULL pointer");
    if (!aligned(packed, 16) || !aligned(kv_out, 16))
        return fail(KV_EINVAL, "packed/kv_out must be 16-byte aligned");
    // the whole list is checked before the first launch
    std::vector<uint64_t> src_off(static_cast<size_t>(n_sel));
    std::vector<int32_t> dst_tok(static_cast<size_t>(n_sel));
    std::vector<uint8_t> sel_bits(static_cast<size_t>(n_sel));
    if (int rc = kv_build_gather(shape, off, bits, chunk_idx, n_sel, src_off.data(), dst_tok.data(),
                                 sel_bits.data()))
        return rc;
    for (int32_t j = 0; j < n_sel; ++j)
        if (src_off[static_cast<size_t>(j)] % 16) return fail(KV_EINVAL, "record offset of chunk %d not 16-byte aligned", chunk_idx[j]);
    // (no query of where `packed` lives here: this is the Fault path, tens of microseconds from call
    // to completion, and the query costs three of them)
    const bool i8 = is_i8(*shape);
    int ppl = 0;
    QuantGeom g = i8 ? quant_geom_i8(*shape, &ppl) : quant_geom(*shape);
    if (!i8) ppl = plan_tasks(&g, kSwapinPiecesPerLane);
    hipStream_t st = static_cast<hipStream_t>(stream);
    for (int32_t j = 0; j < n_sel; j += kBatchMax) {
        SwapinBatch list;
        list.n = std::min<int32_t>(kBatchMax, n_sel - j);
        for (int32_t k = 0; k < list.n; ++k) {
            list.src_off[k] = src_off[static_cast<size_t>(j + k)];
            list.dst_tok[k] = dst_tok[static_cast<size_t>(j + k)];
            list.bits[k] = sel_bits[static_cast<size_t>(j + k)];
        }
        if (int rc = launch_swapin_batch(*shape, g, ppl, static_cast<const uint8_t*>(packed), list,
                                         static_cast<u4_t*>(kv_out), st))
            return rc;
    }
    return KV_OK;
}

// --------------------------------------------------------------------- widths and offsets on the device

int32_t kv_plan_chunks_dev(const kv_shape_t* shape, const float* density_dev, int32_t num8,
                           int32_t num4, int32_t den, uint8_t* bits_dev, uint64_t* off_dev,
                           int32_t* dst_tok_dev, void* stream) {
    if (int rc = check_shape(shape)) return rc;
    if (!density_dev || !bits_dev || !off_dev || !dst_tok_dev) return fail(KV_EINVAL, "NULL device pointer");
    if (!aligned(density_dev, 4) || !aligned(off_dev, 8) || !aligned(dst_tok_dev, 4))
        return fail(KV_EINVAL, "density_dev/dst_tok_dev must be 4-byte aligned, off_dev 8-byte aligned");
    if (den <= 0 || num8 < 0 || num4 < 0 || num8 + num4 > den)
        return fail(KV_EINVAL, "need den > 0, 0 <= num8, 0 <= num4, num8+num4 <= den");
    const int32_t n = shape->n_tokens / shape->chunk_tokens;
    if (n > 65536) return fail(KV_ESHAPE, "device planning handles at most 65536 chunks, not %d", n);
    const int k8 = static_cast<int>(static_cast<int64_t>(n) * num8 / den);
    const int k84 = static_cast<int>(static_cast<int64_t>(n) * (num8 + num4) / den);
    RecordBytes rec;
    const bool i8 = is_i8(*shape);
    rec.w16 = i8 ? 0 : kv_record_bytes(shape, 16);
    rec.w8 = kv_record_bytes(shape, 8);
    rec.w4 = kv_record_bytes(shape, 4);
    rec.w2 = kv_record_bytes(shape, 2);
    rec.w1 = i8 ? kv_record_bytes(shape, 1) : 0;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (n <= kPlanScanThreads) {
        const int width = (n + 63) / 64 * 64;
        int parts = 1;
        while (parts < 16 && 2 * parts * width <= kPlanScanThreads) parts *= 2;
        hipLaunchKernelGGL(plan_small_kernel, dim3(1), dim3(parts * width), 0, st, density_dev, n, width, k8, k84,
                           shape->chunk_tokens, rec, bits_dev, off_dev, dst_tok_dev);
        return launch_status("plan_small_kernel launch");
    }
    hipLaunchKernelGGL(plan_bits_kernel, dim3((n + kPlanRankThreads - 1) / kPlanRankThreads),
                       dim3(kPlanRankThreads), 0, st, density_dev, n, k8, k84, shape->chunk_tokens,
                       bits_dev, dst_tok_dev);
    if (int rc = launch_status("plan_bits_kernel launch")) return rc;
    hipLaunchKernelGGL(plan_offsets_kernel, dim3(1), dim3(kPlanScanThreads), 0, st, bits_dev, n, rec, off_dev);
    return launch_status("plan_offsets_kernel launch");
}

int32_t kv_plan_optimise_dev(const kv_shape_t* shape, const float* density_dev, int32_t ratio_num,
                             int32_t ratio_den, int32_t objective, uint8_t* bits_dev, uint64_t* off_dev,
                             int32_t* dst_tok_dev, int32_t* counts_dev, void* stream) {
    if (int rc = check_shape(shape)) return rc;
    if (is_i8(*shape)) return fail(KV_ESHAPE, "Eq. 3 is stated for the levels {8/8, 4/8, 2/8}: fp16 formats only");
    if (!density_dev || !bits_dev || !off_dev || !dst_tok_dev) return fail(KV_EINVAL, "NULL device pointer");
    if (!aligned(density_dev, 4) || !aligned(off_dev, 8) || !aligned(dst_tok_dev, 4) ||
        (counts_dev && !aligned(counts_dev, 4)))
        return fail(KV_EINVAL, "density_dev/dst_tok_dev/counts_dev must be 4-byte aligned, off_dev 8-byte aligned");
    if (ratio_den <= 0 || ratio_num <= 0) return fail(KV_EINVAL, "need a positive ratio");
    if (static_cast<int64_t>(ratio_num) * 4 < ratio_den || ratio_num > ratio_den)
        return fail(KV_EINVAL, "ratio %d/%d outside [1/4, 1]", ratio_num, ratio_den);
    if (objective != KV_OBJ_BITS_TO_DENSE && objective != KV_OBJ_AS_PRINTED)
        return fail(KV_EINVAL, "objective %d unknown", objective);
    const int32_t n = shape->n_tokens / shape->chunk_tokens;
    if (n > kPlanOptMaxChunks)
        return fail(KV_ESHAPE, "device optimiser handles at most %d chunks, not %d", kPlanOptMaxChunks, n);
    // the one free variable of Eq. 3 and its feasible range, as in kv_bits_optimise
    int64_t M = static_cast<int64_t>(n) * (4LL * ratio_num - ratio_den) / ratio_den;
    if (M == 3LL * n - 1) --M;
    const int64_t k8_lo = std::max<int64_t>(0, (M - n + 1) / 2);
    const int64_t k8_hi = M / 3;
    RecordBytes rec;
    rec.w16 = kv_record_bytes(shape, 16);
    rec.w8 = kv_record_bytes(shape, 8);
    rec.w4 = kv_record_bytes(shape, 4);
    rec.w2 = kv_record_bytes(shape, 2);
    rec.w1 = 0;
    const double w4 = objective == KV_OBJ_BITS_TO_DENSE ? 0.5 : 2.0;
    const double w2 = objective == KV_OBJ_BITS_TO_DENSE ? 0.25 : 4.0;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // ranks into dst_tok_dev, densities in rank order (as doubles) into off_dev: the two outputs serve as
    // the scratch between the kernels
    hipLaunchKernelGGL(plan_rank_kernel, dim3((n + kPlanRankThreads - 1) / kPlanRankThreads), dim3(kPlanRankThreads),
                       0, st, density_dev, n, dst_tok_dev, reinterpret_cast<double*>(off_dev));
    if (int rc = launch_status("plan_rank_kernel launch")) return rc;
    hipLaunchKernelGGL(plan_optimise_kernel, dim3(1), dim3(kPlanScanThreads), 0, st, n, M, static_cast<int>(k8_lo),
                       static_cast<int>(k8_hi), w4, w2, shape->chunk_tokens, rec, off_dev, dst_tok_dev, bits_dev,
                       counts_dev);
    return launch_status("plan_optimise_kernel launch");
}

// --------------------------------------------------------------------- streaming Load / AoT swap-out

// Events of a streaming Load: copied[b] is recorded on the copy stream behind the copies into staging
// slot b, consumed[b] on the compute stream behind the kernel that read the slot.
struct kv_loader {
    hipEvent_t copied[8];
    hipEvent_t consumed[8];
    bool slot_used[8];       // consumed[b] has been recorded: the slot may still be read by that kernel
    int n_events;
    // the staging layout of the last call and the slot its successor starts with (calls one after the
    // other walk the slots round robin instead of all queueing for slot 0)
    const void* staging;
    uint64_t staging_bytes;
    int n_buffers, next;
    // consumed[b] was the seq[b]-th event recorded, all of them on `compute`: an event of that stream
    // having fired, every one recorded before it has fired too
    uint64_t seq[8], recorded;
    const void* compute;
};

static void loader_release(kv_loader* ld) {
    for (int i = 0; i < ld->n_events; ++i) {
        (void)hipEventDestroy(ld->copied[i]);
        (void)hipEventDestroy(ld->consumed[i]);
    }
    ld->n_events = 0;
}

static int loader_init(kv_loader* ld, int n) {
    ld->n_events = 0;
    for (int i = 0; i < 8; ++i) ld->slot_used[i] = false;
    ld->staging = nullptr;
    ld->staging_bytes = 0;
    ld->n_buffers = 0;
    ld->next = 0;
    ld->recorded = 0;
    ld->compute = nullptr;
    for (int i = 0; i < 8; ++i) ld->seq[i] = 0;
    for (; ld->n_events < n; ++ld->n_events) {
        hipError_t e = hipEventCreateWithFlags(&ld->copied[ld->n_events], hipEventDisableTiming);
        if (e == hipSuccess) {
            e = hipEventCreateWithFlags(&ld->consumed[ld->n_events], hipEventDisableTiming);
            if (e != hipSuccess) (void)hipEventDestroy(ld->copied[ld->n_events]);
        }
        if (e != hipSuccess) {
            loader_release(ld);
            return hip_fail(e, "hipEventCreateWithFlags");
        }
    }
    return KV_OK;
}

kv_loader_t* kv_loader_create(void) {
    kv_loader* ld = new (std::nothrow) kv_loader;
    if (!ld) {
        fail(KV_ENOMEM, "out of host memory");
        return nullptr;
    }
    if (loader_init(ld, 8) != KV_OK) {
        delete ld;
        return nullptr;
    }
    return ld;
}

void kv_loader_destroy(kv_loader_t* ld) {
    if (!ld) return;
    loader_release(ld);
    delete ld;
}

int32_t kv_swapin_stream(kv_loader_t* ld, const kv_shape_t* shape, const void* packed_pinned,
                         const uint64_t* src_off, const int32_t* dst_tok, const uint8_t* sel_bits, int32_t n_sel,
                         void* staging_dev, uint64_t staging_bytes, int32_t n_buffers, void* kv_out,
                         void* copy_stream, void* compute_stream) {
    if (!ld) return fail(KV_EINVAL, "NULL loader");
    if (int rc = check_shape(shape)) return rc;
    const int32_t n_chunks = shape->n_tokens / shape->chunk_tokens;
    if (n_sel < 0 || n_sel > n_chunks) return fail(KV_EINVAL, "n_sel %d outside [0,%d]", n_sel, n_chunks);
    if (n_sel == 0) return KV_OK;
    if (!packed_pinned || !src_off || !dst_tok || !sel_bits || !staging_dev || !kv_out)
        return fail(KV_EINVAL, "NULL pointer");
    if (n_buffers < 2 || n_buffers > 8) return fail(KV_EINVAL, "n_buffers %d outside [2,8]", n_buffers);
    if (!copy_stream || !compute_stream || copy_stream == compute_stream)
        return fail(KV_EINVAL, "copy_stream and compute_stream must be two distinct non-NULL streams");
    if (!aligned(staging_dev, 256) || !aligned(kv_out, 16) || !aligned(packed_pinned, 16))
        return fail(KV_EINVAL, "staging_dev must be 256-byte aligned, kv_out/packed_pinned 16-byte");
    const uint64_t slot = (staging_bytes / static_cast<uint64_t>(n_buffers)) & ~static_cast<uint64_t>(255);
    uint64_t largest = 0;
    for (int32_t j = 0; j < n_sel; ++j) {
        if (!valid_bits(*shape, sel_bits[j])) return fail(KV_EBITS, "sel_bits[%d] = %d", j, sel_bits[j]);
        if (dst_tok[j] < 0 || dst_tok[j] % shape->chunk_tokens ||
            dst_tok[j] + shape->chunk_tokens > shape->n_tokens)
            return fail(KV_EINDEX, "dst_tok[%d] = %d is not a chunk start inside the cache", j, dst_tok[j]);
        if (j && src_off[j] < src_off[j - 1] + record_bytes(*shape, sel_bits[j - 1]))
            return fail(KV_EINDEX, "src_off not ascending / records overlap at position %d", j);
        if (src_off[j] % 16) return fail(KV_EINVAL, "src_off[%d] not 16-byte aligned", j);
        largest = std::max(largest, record_bytes(*shape, sel_bits[j]));
    }
    if (slot < largest)
        return fail(KV_ENOMEM, "staging slot %llu bytes, largest record %llu",
                    static_cast<unsigned long long>(slot), static_cast<unsigned long long>(largest));

    const bool i8 = is_i8(*shape);
    int ppl = 0;
    QuantGeom g = i8 ? quant_geom_i8(*shape, &ppl) : quant_geom(*shape);
    if (!i8) ppl = plan_tasks(&g, kSwapinPiecesPerLane);
    hipStream_t cs = static_cast<hipStream_t>(copy_stream);
    hipStream_t ks = static_cast<hipStream_t>(compute_stream);
    const uint8_t* host = static_cast<const uint8_t*>(packed_pinned);
    uint8_t* staging = static_cast<uint8_t*>(staging_dev);
    if (ld->staging != staging_dev || ld->staging_bytes != staging_bytes || ld->n_buffers != n_buffers ||
        ld->compute != compute_stream) {
        // another staging layout than the last call's (its slots do not correspond to the old ones) or another
        // compute stream (its events say nothing about the old one's): the copies of this call wait for
        // every kernel that may still read a slot
        for (int b = 0; b < 8; ++b)
            if (ld->slot_used[b]) {
                KV_HIP(hipStreamWaitEvent(cs, ld->consumed[b], 0));
                ld->slot_used[b] = false;
            }
        ld->staging = staging_dev;
        ld->staging_bytes = staging_bytes;
        ld->n_buffers = n_buffers;
        ld->next = 0;
        ld->compute = compute_stream;
    }
    // Every wait on the copy stream costs the copy engine a pause between two copies (measured: 128 copies of
    // 5.6 MB with a wait before each take 3.5 ms longer than without).  The first n_buffers batches of this
    // call reuse slots of earlier calls in the order these were used: ONE wait, for the newest of those that
    // lie ahead, serves them all; later batches reuse slots of this call and wait one by one.
    uint64_t waited = 0;
    {
        // batches of this call: consecutive records while they fit a slot, at most kBatchMax each (as below)
        int n_batches = 0;
        for (int32_t k = 0; k < n_sel && n_batches < n_buffers; ++n_batches) {
            uint64_t used = 0;
            int n = 0;
            while (k < n_sel && n < kBatchMax && used + record_bytes(*shape, sel_bits[k]) <= slot) {
                used += record_bytes(*shape, sel_bits[k]);
                ++n;
                ++k;
            }
        }
        int newest = -1;
        for (int k = 0; k < n_batches; ++k) {
            const int b = (ld->next + k) % n_buffers;
            if (ld->slot_used[b] && (newest < 0 || ld->seq[b] > ld->seq[newest])) newest = b;
        }
        if (newest >= 0) {
            KV_HIP(hipStreamWaitEvent(cs, ld->consumed[newest], 0));
            waited = ld->seq[newest];
        }
    }
    int32_t j = 0;
    while (j < n_sel) {
        const int b = ld->next;
        ld->next = (ld->next + 1) % n_buffers;
        uint8_t* slot_dev = staging + static_cast<uint64_t>(b) * slot;
        // records of one batch: as many consecutive list entries as fit the slot
        SwapinBatch list;
        list.n = 0;
        uint64_t used = 0;
        // the slot is free once the kernel that last read it has finished (an earlier batch of this
        // call, or of an earlier call through this loader)
        if (ld->slot_used[b] && ld->seq[b] > waited) {
            KV_HIP(hipStreamWaitEvent(cs, ld->consumed[b], 0));
            waited = ld->seq[b];
        }
        while (j < n_sel && list.n < kBatchMax) {
            const uint64_t bytes = record_bytes(*shape, sel_bits[j]);
            if (used + bytes > slot) break;
            // extend the copy over records that are adjacent in the host pool
            int32_t j2 = j;
            uint64_t run = 0;
            while (j2 < n_sel && list.n + (j2 - j) < kBatchMax) {
                const uint64_t bj = record_bytes(*shape, sel_bits[j2]);
                if (src_off[j2] != src_off[j] + run || used + run + bj > slot) break;
                run += bj;
                ++j2;
            }
            KV_HIP(hipMemcpyAsync(slot_dev + used, host + src_off[j], run, hipMemcpyHostToDevice, cs));
            uint64_t o = used;
            for (int32_t k = j; k < j2; ++k) {
                list.src_off[list.n] = o;
                list.dst_tok[list.n] = dst_tok[k];
                list.bits[list.n] = sel_bits[k];
                ++list.n;
                o += record_bytes(*shape, sel_bits[k]);
            }
            used += run;
            j = j2;
        }
        KV_HIP(hipEventRecord(ld->copied[b], cs));
        KV_HIP(hipStreamWaitEvent(ks, ld->copied[b], 0));
        if (int rc = launch_swapin_batch(*shape, g, ppl, slot_dev, list, static_cast<u4_t*>(kv_out), ks)) return rc;
        KV_HIP(hipEventRecord(ld->consumed[b], ks));
        ld->slot_used[b] = true;
        ld->seq[b] = ++ld->recorded;
    }
    return KV_OK;
}

int32_t kv_swapin_pinned(const kv_shape_t* shape, const void* packed_pinned, const uint64_t* src_off,
                         const int32_t* dst_tok, const uint8_t* sel_bits, int32_t n_sel,
                         void* staging_dev, uint64_t staging_bytes, int32_t n_buffers, void* kv_out,
                         void* copy_stream, void* compute_stream) {
    if (n_buffers < 2 || n_buffers > 8) return fail(KV_EINVAL, "n_buffers %d outside [2,8]", n_buffers);
    if (n_sel == 0) {
        if (int rc = check_shape(shape)) return rc;
        return KV_OK;
    }
    kv_loader once;
    if (int rc = loader_init(&once, n_buffers)) return rc;
    const int32_t rc = kv_swapin_stream(&once, shape, packed_pinned, src_off, dst_tok, sel_bits, n_sel, staging_dev,
                                        staging_bytes, n_buffers, kv_out, copy_stream, compute_stream);
    loader_release(&once);
    return rc;
}

int32_t kv_swapout_aot(const void* packed_dev, void* packed_pinned, uint64_t begin, uint64_t end,
                       void* producer_stream, void* copy_stream) {
    if (!packed_dev || !packed_pinned) return fail(KV_EINVAL, "NULL pointer");
    if (end < begin) return fail(KV_EINVAL, "end < begin");
    if (!copy_stream || copy_stream == producer_stream)
        return fail(KV_EINVAL, "copy_stream must be non-NULL and differ from producer_stream");
    if (end == begin) return KV_OK;
    hipEvent_t produced;
    KV_HIP(hipEventCreateWithFlags(&produced, hipEventDisableTiming));
    hipError_t e = hipEventRecord(produced, static_cast<hipStream_t>(producer_stream));
    if (e == hipSuccess) e = hipStreamWaitEvent(static_cast<hipStream_t>(copy_stream), produced, 0);
    if (e == hipSuccess)
        e = hipMemcpyAsync(static_cast<uint8_t*>(packed_pinned) + begin,
                           static_cast<const uint8_t*>(packed_dev) + begin, end - begin,
                           hipMemcpyDeviceToHost, static_cast<hipStream_t>(copy_stream));
    (void)hipEventDestroy(produced);
    if (e != hipSuccess) return hip_fail(e, "AoT swap-out enqueue");
    return KV_OK;
}

}  // extern "C"
