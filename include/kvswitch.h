/*
 * kvswitch.h - C ABI of libkvswitch: chunk-wise KV-cache scoring, compression
 * and swap-in for LLM context switching on one AMD MI355X (gfx950) GPU.
 *
 * The operations are those of "LLM as a System Service on Mobile Devices"
 * (arXiv 2403.11805): the context memory of an LLM is a KV cache cut along the
 * token axis into fixed-size chunks (Sec. 3.1, chunk memory model); a chunk is
 * compressed at a bit-width chosen from its attention-derived information
 * density (Sec. 3.2, Eq. 1 and Eq. 2), swapped out ahead of time (Sec. 3.4,
 * AoT swapping), evicted in LCTRU order (Sec. 3.4) and brought back by the
 * Load primitive (Sec. 3.1, primitives; Sec. 3.3).
 *
 * Conventions
 *  - Every function returns 0 (KV_OK) or a negative kv_status; a text for the
 *    last failure on the calling thread is available from kv_last_error().
 *    No C++ exception crosses this boundary.
 *  - The caller owns every buffer.  "dev" pointers are device (HBM) addresses,
 *    "host" pointers ordinary host memory, "pinned" host memory obtained from
 *    hipHostMalloc (or torch pin_memory).  The library keeps no pointer after a
 *    call returns and allocates no device memory (kv_swapin_pinned and
 *    kv_swapout_aot create and destroy a few HIP events per call, a
 *    kv_loader_t handle owns its events until it is destroyed; a
 *    kv_recompute_t handle owns the GEMM library's handle, with that library's
 *    own device workspace, until it is destroyed).
 *  - Device entry points only enqueue work on the caller's hipStream_t (passed
 *    as void*, NULL = the default stream) and never synchronise (the one
 *    exception, kv_recompute_tune, says so).  Host
 *    arguments are validated before anything is enqueued: a validation error
 *    (KV_EINVAL, KV_ESHAPE, KV_EBITS, KV_EINDEX, KV_ENOMEM) means nothing was
 *    launched and nothing written.  KV_EHIP reports a failed HIP runtime call;
 *    from an entry point that enqueues several launches or copies
 *    (kv_swapin_stream / kv_swapin_pinned, kv_load_chunks with more than 64
 *    records, kv_recompute_layer, kv_score_chunks) the earlier ones may already
 *    be enqueued: the output buffers, staging and workspace are then undefined
 *    until the streams have drained.  Device-side lists
 *    (bits, offsets, gather lists) are trusted: the caller builds them with
 *    the host helpers below, which validate them.
 *  - fp16 inputs must be finite; NaN/Inf give unspecified codes.
 *  - Threads: the pure host functions and the device entry points keep no state
 *    between calls (the error text is per thread) and may be called from several
 *    threads at once, each on streams of its own.  A kv_lctru_t queue, a kv_loader_t and a
 *    kv_recompute_t handle are not synchronised: one thread at a time per object
 *    (the service of Sec. 3 is a single process with one bookkeeping thread).
 *
 * Layouts
 *  fp16 KV cache (dev), contiguous: [n_layers][2 (K=0,V=1)][n_kv_heads][n_tokens][head_dim].
 *  A "slab" is the chunk_tokens x head_dim block of one (layer, K|V, kv-head)
 *  for one token chunk; a chunk is all n_layers*2*n_kv_heads slabs of the same
 *  chunk_tokens tokens and has ONE bit-width (Sec. 3.1: same number of tokens
 *  and same in-chunk ratio per chunk).
 *
 *  Packed record of a chunk with bit-width b in {8,4,2}, sections back to back:
 *    codes : [n_layers][2][n_kv_heads][chunk_tokens][head_dim*b/8] bytes; in a
 *            token row element d sits in byte d*b/8 at bit (d mod (8/b))*b,
 *            lowest-index element in the least-significant bits (Sec. 4:
 *            sub-byte codes are bit-shifted into 8-bit containers);
 *    scale : [n_layers][2][n_kv_heads][chunk_tokens][head_dim/group] fp32;
 *    mn    : same shape, fp32 (the group minimum).
 *  b = 16 is pass-through: the record is the chunk's fp16 bytes in the order
 *  [n_layers][2][n_kv_heads][chunk_tokens][head_dim], no metadata.
 *  Record i starts at byte offset off[i] of the packed pool (kv_chunk_offsets).
 *
 *  The above is format KV_FMT_F16_GROUPS (shape.format = 0).  Format
 *  KV_FMT_I8_CHANNELS (= 1) follows the paper's own setting more closely (Sec. 3.2
 *  "Compressing chunks", Sec. 4): the cache is already stored as 8-bit integers
 *  by the engine, [n_layers][2][n_kv_heads][n_tokens][head_dim] int8, and a chunk
 *  is quantised further, channel-wise: one (scale, mn) pair per head_dim channel
 *  of a slab, taken over the slab's chunk_tokens tokens.  Widths {8, 4, 2, 1};
 *  8 is pass-through (the slab's int8 bytes).  Record for b < 8:
 *    codes : [slab][chunk_tokens][head_dim*b/8] bytes, bit order as above;
 *    scale : [slab][head_dim] fp32;   mn : [slab][head_dim] fp32.
 *  Same arithmetic as below with x the int8 value as binary32; dequantisation
 *  gives int8(clamp(rint(fp32(code) * scale + mn), -128, 127)).
 *
 *  KV_FMT_I8_CHANNELS_H (= 2) is format 1 with the parameters held in binary16:
 *  at 16 tokens per chunk the two fp32 parameters of a channel weigh as much as
 *  its 4-bit codes, and halves cut that in two.  scale is rounded to binary16
 *  (nearest even) BEFORE the codes are computed, so that quantisation and
 *  dequantisation use the same stored value; mn is an integer in [-128, 127],
 *  exact in binary16.  Record for b < 8: codes as in format 1, then
 *    scale : [slab][head_dim] binary16;   mn : [slab][head_dim] binary16.
 *
 *  KV_FMT_F16_GROUPS_H (= 3) is format 0 with scale and mn held in binary16 (the
 *  record's parameter sections shrink from 8 to 4 bytes per group: 8 % smaller
 *  records at group 64 and terciles of 8/4/2 bits, which is what a Load over the
 *  host link pays for).  As in format 2 the scale is rounded to binary16 (nearest
 *  even) BEFORE the codes are computed; mn is one of the fp16 inputs, exact.  A
 *  code may then saturate at 2^b - 1 where the rounded scale falls short of the
 *  range (by at most range * 2^-11).
 *
 *  Quantisation of one group of `group` consecutive head_dim elements of one
 *  token (linear min/max quantisation, Sec. 3.2 "Compressing chunks"), all in
 *  IEEE binary32, round-to-nearest, no contraction:
 *    mn = min x + 0.0f, mx = max x + 0.0f, scale = (mx - mn) / (2^b - 1),
 *    code = scale == 0 ? 0 : clamp(rint((x - mn) / scale), 0, 2^b - 1)
 *  with rint rounding halves to even.  Dequantisation: fp16_rne(fp32(code) *
 *  scale + mn), product and sum rounded separately.
 */
#ifndef KVSWITCH_H
#define KVSWITCH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    KV_OK      = 0,
    KV_EINVAL  = -1,  /* NULL pointer or argument out of range            */
    KV_ESHAPE  = -2,  /* kv_shape_t violates the requirements below        */
    KV_EBITS   = -3,  /* a bit-width outside {16,8,4,2} ({8,4,2,1}: int8 formats) */
    KV_EINDEX  = -4,  /* chunk index out of range, unsorted or repeated    */
    KV_ENOMEM  = -5,  /* capacity too small / not enough evictable bytes   */
    KV_EHIP    = -6   /* a HIP runtime call failed (text has the HIP error) */
} kv_status;

/* Geometry of one context's KV cache.
 * Requirements (else KV_ESHAPE): all fields > 0; n_tokens % chunk_tokens == 0
 * (chunks hold the same number of tokens, Sec. 3.1); head_dim % group == 0;
 * group in {64, 128, 256, 512}; n_q_heads % n_kv_heads == 0; head_dim <= 1024;
 * chunk_tokens <= 1024; chunk_tokens * head_dim % 512 == 0;
 * (chunk_tokens * head_dim / group) % 4 == 0 (keeps every record section
 * 16-byte aligned).
 * Formats 1 and 2 instead of the group rules: head_dim a power of two in [64, 1024];
 * chunk_tokens * head_dim in {1024, 2048, 4096} (one wavefront holds a slab);
 * group is ignored.  Scoring (kv_score_chunks) needs an fp16 cache (format 0 or 3). */
typedef struct {
    int32_t n_layers;
    int32_t n_kv_heads;
    int32_t n_q_heads;     /* used by kv_score_chunks only */
    int32_t head_dim;
    int32_t n_tokens;
    int32_t chunk_tokens;
    int32_t group;         /* quantisation group along head_dim (format 0) */
    int32_t format;        /* KV_FMT_F16_GROUPS (0), KV_FMT_I8_CHANNELS (1), KV_FMT_I8_CHANNELS_H (2), KV_FMT_F16_GROUPS_H (3) */
} kv_shape_t;

enum { KV_FMT_F16_GROUPS = 0, KV_FMT_I8_CHANNELS = 1, KV_FMT_I8_CHANNELS_H = 2, KV_FMT_F16_GROUPS_H = 3 };

enum { KV_NORM_VISIBLE = 0, KV_NORM_NONE = 1 };

/* Text of the last error on this thread (never NULL; "" if none). */
const char* kv_last_error(void);

/* ---------------------------------------------------------------- host, pure */

/* Bytes of one chunk's packed record at bit-width `bits`; 0 if shape or bits
 * are invalid.  Format 0: b<16: slabs*T*(D*b/8 + 8*D/G); b=16: slabs*T*D*2.
 * Format 1: b<8: slabs*(T*D*b/8 + 8*D); b=8: slabs*T*D.  Format 2: 4*D in the place of 8*D.
 * Format 3: format 0 with 4*D/G in the place of 8*D/G. */
uint64_t kv_record_bytes(const kv_shape_t* shape, int32_t bits);

/* Exclusive prefix sum of record sizes: off[0]=0, off[i+1]=off[i]+record_bytes(bits[i]).
 * bits: host [n_chunks]; off: host [n_chunks+1].  Chunks are compressed and
 * swapped independently (Sec. 1 / Sec. 3.1), so records are self-contained. */
int32_t kv_chunk_offsets(const kv_shape_t* shape, const uint8_t* bits, uint64_t* off);

/* Rank chunks by density and bucket them (Sec. 3.2, Eq. 2, with fixed
 * thresholds): order by (density descending, index ascending); the first
 * k8 = n*num8/den chunks get 8 bits, the next k4 = n*(num8+num4)/den - k8 get
 * 4 bits, the rest 2 bits (integer division).  density: host [n]; bits: host [n].
 * Requires den > 0, num8 >= 0, num4 >= 0, num8 + num4 <= den and finite densities
 * (a NaN orders with nothing: KV_EINVAL). */
int32_t kv_bits_from_scores(const float* density, int32_t n, int32_t num8,
                            int32_t num4, int32_t den, uint8_t* bits);

/* Thresholds from a global ratio (Sec. 3.2, Eq. 2 and Eq. 3) for the paper's
 * three levels {8/8, 4/8, 2/8}: chunks are ranked as in kv_bits_from_scores and
 * the k8 densest get 8 bits, the next k4 get 4 bits, the remaining k2 get 2 bits,
 * where (k8, k4, k2) maximises
 *     ctxInfo = w8 * S8 + w4 * S4 + w2 * S2      (S = sum of densities in the bucket)
 * subject to the average ratio (k8 + k4/2 + k2/4) / n being the largest value some
 * split reaches that is not above ratio_num / ratio_den.  That leaves one free variable, k8:
 * 3*k8 + k4 = M = floor(n * (4*ratio_num - ratio_den) / ratio_den), k2 = n - k8 - k4
 * (M = 3n - 1, which no split reaches, is replaced by 3n - 2),
 * and every feasible k8 is tried.  objective selects the weights:
 *   KV_OBJ_BITS_TO_DENSE  (w8, w4, w2) = (1, 1/2, 1/4) = ratio_w: the reading that
 *                          gives denser chunks more bits (the stated intent);
 *   KV_OBJ_AS_PRINTED     (1, 2, 4) = 1 / ratio_w: Eq. 3 exactly as printed.
 * Sums are accumulated in double in rank order; of equal maxima the smallest k8
 * wins.  density, bits: host [n]; counts (may be NULL): host [3] = k8, k4, k2.
 * Requires n >= 0, ratio_den > 0, 1/4 <= ratio_num/ratio_den <= 1, finite densities. */
enum { KV_OBJ_BITS_TO_DENSE = 0, KV_OBJ_AS_PRINTED = 1 };
int32_t kv_bits_optimise(const float* density, int32_t n, int32_t ratio_num,
                         int32_t ratio_den, int32_t objective, uint8_t* bits,
                         int32_t* counts);

/* Swapping-recompute pipeline, profiling and planning (Sec. 3.3 i and ii, Eq. 4).
 * Delays are modelled as lines fitted to a few measured points: recompute
 * T_re(x) = re_per_chunk * x + re_fixed for x chunks, IO T_IO(m) = io_per_byte * m
 * + io_fixed for m bytes; a stage with nothing to do takes no time
 * (T_re(0) = T_IO(0) = 0). */
typedef struct {
    double re_per_chunk, re_fixed;   /* seconds */
    double io_per_byte, io_fixed;    /* seconds */
} kv_pipeline_model_t;

/* Least-squares line t = slope * x + intercept through n >= 2 points with at
 * least two different x (else KV_EINVAL).  All pointers host. */
int32_t kv_fit_line(const double* x, const double* t, int32_t n, double* slope, double* intercept);

/* Eq. 4: of the missing[w] chunks of width w = 8, 4, 2 bits (index 0, 1, 2; record
 * sizes record_bytes[w], strictly decreasing) choose how many to recompute,
 * recompute[w] <= missing[w], so that
 *     max( T_re(sum_w recompute[w]),  T_IO(sum_w (missing[w] - recompute[w]) * record_bytes[w]) )
 * is smallest.  For a given number of recomputed chunks the heaviest records are
 * taken off the IO first (T_IO does not decrease with bytes), so every total
 * 0..sum(missing) is tried with that choice; of equal delays the smallest total
 * wins.  delay (may be NULL) receives the minimum.  Requires non-negative model
 * slopes and intercepts. */
int32_t kv_plan_pipeline(const kv_pipeline_model_t* model, const int32_t* missing,
                         const uint64_t* record_bytes, int32_t* recompute, double* delay);

/* The chunks a plan of Eq. 4 sends to each stage (Sec. 3.3 ii): of the n_missing chunks
 * missing_idx (strictly ascending, else KV_EINDEX) with widths bits[i] (host [n_chunks]), the
 * recompute[w] EARLIEST chunks of width 8, 4, 2 (w = 0, 1, 2) go to the recompute stage, all
 * others - pass-through and 1-bit chunks included - to the Load.  (The paper leaves open which
 * chunks of a width are recomputed; the earliest depend on the fewest loaded chunks.)
 * recompute_idx, load_idx: host, room for n_missing entries each, filled in ascending order;
 * load_idx is what kv_build_gather / kv_load_chunks take, recompute_idx what
 * kv_recompute_layer takes.  KV_EINVAL if the plan recomputes more chunks of a width than are
 * missing. */
int32_t kv_pipeline_split(const kv_shape_t* shape, const uint8_t* bits, const int32_t* missing_idx,
                          int32_t n_missing, const int32_t* recompute,
                          int32_t* recompute_idx, int32_t* n_recompute,
                          int32_t* load_idx, int32_t* n_load);

/* Load primitive, list building (Sec. 3.1, primitive 3): for n_sel strictly
 * ascending chunk indices produce src_off[j] = off[idx_j], dst_tok[j] =
 * idx_j*chunk_tokens, sel_bits[j] = bits[idx_j].  All pointers host. */
int32_t kv_build_gather(const kv_shape_t* shape, const uint64_t* off, const uint8_t* bits,
                        const int32_t* chunk_idx, int32_t n_sel,
                        uint64_t* src_off, int32_t* dst_tok, uint8_t* sel_bits);

/* ------------------------------------------------------------ device, async */

/* Bytes of device workspace kv_score_chunks needs for this shape and number
 * of query rows; 0 on invalid arguments. */
uint64_t kv_score_workspace_bytes(const kv_shape_t* shape, int32_t n_queries);

/* Information density of every chunk (Sec. 3.2, Eq. 1).
 *   q    dev fp16 [n_layers][n_q_heads][n_queries][head_dim]: the query rows of
 *        the last n_queries tokens (row r sits at position n_tokens-n_queries+r);
 *        1 <= n_queries <= min(n_tokens, 256).  Scoring additionally needs
 *        head_dim in {64,128,256}, chunk_tokens a power of two >= 8 and
 *        n_tokens % 32 == 0, and at most 2 097 152 tokens (16 777 216 where
 *        several blocks of 32 query rows share a kv head) (else KV_ESHAPE).
 *   kv   dev fp16 cache; only the K planes are read.  Query head h attends to
 *        kv head h / (n_q_heads / n_kv_heads).
 *   A = softmax(causal_mask(Q K^T / sqrt(head_dim))) per (layer, head), fp32.
 *   norm_mode KV_NORM_VISIBLE: each column is averaged over the rows that can
 *        see it (the reading fixed by the paper's worked example of Eq. 1);
 *        KV_NORM_NONE: plain column sums (their total per head is n_queries).
 *   chunk_mass dev fp32 [n_layers][n_q_heads][n_chunks]: sum over the chunk's
 *        columns of the normalised column mass.
 *   density    dev fp32 [n_chunks]: mean of chunk_mass over layers and heads,
 *        divided by chunk_tokens (= D_i of Eq. 1).
 *   workspace  dev, >= kv_score_workspace_bytes(), 256-byte aligned; contents
 *        are scratch. */
int32_t kv_score_chunks(const kv_shape_t* shape, const void* q, int32_t n_queries,
                        const void* kv, int32_t norm_mode,
                        void* workspace, uint64_t workspace_bytes,
                        float* chunk_mass, float* density, void* stream);

/* The same for a context of n_valid tokens in a cache padded to n_tokens (Sec. 3.2,
 * Eq. 1 on the valid prefix; contexts whose length is no multiple of chunk_tokens or
 * of 32 are padded by the caller): n_queries <= n_valid <= n_tokens (else KV_EINVAL);
 * the query rows are the last n_queries VALID tokens (row r sits at position
 * n_valid-n_queries+r), no row sees a padding token and what the padding holds is
 * never used (it may be anything, NaN included).  Chunk i holds its tokens
 * [i*chunk_tokens, min((i+1)*chunk_tokens, n_valid)): its chunk_mass sums those columns
 * and its density is divided by the number of tokens it really has (0 for a chunk of
 * padding only).  With n_valid == n_tokens this is kv_score_chunks.  Compression and
 * swap-in treat the padded cache like any other. */
int32_t kv_score_chunks_valid(const kv_shape_t* shape, const void* q, int32_t n_queries,
                              const void* kv, int32_t n_valid, int32_t norm_mode,
                              void* workspace, uint64_t workspace_bytes,
                              float* chunk_mass, float* density, void* stream);

/* kv_score_chunks for callers that cannot allocate device memory and so have no workspace to
 * hand over: code running under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  The partial results live in a static device array of KV_SCORE_STATIC_BYTES that
 * every GPU the library runs on holds until the process ends; the call allocates and frees
 * nothing (its first call on a device looks the array's address up).  Same arguments and
 * results as kv_score_chunks without the workspace pair.  A shape whose scoring needs more
 * scratch than the array holds is refused with KV_ENOMEM (kv_score_workspace_bytes tells; a
 * shape that one workgroup per head scores in LDS - one block of query rows per head and at
 * least 256 (layer, head) pairs, e.g. a 4096-token multi-head cache - needs none).  All calls
 * on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two
 * threads) race and give undefined results; calls one after the other on a stream need no
 * clearing in between. */
#define KV_SCORE_STATIC_BYTES (32u << 20)
int32_t kv_score_chunks_static(const kv_shape_t* shape, const void* q, int32_t n_queries,
                               const void* kv, int32_t norm_mode,
                               float* chunk_mass, float* density, void* stream);

/* Widths, record offsets and the whole-cache gather list computed on the device
 * (Sec. 3.2, Eq. 2 with fixed thresholds; Sec. 3.1 primitive 3), for callers that
 * keep scoring, compression and swap-in on one stream with no host round trip.
 * The results equal, bit for bit, those of kv_bits_from_scores(density, n_chunks,
 * num8, num4, den) followed by kv_chunk_offsets and by kv_build_gather over all
 * chunks:
 *   density_dev dev fp32 [n_chunks], finite (e.g. kv_score_chunks' output on the
 *               same stream);
 *   bits_dev    dev u8  [n_chunks]    widths; also the sel_bits list;
 *   off_dev     dev u64 [n_chunks+1]  record offsets; its first n_chunks entries
 *               are the src_off list, off_dev[n_chunks] the packed size;
 *   dst_tok_dev dev i32 [n_chunks]    i * chunk_tokens.
 * Fractions as for kv_bits_from_scores (else KV_EINVAL); n_chunks <= 65536 (else
 * KV_ESHAPE).  The packed pool must hold the worst case, n_chunks records of 8
 * bits, since the host does not learn the packed size before it enqueues the
 * compression. */
int32_t kv_plan_chunks_dev(const kv_shape_t* shape, const float* density_dev,
                           int32_t num8, int32_t num4, int32_t den,
                           uint8_t* bits_dev, uint64_t* off_dev, int32_t* dst_tok_dev,
                           void* stream);

/* The same with the thresholds chosen from a global ratio (Sec. 3.2, Eq. 2 and Eq. 3): the
 * results equal, bit for bit, those of kv_bits_optimise(density, n_chunks, ratio_num, ratio_den,
 * objective) followed by kv_chunk_offsets and by kv_build_gather over all chunks.  Chunks are
 * ranked by counting; the densities are added up in rank order, in double, by one thread (the
 * host function's order, so that equal maxima of ctxInfo break the same way) and every feasible
 * k8 is tried in parallel.
 *   density_dev / bits_dev / off_dev / dst_tok_dev as for kv_plan_chunks_dev (off_dev and
 *   dst_tok_dev also serve as scratch between the two kernels of the call);
 *   counts_dev  dev i32 [3] = (k8, k4, k2), may be NULL.
 * fp16 formats only (Eq. 3 is stated for the levels {8/8, 4/8, 2/8}); ratio and objective as
 * for kv_bits_optimise (else KV_EINVAL); n_chunks <= 8192 (else KV_ESHAPE: plan on the host).
 * The packed pool must hold the worst case, n_chunks records of 8 bits. */
int32_t kv_plan_optimise_dev(const kv_shape_t* shape, const float* density_dev,
                             int32_t ratio_num, int32_t ratio_den, int32_t objective,
                             uint8_t* bits_dev, uint64_t* off_dev, int32_t* dst_tok_dev,
                             int32_t* counts_dev, void* stream);

/* Quantise and bit-pack every chunk at its bit-width (Sec. 3.2 "Compressing
 * chunks"; Sec. 4 bit-shift packing).
 *   kv dev fp16 cache (read only); bits_dev dev u8 [n_chunks];
 *   off_dev dev u64 [n_chunks+1] from kv_chunk_offsets;
 *   packed_out dev, >= off[n_chunks] bytes, 16-byte aligned. */
int32_t kv_compress_chunks(const kv_shape_t* shape, const void* kv,
                           const uint8_t* bits_dev, const uint64_t* off_dev,
                           void* packed_out, void* stream);

/* The same for n_sel listed chunks only (the chunks a call has added or changed are
 * compressed and swapped out ahead of time when the call returns, Sec. 3.4 i): record
 * i of the list is written at off_dev[idx_i] with width bits_dev[idx_i]; other records
 * of the pool are not touched.
 *   chunk_idx_dev dev i32 [n_sel], distinct indices in [0, n_chunks) (trusted like the
 *   other device lists); bits_dev / off_dev as above, indexed by chunk.  n_sel == 0
 *   is a no-op. */
int32_t kv_compress_selected(const kv_shape_t* shape, const void* kv,
                             const uint8_t* bits_dev, const uint64_t* off_dev,
                             const int32_t* chunk_idx_dev, int32_t n_sel,
                             void* packed_out, void* stream);

/* Load primitive, data movement (Sec. 3.1 primitive 3; Sec. 3.3): unpack and
 * dequantise the n_sel listed records into tokens [dst_tok[j], dst_tok[j] +
 * chunk_tokens) of every slab of kv_out; other tokens are untouched.
 *   packed dev pool; src_off_dev dev u64 [n_sel] (byte offsets into packed);
 *   dst_tok_dev dev i32 [n_sel]; sel_bits_dev dev u8 [n_sel]; kv_out dev fp16
 *   cache.  n_sel == 0 is a no-op.  The Fault primitive is this call with
 *   n_sel == 1.
 * packed (here, in kv_swapin_layers and in kv_load_chunks) may also be PINNED HOST
 * memory that the device can address (hipHostMalloc, torch pin_memory): the kernel
 * then fetches the records over the host link itself, with no staging buffer and no
 * copy engine (measured on MI355X: the link's full rate, 56.6 GB/s).  While such a
 * launch runs its wavefronts wait on the link and hold their places on the compute
 * units; kv_swapin_pinned keeps the compute units free instead. */
int32_t kv_swapin_chunks(const kv_shape_t* shape, const void* packed,
                         const uint64_t* src_off_dev, const int32_t* dst_tok_dev,
                         const uint8_t* sel_bits_dev, int32_t n_sel,
                         void* kv_out, void* stream);

/* Layer-wise Load (Sec. 3.3, swapping-recompute pipeline: the chunks of the next layer
 * are loaded while the current layer is recomputed): kv_swapin_chunks restricted to the
 * layers [layer_begin, layer_end) of the listed records; the other layers of kv_out are
 * untouched.  A record holds its layers one after the other in every section, so a
 * layer's share is three contiguous pieces (codes, scale, mn) that the kernel addresses
 * itself.  0 <= layer_begin <= layer_end <= n_layers (else KV_EINVAL); an empty range
 * is a no-op; the full range is kv_swapin_chunks. */
int32_t kv_swapin_layers(const kv_shape_t* shape, const void* packed,
                         const uint64_t* src_off_dev, const int32_t* dst_tok_dev,
                         const uint8_t* sel_bits_dev, int32_t n_sel,
                         int32_t layer_begin, int32_t layer_end,
                         void* kv_out, void* stream);

/* The Load primitive in one call (Sec. 3.1 primitive 3; the Fault primitive with
 * n_sel == 1): kv_build_gather + kv_swapin_chunks with the gather list carried in
 * the kernel arguments (up to 64 records per launch), so no list is uploaded and
 * no device list buffers are needed; the shortest route for a few chunks.
 *   packed dev pool; off HOST u64 [n_chunks+1]; bits HOST u8 [n_chunks];
 *   chunk_idx HOST i32 [n_sel], strictly ascending (else KV_EINDEX); kv_out dev
 *   cache.  The whole list is checked before the first launch; n_sel == 0 is a
 *   no-op.  The host arrays may be reused as soon as the call returns. */
int32_t kv_load_chunks(const kv_shape_t* shape, const void* packed, const uint64_t* off,
                       const uint8_t* bits, const int32_t* chunk_idx, int32_t n_sel,
                       void* kv_out, void* stream);

/* Streaming Load from pinned host memory: the IO half of the swapping-
 * recompute pipeline (Sec. 3.3), with the dequantise kernel in the place of
 * the recompute stage.  The listed records are copied host->device in batches
 * on copy_stream into n_buffers staging slots while earlier batches are
 * dequantised on compute_stream.
 *   ld  a loader handle: it owns the HIP events that order copies and kernels (created
 *   once, by kv_loader_create, on the device that is current then) and remembers which
 *   staging slots a kernel of an earlier call may still be reading, so that calls one
 *   after the other through one loader may share their staging memory and streams
 *   (they walk the slots round robin; a call with another staging_dev, staging_bytes or
 *   n_buffers than its predecessor first waits, on copy_stream, for all of that call's kernels).
 *   One thread at a time per loader.
 *   packed_pinned pinned host pool; src_off/dst_tok/sel_bits HOST lists [n_sel]
 *   as produced by kv_build_gather (ascending chunks, hence ascending offsets);
 *   staging_dev dev scratch of staging_bytes, 256-byte aligned, split into
 *   n_buffers (2..8) equal slots (rounded down to 256 bytes), each of which
 *   must hold the largest listed record (else KV_ENOMEM);
 *   kv_out dev fp16 cache.  copy_stream and compute_stream must differ and
 *   must not be the NULL stream.  Returns after enqueuing everything;
 *   completion = both streams idle (the last kernel is on compute_stream).
 *   A context kept as one pool per layer (records of a shape with n_layers = 1,
 *   kv_out pointing at the layer's slice of the cache) is loaded layer by layer
 *   with one such call per layer: the order of the swapping-recompute pipeline
 *   (Sec. 3.3), with the copies on the DMA engines. */
typedef struct kv_loader kv_loader_t;
kv_loader_t* kv_loader_create(void);               /* NULL on failure (kv_last_error has the text) */
void         kv_loader_destroy(kv_loader_t* ld);   /* after the streams it was used on have drained */
int32_t kv_swapin_stream(kv_loader_t* ld, const kv_shape_t* shape, const void* packed_pinned,
                         const uint64_t* src_off, const int32_t* dst_tok,
                         const uint8_t* sel_bits, int32_t n_sel,
                         void* staging_dev, uint64_t staging_bytes, int32_t n_buffers,
                         void* kv_out, void* copy_stream, void* compute_stream);

/* kv_swapin_stream for a single Load, without a loader: the events are created for the call
 * and destroyed when it returns (the enqueued work keeps what it needs).  The staging slots
 * belong to the call until its last kernel has finished: a further call on the same streams
 * needs staging memory of its own, or copy_stream must first wait for compute_stream. */
int32_t kv_swapin_pinned(const kv_shape_t* shape, const void* packed_pinned,
                         const uint64_t* src_off, const int32_t* dst_tok,
                         const uint8_t* sel_bits, int32_t n_sel,
                         void* staging_dev, uint64_t staging_bytes, int32_t n_buffers,
                         void* kv_out, void* copy_stream, void* compute_stream);

/* Ahead-of-time swap-out (Sec. 3.4 i): enqueue on copy_stream, after the work
 * currently enqueued on producer_stream, a device->pinned-host copy of
 * packed_dev[begin, end) to the same offsets of packed_pinned, so that a later
 * Reclaim of these chunks moves no data. */
int32_t kv_swapout_aot(const void* packed_dev, void* packed_pinned,
                       uint64_t begin, uint64_t end,
                       void* producer_stream, void* copy_stream);

/* ------------------------------------ recompute of interleaved chunks (Sec. 3.3) */

/* The paper recovers missing chunks either from their swapped-out records or by
 * recomputing them from their tokens while other chunks are loaded (Sec. 3.3,
 * swapping-recompute pipeline).  "Making interleaved chunks recomputable" (Sec. 3.3
 * and its six-token example): the tokens of the missing chunks go through a layer with
 * their GLOBAL positions in the rotary encoding of q and k; the recomputed K/V are
 * inserted between the resident K/V of the layer; the recomputed queries attend to the
 * recovered K/V under a causal mask by global position; the result is the input of the
 * next layer for these tokens.  kv_recompute_layer does this for ONE Llama-style block
 * (the paper's example uses a Llama2-7B layer):
 *   xn = rmsnorm(x; w_norm1);  q, k, v = xn wq, xn wk, xn wv;
 *   q, k = rope(q, k; global position, pairs (i, i + head_dim/2), angle pos * rope_base^(-2i/head_dim));
 *   cache[layer][K|V][kv head][position][:] = fp16(k), fp16(v);
 *   o = softmax(q K^T / sqrt(head_dim), keys at positions <= the query's) V   per query head,
 *       query head h reading kv head h / (n_q_heads / n_kv_heads);
 *   x1 = x + o wo;  y = x1 + (silu(rmsnorm(x1; w_norm2) w_gate) * (rmsnorm(x1; w_norm2) w_up)) w_down.
 * Heads, head_dim, cache geometry and chunk size come from kv_shape_t (format 0,
 * head_dim 64 or 128).  Weights are fp16, row-major [in][out], 16-byte aligned, device. */
typedef struct {
    int32_t d_model;      /* hidden size, multiple of 8 */
    int32_t d_ff;         /* feed-forward width, multiple of 8 */
    float   rope_base;    /* e.g. 10000 */
    float   rms_eps;      /* e.g. 1e-5 */
} kv_layer_dims_t;

typedef struct {
    const void* w_norm1;  /* [d_model]                       */
    const void* wq;       /* [d_model][n_q_heads * head_dim]  */
    const void* wk;       /* [d_model][n_kv_heads * head_dim] */
    const void* wv;       /* [d_model][n_kv_heads * head_dim] */
    const void* wo;       /* [n_q_heads * head_dim][d_model]  */
    const void* w_norm2;  /* [d_model]                       */
    const void* w_gate;   /* [d_model][d_ff]                  */
    const void* w_up;     /* [d_model][d_ff]                  */
    const void* w_down;   /* [d_ff][d_model]                  */
} kv_layer_weights_t;

/* Handle of the recompute path.  The projections of up to KV_RECOMPUTE_OWN_GEMM_ROWS recomputed
 * tokens (what a plan of Eq. 4 recomputes beside a Load) run on the library's own MFMA GEMM,
 * which is the faster one there (0.26 against 0.34 ms per Llama-2-7B layer at 128 tokens, 0.33
 * against 0.35 at 256, 0.46 against 0.49 at 512, rocBLAS with its best kernels); larger ones are handed
 * to rocBLAS, which is loaded on creation if it is installed (the handle then owns that
 * library's handle, whose device workspace lives until kv_recompute_destroy).  Without
 * rocBLAS, or with KVSWITCH_OWN_GEMM=1 in the environment at creation, every size runs on the
 * library's own kernel (about half the GEMM library's rate at thousands of rows).  NULL on
 * failure (kv_last_error has the text).  One handle serves one stream at a time. */
#define KV_RECOMPUTE_OWN_GEMM_ROWS 512
typedef struct kv_recompute kv_recompute_t;
kv_recompute_t* kv_recompute_create(void);
void            kv_recompute_destroy(kv_recompute_t* rc);

/* Bytes of device workspace kv_recompute_layer needs for n_missing chunks; 0 on invalid arguments. */
uint64_t kv_recompute_workspace_bytes(const kv_shape_t* shape, const kv_layer_dims_t* dims,
                                      int32_t n_missing);

/* Optional, once per (handle, n_missing): choose the GEMM library's kernels for the five projection
 * shapes of a block over n_missing chunks by timing them on the caller's weights and workspace
 * (Sec. 3.3 i profiles the recompute delay before planning; for a few hundred tokens the
 * library's default kernels are far from the best it has).  Every listed kernel is timed back to
 * back; the standard choice and the best few are timed again with cold weights, the other
 * projections of the block running in between as in a layer; the winner is used by later
 * kv_recompute_layer calls with the same n_missing if it beats the standard choice by more than
 * 5 %.  Unlike every other device call this one SYNCHRONISES `stream`, takes of the order of a
 * second, and overwrites the workspace.  n_improved (may be NULL) receives the number of shapes
 * that got another kernel; 0 and KV_OK if the library cannot list its kernels, and where the
 * projections do not go to the GEMM library at all (few tokens, see above, or no rocBLAS): nothing is
 * then timed.  Results are the same up to the summation order inside a GEMM. */
int32_t kv_recompute_tune(kv_recompute_t* rc, const kv_shape_t* shape, const kv_layer_dims_t* dims,
                          const kv_layer_weights_t* weights, int32_t n_missing, void* workspace,
                          uint64_t workspace_bytes, void* stream, int32_t* n_improved);

/* One block over the tokens of n_missing chunks (1 <= n_missing <= n_chunks).
 *   chunk_idx_dev dev i32 [n_missing], strictly ascending chunk indices (trusted, like the
 *                 gather lists: an index outside the cache makes the kernels write outside it);
 *   x_in   dev fp16 [n_missing * chunk_tokens][d_model]: the layer inputs of these tokens,
 *          chunk by chunk in the order of chunk_idx_dev;
 *   kv     dev fp16 cache; the K and V planes of `layer` must hold every resident chunk that
 *          lies before the last recomputed token; the recomputed chunks' entries are written;
 *   x_out  dev fp16, same shape as x_in: the layer outputs (may not alias x_in);
 *   workspace dev, >= kv_recompute_workspace_bytes(), 256-byte aligned, contents scratch.
 * Enqueues on `stream` and returns; nothing is launched if a host argument is invalid. */
int32_t kv_recompute_layer(kv_recompute_t* rc, const kv_shape_t* shape, const kv_layer_dims_t* dims,
                           const kv_layer_weights_t* weights, int32_t layer,
                           const int32_t* chunk_idx_dev, int32_t n_missing, const void* x_in,
                           void* kv, void* x_out, void* workspace, uint64_t workspace_bytes,
                           void* stream);

/* -------------------------------------------- host lifecycle (Sec. 3.4 ii) */

/* LCTRU queue: concatenated sub-queues, one per bit-width, least compressed
 * first; inside a sub-queue the least recently used context first; ties by
 * (ctx, chunk) ascending.  Only memory-resident chunks are queued.  Contexts
 * locked as a working set are skipped by eviction (Sec. 3.4, working set). */
typedef struct kv_lctru kv_lctru_t;

kv_lctru_t* kv_lctru_create(void);
void        kv_lctru_destroy(kv_lctru_t* q);

/* Claim: a chunk becomes resident.  KV_EINVAL if (ctx,chunk) is already queued. */
int32_t kv_lctru_insert(kv_lctru_t* q, int32_t ctx, int32_t chunk, int32_t bits,
                        uint64_t bytes, uint64_t now);
/* On every call into a context: all its resident chunks get last_access = now. */
int32_t kv_lctru_touch_ctx(kv_lctru_t* q, int32_t ctx, uint64_t now);
int32_t kv_lctru_lock(kv_lctru_t* q, int32_t ctx);
int32_t kv_lctru_unlock(kv_lctru_t* q, int32_t ctx);
/* Reclaim: pop from the front until the popped bytes reach bytes_needed.
 * KV_ENOMEM (nothing popped) if the unlocked resident bytes are fewer than
 * bytes_needed or more than cap entries would be needed. */
int32_t kv_lctru_evict(kv_lctru_t* q, uint64_t bytes_needed, int32_t* out_ctx,
                       int32_t* out_chunk, int32_t cap, int32_t* n_out);
/* Current eviction order of all unlocked entries, front first (no change). */
int32_t kv_lctru_order(const kv_lctru_t* q, int32_t* out_ctx, int32_t* out_chunk,
                       int32_t cap, int32_t* n_out);
/* Context deleted: drop all its entries (and its lock). */
int32_t kv_lctru_remove_ctx(kv_lctru_t* q, int32_t ctx);
/* Number of queued (resident) entries and their total bytes. */
int32_t kv_lctru_size(const kv_lctru_t* q, int32_t* n_entries, uint64_t* bytes);

#ifdef __cplusplus
}
#endif
#endif /* KVSWITCH_H */
