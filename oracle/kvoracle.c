/*
 * kvoracle.c - TEST INFRASTRUCTURE ONLY.  A plain, slow, CPU implementation of
 * what the chunk-wise KV-cache context-switch path of arXiv 2403.11805 computes.
 * It exists so that tests, the smoke check and the benchmark's cpu_baseline leg
 * have an independent answer to compare the GPU library with.  Nothing in the
 * product may call it, and it shares no source with the GPU library.
 *
 * Every function takes host pointers.  fp16 is carried as uint16_t bit
 * patterns.  Scoring works in double precision on the exact fp16 inputs;
 * quantisation works in IEEE binary32 exactly as the format contract states
 * (build with -O2 -ffp-contract=off, never -ffast-math).
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py against
 * the paper's worked example, closed forms, invariants or library routines; no
 * function is "parity unpinned".
 *
 * Shapes: KV cache [L][2 (K=0,V=1)][Hkv][N][D] fp16 (or int8 for the channel-wise
 * variant); a chunk is T tokens of every (layer, K|V, kv-head) slab and has one
 * bit-width (Sec. 3.1).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t L, Hkv, Hq, D, N, T, G;
    int32_t fmt;   /* 0: fp16 cache, groups of G along head_dim (3: the same with binary16 parameters); 1: int8 cache, channel-wise;
                      2: as 1 with the parameters stored (and used) in binary16 */
} orc_shape;

/* Number of threads the parallel loops below may use from now on (timing the checker on one core). */
void orc_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int orc_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ----------------------------------------------------------------- fp16 <-> fp32 */

/* IEEE binary16 -> binary32, exact. */
float orc_half_to_float(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) & 1u;
    int32_t  e    = (h >> 10) & 0x1f;
    uint32_t m    = h & 0x3ffu;
    double v;
    if (e == 31) {
        v = m ? NAN : INFINITY;
    } else if (e == 0) {
        v = ldexp((double)m, -24);            /* subnormal: m * 2^-24 */
    } else {
        v = ldexp((double)(m | 0x400u), e - 25); /* (1024+m) * 2^(e-15-10) */
    }
    return (float)(sign ? -v : v);
}

/* IEEE binary32 -> binary16, round to nearest, ties to even. */
uint16_t orc_float_to_half(float f)
{
    uint32_t sign = signbit(f) ? 0x8000u : 0u;
    double a = fabs((double)f);
    if (isnan(f)) return (uint16_t)(sign | 0x7e00u);
    if (a >= 65520.0) return (uint16_t)(sign | 0x7c00u);   /* rounds to inf */
    if (a == 0.0) return (uint16_t)sign;
    int ex;
    (void)frexp(a, &ex);                 /* a = frac * 2^ex, frac in [0.5,1) */
    int e = ex - 1;                      /* a in [2^e, 2^(e+1)) */
    if (e < -14) e = -14;                /* subnormal range: fixed quantum 2^-24 */
    /* quantum of the target format at this exponent is 2^(e-10) */
    double scaled = ldexp(a, 10 - e);    /* exact: power-of-two scaling */
    double r = nearbyint(scaled);        /* default mode: ties to even */
    /* r in [0, 2048]; 2048 means carry into the next binade */
    uint32_t bits;
    if (e == -14 && r < 1024.0) {
        bits = (uint32_t)r;                              /* subnormal or zero */
    } else {
        if (r >= 2048.0) { r = 1024.0; e += 1; }
        bits = ((uint32_t)(e + 15) << 10) | ((uint32_t)r - 1024u);
    }
    return (uint16_t)(sign | bits);
}

/* ----------------------------------------------------------------- scoring (Sec. 3.2, Eq. 1) */

/*
 * Attention matrix of one (layer, head): A = softmax(mask(Q K^T / sqrt(D))).
 * q [R][D], k [N][D] fp16; A [R][N] doubles.  The R query rows are the last R
 * tokens of the N-token context: row r sits at position P_r = N - R + r and
 * sees columns c <= P_r (lower-triangular mask); masked entries are 0.
 */
void orc_attention(const uint16_t* q, const uint16_t* k, int R, int N, int D, double* A)
{
    const double inv_sqrt_d = 1.0 / sqrt((double)D);
    /* the fp16 inputs widened once (exactly) instead of inside the dot products */
    double* qd = (double*)malloc((size_t)R * D * sizeof(double));
    double* kd = (double*)malloc((size_t)N * D * sizeof(double));
    if (!qd || !kd) { free(qd); free(kd); for (size_t i = 0; i < (size_t)R * N; ++i) A[i] = NAN; return; }
    for (size_t i = 0; i < (size_t)R * D; ++i) qd[i] = (double)orc_half_to_float(q[i]);
    for (size_t i = 0; i < (size_t)N * D; ++i) kd[i] = (double)orc_half_to_float(k[i]);
    for (int r = 0; r < R; ++r) {
        const int last = N - R + r;            /* last visible column */
        double* row = A + (size_t)r * N;
        double mx = -INFINITY;
        for (int c = 0; c <= last; ++c) {
            double s = 0.0;
            for (int d = 0; d < D; ++d)
                s += qd[(size_t)r * D + d] * kd[(size_t)c * D + d];
            s *= inv_sqrt_d;
            row[c] = s;
            if (s > mx) mx = s;
        }
        double denom = 0.0;
        for (int c = 0; c <= last; ++c) {
            row[c] = exp(row[c] - mx);
            denom += row[c];
        }
        for (int c = 0; c <= last; ++c) row[c] /= denom;
        for (int c = last + 1; c < N; ++c) row[c] = 0.0;
    }
    free(qd);
    free(kd);
}

/*
 * Per-chunk mass of one attention matrix.  Column c is summed over the rows
 * and (norm_mode 0) divided by the number of rows that can see it,
 * v[c] = N - max(c, N - R), which is the averaging the worked example of
 * Eq. 1 uses (three visible entries, divided by three); norm_mode 1 keeps the
 * plain column sum.  chunk_mass[i] = sum of that over columns [iT, iT+T).
 */
void orc_column_density(const double* A, int R, int N, int T, int norm_mode,
                        double* chunk_mass)
{
    const int n_chunks = N / T;
    for (int i = 0; i < n_chunks; ++i) {
        double acc = 0.0;
        for (int c = i * T; c < (i + 1) * T; ++c) {
            double m = 0.0;
            for (int r = 0; r < R; ++r) m += A[(size_t)r * N + c];
            if (norm_mode == 0) {
                int first_row_pos = N - R;
                int visible = N - (c > first_row_pos ? c : first_row_pos);
                m /= (double)visible;
            }
            acc += m;
        }
        chunk_mass[i] = acc;
    }
}

/* chunk mass of one (layer l, query head h) as doubles [N/T]. */
int orc_score_head(const orc_shape* s, const uint16_t* q, int R, const uint16_t* kv,
                   int l, int h, int norm_mode, double* chunk_mass)
{
    const int g = h / (s->Hq / s->Hkv);
    const uint16_t* q_lh = q + ((size_t)l * s->Hq + h) * R * s->D;
    const uint16_t* k_lg = kv + (((size_t)l * 2 + 0) * s->Hkv + g) * (size_t)s->N * s->D;
    double* A = (double*)malloc((size_t)R * s->N * sizeof(double));
    if (!A) return -1;
    orc_attention(q_lh, k_lg, R, s->N, s->D, A);
    orc_column_density(A, R, s->N, s->T, norm_mode, chunk_mass);
    free(A);
    return 0;
}

/*
 * Eq. 1 for a whole context: chunk_mass [L][Hq][N/T] (fp32 out) and
 * density[i] = (1 / (T * L * Hq)) * sum_l sum_h chunk_mass[l][h][i].
 * Query head h reads kv head h / (Hq / Hkv).
 */
int orc_score_chunks(const orc_shape* s, const uint16_t* q, int R, const uint16_t* kv,
                     int norm_mode, float* chunk_mass, float* density)
{
    const int n_chunks = s->N / s->T;
    const int LH = s->L * s->Hq;
    double* cm = (double*)malloc((size_t)LH * n_chunks * sizeof(double));
    if (!cm) return -1;
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int lh = 0; lh < LH; ++lh) {
        if (orc_score_head(s, q, R, kv, lh / s->Hq, lh % s->Hq, norm_mode,
                           cm + (size_t)lh * n_chunks))
            fail = 1;
    }
    if (!fail) {
        for (int i = 0; i < n_chunks; ++i) {
            double acc = 0.0;
            for (int lh = 0; lh < LH; ++lh) {
                acc += cm[(size_t)lh * n_chunks + i];
                chunk_mass[(size_t)lh * n_chunks + i] = (float)cm[(size_t)lh * n_chunks + i];
            }
            density[i] = (float)(acc / ((double)s->T * s->L * s->Hq));
        }
    }
    free(cm);
    return fail ? -1 : 0;
}

/* ----------------------------------------------------------------- compress (Sec. 3.2; Sec. 4 packing) */

/*
 * Quantise one group of n values to b bits.  binary32 throughout:
 *   mn = min + 0.0f, mx = max + 0.0f (turns -0 into +0),
 *   scale = (mx - mn) / (2^b - 1),
 *   code = scale == 0 ? 0 : clamp(rintf((x - mn) / scale), 0, 2^b - 1).
 */
static void quantise_group(const uint16_t* x, int n, int b, int half_params, uint8_t* code,
                           float* scale_out, float* mn_out)
{
    float mn = orc_half_to_float(x[0]);
    float mx = mn;
    for (int k = 1; k < n; ++k) {
        float v = orc_half_to_float(x[k]);
        if (v < mn) mn = v;
        if (v > mx) mx = v;
    }
    mn = mn + 0.0f;
    mx = mx + 0.0f;
    const float levels = (float)((1 << b) - 1);
    const float range = mx - mn;
    float scale = range / levels;
    /* parameters kept in binary16 (fmt 3): the scale is rounded to binary16 BEFORE the codes are
     * computed, so that both directions use the stored value; mn is one of the inputs, exact */
    if (half_params) scale = orc_half_to_float(orc_float_to_half(scale));
    for (int k = 0; k < n; ++k) {
        float c = 0.0f;
        if (scale != 0.0f) {
            float v = orc_half_to_float(x[k]);
            float d = v - mn;
            float qv = d / scale;
            c = rintf(qv);
            if (c < 0.0f) c = 0.0f;
            if (c > levels) c = levels;
        }
        code[k] = (uint8_t)c;
    }
    *scale_out = scale;
    *mn_out = mn;
}

/*
 * Compress every chunk i at bits[i] into packed + off[i].
 * Record: codes [slab][T][D*b/8], then scale [slab][T][D/G] fp32, then mn
 * (same shape); fmt 3 keeps scale and mn in binary16.  Element d of a token row goes to byte d*b/8, bit position
 * (d mod (8/b))*b: the lowest-index element in the least-significant bits.
 * b = 16: the chunk's fp16 bytes, slab after slab, nothing else.
 */
int orc_compress_chunks(const orc_shape* s, const uint16_t* kv, const uint8_t* bits,
                        const uint64_t* off, uint8_t* packed)
{
    const int n_chunks = s->N / s->T;
    const int slabs = s->L * 2 * s->Hkv;
    const int groups = s->D / s->G;
    for (int i = 0; i < n_chunks; ++i) {
        const int b = bits[i];
        if (b != 16 && b != 8 && b != 4 && b != 2) return -3;
    }
#pragma omp parallel for collapse(2) schedule(static)
    for (int i = 0; i < n_chunks; ++i) {
        for (int sl = 0; sl < slabs; ++sl) {
            const int b = bits[i];
            uint8_t* rec = packed + off[i];
            const uint16_t* src = kv + ((size_t)sl * s->N + (size_t)i * s->T) * s->D;
            if (b == 16) {
                memcpy(rec + (size_t)sl * s->T * s->D * 2, src, (size_t)s->T * s->D * 2);
                continue;
            }
            const size_t row_bytes = (size_t)s->D * b / 8;
            const int half = s->fmt == 3;
            uint8_t* codes = rec + (size_t)sl * s->T * row_bytes;
            uint8_t* meta = rec + (size_t)slabs * s->T * row_bytes;     /* scale section, then mn section */
            float* scale = (float*)meta + (size_t)sl * s->T * groups;
            float* mn = scale + (size_t)slabs * s->T * groups;
            uint16_t* scale_h = (uint16_t*)meta + (size_t)sl * s->T * groups;
            uint16_t* mn_h = scale_h + (size_t)slabs * s->T * groups;
            uint8_t tmp[1024];
            for (int t = 0; t < s->T; ++t) {
                uint8_t* row = codes + (size_t)t * row_bytes;
                memset(row, 0, row_bytes);
                for (int j = 0; j < groups; ++j) {
                    float sc, m;
                    quantise_group(src + (size_t)t * s->D + (size_t)j * s->G, s->G, b, half, tmp, &sc, &m);
                    if (half) {
                        scale_h[t * groups + j] = orc_float_to_half(sc);
                        mn_h[t * groups + j] = orc_float_to_half(m);
                    } else {
                        scale[t * groups + j] = sc;
                        mn[t * groups + j] = m;
                    }
                    for (int k = 0; k < s->G; ++k) {
                        const int d = j * s->G + k;
                        const int per_byte = 8 / b;
                        row[d / per_byte] |= (uint8_t)(tmp[k] << ((d % per_byte) * b));
                    }
                }
            }
        }
    }
    return 0;
}

/* ----------------------------------------------------------------- int8 cache, channel-wise (Sec. 3.2 / Sec. 4) */

/*
 * The paper's own setting: the cache is held as 8-bit integers and a chunk is
 * quantised further, channel-wise.  For one slab (T tokens x D channels of one
 * (layer, K|V, kv-head)) and every channel d, over the T tokens:
 *   mn = min x + 0.0f, mx = max x + 0.0f, scale = (mx - mn) / (2^b - 1),
 *   code = scale == 0 ? 0 : clamp(rintf((x - mn) / scale), 0, 2^b - 1)   (binary32)
 * b in {4, 2, 1}; b = 8 copies the int8 bytes.  Record: codes [slab][T][D*b/8]
 * (lowest-index element in the least-significant bits), scale [slab][D], mn [slab][D].
 * fmt 2 keeps the parameters in binary16: the scale is rounded to binary16 (nearest even)
 * BEFORE the codes are computed, so that quantisation and reconstruction use the same
 * value; mn is an integer in [-128, 127] and needs no rounding.
 */
int orc_compress_chunks_i8(const orc_shape* s, const int8_t* kv, const uint8_t* bits,
                           const uint64_t* off, uint8_t* packed)
{
    const int n_chunks = s->N / s->T;
    const int slabs = s->L * 2 * s->Hkv;
    for (int i = 0; i < n_chunks; ++i) {
        const int b = bits[i];
        if (b != 8 && b != 4 && b != 2 && b != 1) return -3;
    }
#pragma omp parallel for collapse(2) schedule(static)
    for (int i = 0; i < n_chunks; ++i) {
        for (int sl = 0; sl < slabs; ++sl) {
            const int b = bits[i];
            uint8_t* rec = packed + off[i];
            const int8_t* src = kv + ((size_t)sl * s->N + (size_t)i * s->T) * s->D;
            if (b == 8) {
                memcpy(rec + (size_t)sl * s->T * s->D, src, (size_t)s->T * s->D);
                continue;
            }
            const size_t row_bytes = (size_t)s->D * b / 8;
            const int per_byte = 8 / b;
            const float levels = (float)((1 << b) - 1);
            uint8_t* codes = rec + (size_t)sl * s->T * row_bytes;
            const int half = s->fmt == 2;
            uint8_t* meta = rec + (size_t)slabs * s->T * row_bytes;
            float* scale = (float*)meta + (size_t)sl * s->D;
            float* mn_out = scale + (size_t)slabs * s->D;
            uint16_t* scale_h = (uint16_t*)meta + (size_t)sl * s->D;
            uint16_t* mn_h = scale_h + (size_t)slabs * s->D;
            memset(codes, 0, (size_t)s->T * row_bytes);
            for (int d = 0; d < s->D; ++d) {
                float mn = (float)src[d], mx = mn;
                for (int t = 1; t < s->T; ++t) {
                    const float v = (float)src[(size_t)t * s->D + d];
                    if (v < mn) mn = v;
                    if (v > mx) mx = v;
                }
                mn = mn + 0.0f;
                mx = mx + 0.0f;
                const float range = mx - mn;
                float sc = range / levels;
                if (half) {
                    scale_h[d] = orc_float_to_half(sc);
                    sc = orc_half_to_float(scale_h[d]);
                    mn_h[d] = orc_float_to_half(mn);
                } else {
                    scale[d] = sc;
                    mn_out[d] = mn;
                }
                for (int t = 0; t < s->T; ++t) {
                    float c = 0.0f;
                    if (sc != 0.0f) {
                        const float dv = (float)src[(size_t)t * s->D + d] - mn;
                        const float qv = dv / sc;
                        c = rintf(qv);
                        if (c < 0.0f) c = 0.0f;
                        if (c > levels) c = levels;
                    }
                    codes[(size_t)t * row_bytes + d / per_byte] |= (uint8_t)((uint8_t)c << ((d % per_byte) * b));
                }
            }
        }
    }
    return 0;
}

/* Load for the int8 format: x = int8(clamp(rintf((float)code * scale + mn), -128, 127)),
 * product and sum rounded separately; b = 8 copies the bytes. */
int orc_swapin_chunks_i8(const orc_shape* s, const uint8_t* packed, const uint64_t* src_off,
                         const int32_t* dst_tok, const uint8_t* sel_bits, int n_sel, int8_t* kv_out)
{
    const int slabs = s->L * 2 * s->Hkv;
    for (int j = 0; j < n_sel; ++j) {
        const int b = sel_bits[j];
        if (b != 8 && b != 4 && b != 2 && b != 1) return -3;
        if (dst_tok[j] < 0 || dst_tok[j] + s->T > s->N) return -4;
    }
#pragma omp parallel for collapse(2) schedule(static)
    for (int j = 0; j < n_sel; ++j) {
        for (int sl = 0; sl < slabs; ++sl) {
            const int b = sel_bits[j];
            const uint8_t* rec = packed + src_off[j];
            int8_t* dst = kv_out + ((size_t)sl * s->N + (size_t)dst_tok[j]) * s->D;
            if (b == 8) {
                memcpy(dst, rec + (size_t)sl * s->T * s->D, (size_t)s->T * s->D);
                continue;
            }
            const size_t row_bytes = (size_t)s->D * b / 8;
            const int per_byte = 8 / b;
            const unsigned mask = (1u << b) - 1u;
            const uint8_t* codes = rec + (size_t)sl * s->T * row_bytes;
            const int half = s->fmt == 2;
            const uint8_t* meta = rec + (size_t)slabs * s->T * row_bytes;
            const float* scale = (const float*)meta + (size_t)sl * s->D;
            const float* mn = scale + (size_t)slabs * s->D;
            const uint16_t* scale_h = (const uint16_t*)meta + (size_t)sl * s->D;
            const uint16_t* mn_h = scale_h + (size_t)slabs * s->D;
            for (int t = 0; t < s->T; ++t) {
                for (int d = 0; d < s->D; ++d) {
                    const unsigned code = (codes[(size_t)t * row_bytes + d / per_byte] >> ((d % per_byte) * b)) & mask;
                    const float sc = half ? orc_half_to_float(scale_h[d]) : scale[d];
                    const float m = half ? orc_half_to_float(mn_h[d]) : mn[d];
                    const float prod = (float)code * sc;
                    float v = rintf(prod + m);
                    if (v < -128.0f) v = -128.0f;
                    if (v > 127.0f) v = 127.0f;
                    dst[(size_t)t * s->D + d] = (int8_t)v;
                }
            }
        }
    }
    return 0;
}

/* ----------------------------------------------------------------- swap-in (Load, Sec. 3.1 / 3.3) */

/*
 * For each listed record j (at packed + src_off[j], width sel_bits[j]) write
 * tokens [dst_tok[j], dst_tok[j]+T) of every slab of kv_out:
 *   x = fp16_rne( (float)code * scale + mn ), product and sum rounded separately.
 * b = 16 copies the bytes.  Other tokens of kv_out are left alone.
 */
int orc_swapin_chunks(const orc_shape* s, const uint8_t* packed, const uint64_t* src_off,
                      const int32_t* dst_tok, const uint8_t* sel_bits, int n_sel,
                      uint16_t* kv_out)
{
    const int slabs = s->L * 2 * s->Hkv;
    const int groups = s->D / s->G;
    for (int j = 0; j < n_sel; ++j) {
        const int b = sel_bits[j];
        if (b != 16 && b != 8 && b != 4 && b != 2) return -3;
        if (dst_tok[j] < 0 || dst_tok[j] + s->T > s->N) return -4;
    }
#pragma omp parallel for collapse(2) schedule(static)
    for (int j = 0; j < n_sel; ++j) {
        for (int sl = 0; sl < slabs; ++sl) {
            const int b = sel_bits[j];
            const uint8_t* rec = packed + src_off[j];
            uint16_t* dst = kv_out + ((size_t)sl * s->N + (size_t)dst_tok[j]) * s->D;
            if (b == 16) {
                memcpy(dst, rec + (size_t)sl * s->T * s->D * 2, (size_t)s->T * s->D * 2);
                continue;
            }
            const size_t row_bytes = (size_t)s->D * b / 8;
            const uint8_t* codes = rec + (size_t)sl * s->T * row_bytes;
            const int half = s->fmt == 3;
            const uint8_t* meta = rec + (size_t)slabs * s->T * row_bytes;
            const float* scale = (const float*)meta + (size_t)sl * s->T * groups;
            const float* mn = scale + (size_t)slabs * s->T * groups;
            const uint16_t* scale_h = (const uint16_t*)meta + (size_t)sl * s->T * groups;
            const uint16_t* mn_h = scale_h + (size_t)slabs * s->T * groups;
            const int per_byte = 8 / b;
            const unsigned mask = (1u << b) - 1u;
            for (int t = 0; t < s->T; ++t) {
                const uint8_t* row = codes + (size_t)t * row_bytes;
                for (int d = 0; d < s->D; ++d) {
                    const unsigned code = (row[d / per_byte] >> ((d % per_byte) * b)) & mask;
                    const int gidx = t * groups + d / s->G;
                    const float sc = half ? orc_half_to_float(scale_h[gidx]) : scale[gidx];
                    const float m = half ? orc_half_to_float(mn_h[gidx]) : mn[gidx];
                    const float prod = (float)code * sc;
                    const float val = prod + m;
                    dst[(size_t)t * s->D + d] = orc_float_to_half(val);
                }
            }
        }
    }
    return 0;
}
